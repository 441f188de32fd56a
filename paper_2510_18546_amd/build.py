"""Build libefficientnav.so (host planner + HIP kernels) for gfx950 with hipcc.

The library is built in-tree, next to this file, so that it travels with the
source tree; nothing is installed.
"""
from __future__ import annotations

import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
LIB_PATH = os.path.join(_HERE, "libefficientnav.so")
_CSRC = os.path.join(_HERE, "csrc")
SOURCES = [os.path.join(_CSRC, f) for f in
           ("en_host.cpp", "en_tier.cpp", "en_gather.hip", "en_attn_prefill.hip", "en_attn_decode.hip",
            "en_merge_mass.hip", "en_static_scratch.hip", "en_ceilings.hip")]
HEADERS = [os.path.join(_CSRC, "en_internal.h"), os.path.join(_CSRC, "en_device.h"),
           os.path.join(_ROOT, "include", "efficientnav.h")]
OBJ_DIR = os.path.join(_HERE, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # no NaN is ever produced (masked scores are -inf and guarded): lets the
    # compiler drop the canonicalising copies around every max
    "-fno-honor-nans",
    # packed fp32 arithmetic stays off for every device function
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def _run(cmd) -> str:
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    return err


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library: every source to an object of its own, side by side, then one link.
    With force=False an up-to-date library is kept."""
    if not force and not is_stale():
        return LIB_PATH
    os.makedirs(OBJ_DIR, exist_ok=True)
    inc = ["-I", os.path.join(_ROOT, "include"), "-I", _CSRC]
    objs = [os.path.join(OBJ_DIR, os.path.basename(src) + ".o") for src in SOURCES]
    jobs = [[hipcc()] + HIPCC_FLAGS + inc + ["-c", src, "-o", obj] for src, obj in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 1)) as pool:
        errs = list(pool.map(_run, jobs))
    errs.append(_run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB_PATH]))
    if verbose and any(e.strip() for e in errs):
        print("\n".join(e for e in errs if e.strip()))
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
