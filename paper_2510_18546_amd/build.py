"""Build libefficientnav.so (host planner + HIP kernels) for gfx950 with hipcc.

The library is built in-tree, next to this file, so that it travels with the
source tree; nothing is installed.
"""
from __future__ import annotations

import os
import shutil
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
LIB_PATH = os.path.join(_HERE, "libefficientnav.so")
SOURCES = [os.path.join(_HERE, "csrc", "en_host.cpp"), os.path.join(_HERE, "csrc", "en_tier.cpp"),
           os.path.join(_HERE, "csrc", "en_kernels.hip")]
HEADERS = [os.path.join(_HERE, "csrc", "en_internal.h"), os.path.join(_ROOT, "include", "efficientnav.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
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


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library. With force=False an up-to-date library is kept."""
    if not force and not is_stale():
        return LIB_PATH
    cmd = [hipcc()] + HIPCC_FLAGS + ["-I", os.path.join(_ROOT, "include"),
                                     "-I", os.path.join(_HERE, "csrc")] + SOURCES + ["-o", LIB_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
