"""Python face of the CPU oracle (float64, explicit gather + RoPE).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
cpu_baseline leg use it; the product path never does. The attention part is
``en_oracle.c`` (plain loops, see its header for the passages it follows);
the retrieval knapsack of Section 3.4, Eq. (1) is written out here.

Nothing in this file imports the GPU package.
"""
from __future__ import annotations

import ctypes as C
import itertools
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "en_oracle.c")
_LIB = os.path.join(_HERE, "libenoracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile en_oracle.c with gcc (OpenMP over output rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.en_oracle_threads.restype = C.c_int
        _lib.en_oracle_plan.restype = C.c_int
        _lib.en_oracle_gather_rope.restype = C.c_int
        _lib.en_oracle_attention.restype = C.c_int
        _lib.en_oracle_rope.restype = None
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def threads() -> int:
    return int(_load().en_oracle_threads())


def plan(lens: np.ndarray, sel: Sequence[int]) -> np.ndarray:
    """offset[S+1]: exclusive prefix sum of the selected groups' lengths."""
    lens = _i32(lens)
    sel = _i32(sel)
    off = np.zeros(len(sel) + 1, dtype=np.int32)
    rc = _load().en_oracle_plan(C.c_int(len(lens)), _p(lens, C.c_int32), C.c_int(len(sel)),
                                _p(sel, C.c_int32), _p(off, C.c_int32))
    if rc != 0:
        raise ValueError("group id out of range")
    return off


def rope(x: np.ndarray, pos: int, base: float) -> np.ndarray:
    y = np.array(x, dtype=np.float64).copy()
    _load().en_oracle_rope(_p(y, C.c_double), C.c_int(y.shape[-1]), C.c_int64(int(pos)),
                           C.c_double(base))
    return y


def gather_rope(k_pool, v_pool, lens, sel, k_new, v_new, rope_base) -> Tuple[np.ndarray, np.ndarray]:
    """One agent: (Kc, Vc), each [Hkv, L_c + Nq, D] float64."""
    k_pool, v_pool, k_new, v_new = map(_f32, (k_pool, v_pool, k_new, v_new))
    lens, sel = _i32(lens), _i32(sel)
    G, Hkv, Cap, D = k_pool.shape
    Nq = k_new.shape[0]
    L = int(lens[sel].sum()) + Nq if len(sel) else Nq
    kc = np.zeros((Hkv, L, D), dtype=np.float64)
    vc = np.zeros((Hkv, L, D), dtype=np.float64)
    rc = _load().en_oracle_gather_rope(
        C.c_int(G), C.c_int(Hkv), C.c_int(Cap), C.c_int(D), _p(k_pool, C.c_float),
        _p(v_pool, C.c_float), _p(lens, C.c_int32), C.c_int(len(sel)), _p(sel, C.c_int32),
        C.c_int(Nq), _p(k_new, C.c_float), _p(v_new, C.c_float), C.c_double(rope_base),
        _p(kc, C.c_double), _p(vc, C.c_double))
    if rc != 0:
        raise ValueError(f"oracle gather failed ({rc})")
    return kc, vc


def attention(k_pool, v_pool, lens, sel, sel_ptr, q, k_new, v_new, rope_base,
              rows: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Attention output and per-segment mass.

    Without ``rows``: out [B,Nq,Hq,D], mass [B,Nq,Hq,Smax+1] (float64).
    With ``rows`` (int32 [n,3] of (b, i, hq)): out [n,D], mass [n,Smax+1].
    """
    k_pool, v_pool, q, k_new, v_new = map(_f32, (k_pool, v_pool, q, k_new, v_new))
    lens, sel, sel_ptr = _i32(lens), _i32(sel), _i32(sel_ptr)
    G, Hkv, Cap, D = k_pool.shape
    B, Nq, Hq, _ = q.shape
    Smax = int(np.max(np.diff(sel_ptr))) if B > 0 else 0
    if rows is None:
        n = B * Nq * Hq
        rows_p, n_rows = None, 0
    else:
        rows = _i32(rows).reshape(-1, 3)
        n, n_rows = rows.shape[0], rows.shape[0]
        rows_p = _p(rows, C.c_int32)
    out = np.zeros((n, D), dtype=np.float64)
    mass = np.zeros((n, Smax + 1), dtype=np.float64)
    rc = _load().en_oracle_attention(
        C.c_int(B), C.c_int(Hq), C.c_int(Hkv), C.c_int(D), C.c_int(G), C.c_int(Cap),
        _p(k_pool, C.c_float), _p(v_pool, C.c_float), _p(lens, C.c_int32),
        _p(sel, C.c_int32), _p(sel_ptr, C.c_int32), C.c_int(Nq), _p(q, C.c_float),
        _p(k_new, C.c_float), _p(v_new, C.c_float), C.c_double(rope_base), C.c_int(Smax),
        C.c_int(n_rows), rows_p, _p(out, C.c_double), _p(mass, C.c_double))
    if rc != 0:
        raise ValueError(f"oracle attention failed ({rc})")
    if rows is None:
        return out.reshape(B, Nq, Hq, D), mass.reshape(B, Nq, Hq, Smax + 1)
    return out, mass


def append(k_pool, v_pool, lens, group: int, k_rows, v_rows):
    """Section 3.2, memory caching: the KV of objects that join a group is saved
    at the end of that group's cache, the rows already there stay untouched.
    k_rows, v_rows: [n, Hkv, D] (keys unrotated). Returns new (k_pool, v_pool,
    lens); the inputs are not modified."""
    k_pool, v_pool, lens = np.array(k_pool, copy=True), np.array(v_pool, copy=True), np.array(lens, copy=True)
    n = int(k_rows.shape[0])
    first = int(lens[group])
    if not 0 <= group < k_pool.shape[0]:
        raise ValueError("group id out of range")
    if first + n > k_pool.shape[2]:
        raise ValueError("capacity exceeded")
    for t in range(n):
        for h in range(k_pool.shape[1]):
            k_pool[group, h, first + t, :] = k_rows[t, h, :]
            v_pool[group, h, first + t, :] = v_rows[t, h, :]
    lens[group] = first + n
    return k_pool, v_pool, lens


def quantize_rows(x) -> Tuple[np.ndarray, np.ndarray]:
    """KV rows as 8-bit codes with one scale per (token, head) row: an option beside the paper's
    method, which names quantisation as compatible with it (Section 2). x: [..., D].
    scale = max|x| / 127, code = x / scale rounded to the nearest integer, ties to even, in
    [-127, 127]; a row of zeros has scale 0 and codes 0. The divisions and the rounding are taken
    in float32: that is the precision in which the library decides the codes."""
    x = np.asarray(x, dtype=np.float32)
    amax = np.max(np.abs(x), axis=-1).astype(np.float32)
    scale = (amax / np.float32(127.0)).astype(np.float32)
    safe = np.where(scale > 0, scale, np.float32(1.0)).astype(np.float32)
    q = np.rint((x / safe[..., None]).astype(np.float32))
    q = np.clip(q, -127, 127).astype(np.int8)
    q[scale == 0] = 0
    return q, scale


def dequantize_rows(codes, scale) -> np.ndarray:
    """code * scale in float32, what the gather computes before it rotates and rounds to bf16."""
    return (np.asarray(codes).astype(np.float32) * np.asarray(scale, dtype=np.float32)[..., None]).astype(np.float32)


def cluster_scores(mass: np.ndarray, seg_lens: Sequence[int], spans: Sequence[int], per_key: bool) -> np.ndarray:
    """Section 3.3: attention between a newly detected object and an existing
    group. mass: [N_q, Hq, S+1] of ONE agent; an object o is the new tokens
    spans[o] .. spans[o+1]-1. Returns [n_obj, S+1]: the mean over the object's
    tokens and over the heads of the mass on each bucket; with per_key each
    cached bucket is further divided by its number of keys (mean attention
    weight per query-key pair)."""
    mass = np.asarray(mass, dtype=np.float64)
    S = len(seg_lens)
    out = np.zeros((len(spans) - 1, mass.shape[2]))
    for o in range(len(spans) - 1):
        lo, hi = int(spans[o]), int(spans[o + 1])
        for s in range(mass.shape[2]):
            tot = 0.0
            for i in range(lo, hi):
                for h in range(mass.shape[1]):
                    tot += mass[i, h, s]
            tot /= (hi - lo) * mass.shape[1]
            if per_key and s < S and seg_lens[s] > 0:
                tot /= seg_lens[s]
            out[o, s] = tot
    return out


def cluster_assign(scores: np.ndarray, seg_lens: Sequence[int], threshold: float) -> np.ndarray:
    """The decision of Section 3.3: the cached segment with the largest score
    (the lowest index among equals; empty segments and the new tokens' bucket
    never win) if that score reaches the threshold, else -1: a new group."""
    S = len(seg_lens)
    out = np.full(scores.shape[0], -1, dtype=np.int32)
    for o in range(scores.shape[0]):
        best, best_s = -np.inf, -1
        for s in range(S):
            if seg_lens[s] > 0 and scores[o, s] > best:
                best, best_s = scores[o, s], s
        if best_s >= 0 and best >= threshold:
            out[o] = best_s
    return out


def reduce_mass(mass: np.ndarray) -> np.ndarray:
    """[B,Nq,Hq,S+1] -> [B,S+1]: mass summed over query tokens and heads
    (Section 3.3's attention between new tokens and a group; dividing by
    Nq*Hq gives the average)."""
    return mass.sum(axis=(1, 2))


# ---------------------------------------------------------------------------
# Retrieval knapsack, Section 3.4, Eq. (1):
#   maximise sum (P_i - threshold) x_i   s.t.  sum M_i x_i <= M,  x_i in {0,1}.
# Memory is counted in tokens (KV bytes are proportional to tokens for a fixed
# model). The objective is evaluated in fixed point so that ties are exact:
#   value_i = round_half_even((double(P_i) - double(threshold)) * 2^32).
# Among optimal sets the one with fewest tokens wins, then the one whose sorted
# id list is lexicographically smallest. Groups with value <= 0 are never taken.
# ---------------------------------------------------------------------------

def knapsack_values(p: np.ndarray, threshold: float) -> np.ndarray:
    d = np.asarray(p, dtype=np.float32).astype(np.float64) - np.float64(np.float32(threshold))
    return np.rint(d * 4294967296.0).astype(np.int64)


def knapsack_bruteforce(p, lens, threshold, budget) -> list:
    """Exhaustive search over all subsets (n <= 20)."""
    v = knapsack_values(p, threshold)
    lens = np.asarray(lens, dtype=np.int64)
    n = len(v)
    assert n <= 20
    best_key, best_set = None, []
    for mask in range(1 << n):
        ids = [i for i in range(n) if mask >> i & 1]
        if any(v[i] <= 0 for i in ids):
            continue
        w = int(sum(lens[i] for i in ids))
        if w > budget:
            continue
        val = int(sum(int(v[i]) for i in ids))
        key = (-val, w, ids)
        if best_key is None or key < best_key:
            best_key, best_set = key, ids
    return best_set


def knapsack(p, lens, threshold, budget) -> list:
    """Exact solution: brute force for small n, else dynamic programming."""
    if len(p) <= 16:
        return knapsack_bruteforce(p, lens, threshold, budget)
    return knapsack_dp(p, lens, threshold, budget)


def knapsack_dp(p, lens, threshold, budget) -> list:
    """Dynamic programming over token capacity with the same tie rules as the
    exhaustive search (pinned against it for n <= 16)."""
    v = knapsack_values(p, threshold)
    lens = np.asarray(lens, dtype=np.int64)
    n = len(v)
    cand = [i for i in range(n) if v[i] > 0]
    W = int(min(max(int(budget), 0), int(lens[cand].sum()) if cand else 0))
    # best[i][w] = (value, -tokens) using candidates i.. with capacity w
    m = len(cand)
    val = np.zeros((m + 1, W + 1), dtype=np.int64)
    tok = np.zeros((m + 1, W + 1), dtype=np.int64)
    for a in range(m - 1, -1, -1):
        i = cand[a]
        wi, vi = int(lens[i]), int(v[i])
        val[a] = val[a + 1]
        tok[a] = tok[a + 1]
        if wi <= W:
            tv = val[a + 1, :W + 1 - wi] + vi
            tt = tok[a + 1, :W + 1 - wi] + wi
            cur_v = val[a, wi:]
            cur_t = tok[a, wi:]
            better = (tv > cur_v) | ((tv == cur_v) & (tt <= cur_t))
            val[a, wi:] = np.where(better, tv, cur_v)
            tok[a, wi:] = np.where(better, tt, cur_t)
    out, w = [], W
    for a in range(m):
        i = cand[a]
        wi, vi = int(lens[i]), int(v[i])
        if wi <= w and val[a + 1, w - wi] + vi == val[a, w] and tok[a + 1, w - wi] + wi == tok[a, w]:
            out.append(i)
            w -= wi
    return out
