"""ctypes binding over the C ABI of libefficientnav.so (include/efficientnav.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels. torch supplies device memory and the stream; there is no fallback
of any kind: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os
import sys
import weakref
from typing import Optional, Sequence, Tuple

import numpy as np

from . import build as _build

EN_F32, EN_BF16, EN_I8 = 0, 1, 2
STATUS = {0: "EN_OK", 1: "EN_ERR_INVALID_ARG", 2: "EN_ERR_OUT_OF_RANGE", 3: "EN_ERR_DUPLICATE",
          4: "EN_ERR_CAPACITY", 5: "EN_ERR_UNSUPPORTED", 6: "EN_ERR_DEVICE"}

EXPORTS = [
    "kv_pool_create", "kv_pool_set_scales", "kv_pool_set_len", "kv_pool_append", "kv_pool_destroy", "segment_select",
    "segment_select_scored", "en_plan_get_info", "en_plan_query", "en_plan_set_splits",
    "en_plan_values_from_pool",
    "en_plan_destroy", "en_context_bytes", "gather_rope", "gather_rope_queries", "en_workspace_bytes",
    "segmented_prefill_attention", "segmented_prefill_attention_prepared", "segment_attention_mass",
    "segment_cluster_assign",
    "segment_cluster_assign_rows",
    "en_decode_workspace_bytes", "segmented_decode_step", "segmented_decode_step_static", "en_timing_enable",
    "en_timing_collect", "en_last_error", "en_ceiling_mfma_bf16", "en_ceiling_read_stream",
    "kv_tier_slot_bytes", "kv_tier_create", "kv_tier_pool", "kv_tier_put", "kv_tier_append",
    "kv_tier_select_scored",
    "kv_tier_fetch", "kv_tier_fence", "kv_tier_prefetch", "kv_tier_get_stats", "kv_tier_residency",
    "kv_tier_destroy",
]


class EnError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"{STATUS.get(code, code)}: {text}")
        self.code = code


class PoolDesc(C.Structure):
    _fields_ = [("n_groups", C.c_int32), ("capacity", C.c_int32), ("n_kv_heads", C.c_int32),
                ("n_q_heads", C.c_int32), ("head_dim", C.c_int32), ("dtype", C.c_int32),
                ("max_ctx", C.c_int32), ("reserved", C.c_int32), ("rope_base", C.c_double)]


class PlanInfo(C.Structure):
    _fields_ = [("n_agents", C.c_int32), ("n_new", C.c_int32), ("max_segments", C.c_int32),
                ("ctx_stride", C.c_int32), ("max_ctx_len", C.c_int32), ("n_splits", C.c_int32),
                ("total_pairs", C.c_int64), ("total_cached", C.c_int64)]


class TierStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("fetches", "requested", "hits", "prefetched", "misses", "loads",
                                         "bytes_loaded", "evictions")]


_lib = None


def load(path: Optional[str] = None) -> C.CDLL:
    """Load the built library; build it first only if nothing has been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = path or _build.LIB_PATH
    if not os.path.exists(path):
        _build.build()
    lib = C.CDLL(path)
    vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
    lib.kv_pool_create.argtypes = [C.POINTER(PoolDesc), vp, vp, i32p, C.POINTER(vp)]
    lib.kv_pool_set_scales.argtypes = [vp, vp, vp]
    lib.kv_pool_set_len.argtypes = [vp, C.c_int32, C.c_int32]
    lib.kv_pool_append.argtypes = [vp, C.c_int32, vp, vp, C.c_int32, vp]
    lib.kv_pool_destroy.argtypes = [vp]
    lib.segment_select.argtypes = [vp, C.c_int32, i32p, i32p, C.c_int32, C.POINTER(vp)]
    lib.segment_select_scored.argtypes = [vp, C.POINTER(C.c_float), C.c_float, C.c_int64, C.c_int32,
                                          i32p, i32p, C.POINTER(vp)]
    lib.en_plan_get_info.argtypes = [vp, C.POINTER(PlanInfo)]
    lib.en_plan_query.argtypes = [vp, C.c_int32, i32p, i32p]
    lib.en_plan_set_splits.argtypes = [vp, C.c_int32]
    lib.en_plan_values_from_pool.argtypes = [vp, C.c_int32]
    lib.en_plan_destroy.argtypes = [vp]
    lib.en_context_bytes.argtypes = [vp, vp]
    lib.en_context_bytes.restype = C.c_size_t
    lib.en_workspace_bytes.argtypes = [vp, vp]
    lib.en_workspace_bytes.restype = C.c_size_t
    lib.gather_rope.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.segmented_prefill_attention.argtypes = [vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.gather_rope_queries.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.segmented_prefill_attention_prepared.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.segment_attention_mass.argtypes = [vp, vp, vp, C.c_int32, vp, vp]
    lib.segment_cluster_assign.argtypes = [vp, vp, vp, C.c_int32, i32p, C.c_int32, C.c_int32, C.c_float,
                                           C.c_float, vp, vp, vp]
    lib.segment_cluster_assign_rows.argtypes = [vp, vp, C.c_int32, C.c_int32, vp, C.c_int32, i32p, C.c_int32,
                                                C.c_int32, C.c_float, C.c_float, vp, vp, vp]
    lib.en_decode_workspace_bytes.argtypes = [vp, vp, C.c_int32]
    lib.en_decode_workspace_bytes.restype = C.c_size_t
    lib.segmented_decode_step.argtypes = [vp, vp, C.c_int32, C.c_int32, vp, vp, vp, vp, vp, vp, vp, vp,
                                          C.c_size_t, vp]
    lib.segmented_decode_step_static.argtypes = [vp, vp, C.c_int32, C.c_int32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.en_timing_enable.argtypes = [vp, C.c_int32]
    lib.en_timing_collect.argtypes = [vp, C.POINTER(C.c_float), C.c_int32, i32p]
    lib.en_last_error.restype = C.c_char_p
    lib.en_ceiling_mfma_bf16.argtypes = [vp, C.c_size_t, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_double), vp]
    lib.en_ceiling_read_stream.argtypes = [vp, C.c_size_t, vp, C.c_size_t, C.c_int32, vp]
    lib.kv_tier_slot_bytes.argtypes = [C.POINTER(PoolDesc)]
    lib.kv_tier_slot_bytes.restype = C.c_int64
    lib.kv_tier_create.argtypes = [C.POINTER(PoolDesc), C.c_int32, vp, vp, C.POINTER(vp)]
    lib.kv_tier_pool.argtypes = [vp]
    lib.kv_tier_pool.restype = vp
    lib.kv_tier_put.argtypes = [vp, C.c_int32, vp, vp, C.c_int32]
    lib.kv_tier_append.argtypes = [vp, C.c_int32, vp, vp, C.c_int32, vp]
    lib.kv_tier_select_scored.argtypes = [vp, C.POINTER(C.c_float), C.c_float, C.c_int64, i32p, i32p]
    lib.kv_tier_fetch.argtypes = [vp, i32p, C.c_int32, i32p, vp]
    lib.kv_tier_fence.argtypes = [vp, vp]
    lib.kv_tier_prefetch.argtypes = [vp, i32p, C.c_int32, i32p]
    lib.kv_tier_get_stats.argtypes = [vp, C.POINTER(TierStats)]
    lib.kv_tier_residency.argtypes = [vp, i32p]
    lib.kv_tier_destroy.argtypes = [vp]
    for name in EXPORTS:
        if name not in ("en_context_bytes", "en_workspace_bytes", "en_decode_workspace_bytes", "en_last_error",
                        "kv_tier_slot_bytes", "kv_tier_pool"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise EnError(rc, load().en_last_error().decode())


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ip(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _stream(stream) -> C.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    return C.c_void_p(int(stream))


class Pool:
    """Handle of a KV pool. Keeps the K/V tensors alive."""

    def __init__(self, handle, k, v, desc: PoolDesc, owned: bool = True):
        self.handle, self.k, self.v, self.desc = handle, k, v, desc
        self._owned = owned                  # False: the handle belongs to a tier, which destroys it
        self._plans = weakref.WeakSet()      # a pool must outlive its plans: it closes them first

    def close(self):
        if self.handle:
            for p in list(self._plans):
                p.close()
            if self._owned:
                load().kv_pool_destroy(self.handle)
            self.handle = None

    def __del__(self):
        # at interpreter shutdown the HIP runtime may already be gone: the process frees everything
        if sys is None or sys.is_finalizing():
            return
        try:
            self.close()
        except Exception:
            pass


class Plan:
    def __init__(self, handle, pool: Pool):
        self.handle, self.pool = handle, pool
        pool._plans.add(self)

    @property
    def info(self) -> PlanInfo:
        inf = PlanInfo()
        _check(load().en_plan_get_info(self.handle, C.byref(inf)))
        return inf

    def offsets(self, agent: int) -> np.ndarray:
        n = C.c_int32()
        _check(load().en_plan_query(self.handle, agent, None, C.byref(n)))
        off = np.zeros(n.value + 1, dtype=np.int32)
        _check(load().en_plan_query(self.handle, agent, _ip(off), None))
        return off

    def set_splits(self, n: int):
        _check(load().en_plan_set_splits(self.handle, int(n)))

    def values_from_pool(self, on: bool):
        _check(load().en_plan_values_from_pool(self.handle, 1 if on else 0))

    def close(self):
        if self.handle:
            load().en_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        # at interpreter shutdown the HIP runtime may already be gone: the process frees everything
        if sys is None or sys.is_finalizing():
            return
        try:
            self.close()
        except Exception:
            pass


def kv_pool_create(k_pool, v_pool, lens, n_q_heads: int, rope_base: float, max_ctx: int,
                   dtype: Optional[int] = None, k_ptr: Optional[int] = None,
                   v_ptr: Optional[int] = None, shape: Optional[Sequence[int]] = None) -> Pool:
    """k_pool, v_pool: torch tensors [G,Hkv,C,D] on the GPU (float32 or bfloat16).
    For host-only planner use, pass k_pool=v_pool=None with ``shape``, ``dtype``
    and opaque non-null ``k_ptr``/``v_ptr`` values that are never dereferenced."""
    if k_pool is not None:
        import torch
        assert k_pool.is_contiguous() and v_pool.is_contiguous() and k_pool.shape == v_pool.shape
        shape = tuple(k_pool.shape)
        dtype = EN_BF16 if k_pool.dtype == torch.bfloat16 else EN_I8 if k_pool.dtype == torch.int8 else EN_F32
        k_ptr, v_ptr = k_pool.data_ptr(), v_pool.data_ptr()
    G, Hkv, Cap, D = shape
    desc = PoolDesc(G, Cap, Hkv, n_q_heads, D, dtype, max_ctx, 0, rope_base)
    lens = _i32(lens)
    h = C.c_void_p()
    _check(load().kv_pool_create(C.byref(desc), C.c_void_p(k_ptr), C.c_void_p(v_ptr), _ip(lens),
                                 C.byref(h)))
    return Pool(h, k_pool, v_pool, desc)


def kv_pool_set_scales(pool: Pool, k_scale, v_scale):
    """k_scale, v_scale: float32 tensors [G, Hkv, C] on the GPU (kept alive by the pool), or integers as
    opaque pointers for host-only tests."""
    if hasattr(k_scale, "data_ptr"):
        assert k_scale.is_contiguous() and v_scale.is_contiguous()
        pool.k_scale, pool.v_scale = k_scale, v_scale
        kp, vp_ = k_scale.data_ptr(), v_scale.data_ptr()
    else:
        kp, vp_ = k_scale, v_scale
    _check(load().kv_pool_set_scales(pool.handle, C.c_void_p(kp), C.c_void_p(vp_)))


def kv_pool_set_len(pool: Pool, group: int, length: int):
    _check(load().kv_pool_set_len(pool.handle, group, length))


def kv_pool_append(pool: Pool, group: int, k_rows, v_rows, n_tokens: Optional[int] = None, stream=None):
    """k_rows, v_rows: torch tensors [n, Hkv, D] (contiguous, pool dtype, keys unrotated) on the GPU;
    for host-only tests pass integers as opaque pointers together with n_tokens."""
    if hasattr(k_rows, "data_ptr"):
        assert k_rows.is_contiguous() and v_rows.is_contiguous() and k_rows.shape == v_rows.shape
        n_tokens = int(k_rows.shape[0]) if n_tokens is None else int(n_tokens)
        kp, vp_ = k_rows.data_ptr(), v_rows.data_ptr()
        stream = _stream(stream)
    else:
        kp, vp_ = k_rows, v_rows
        stream = C.c_void_p(0)
    _check(load().kv_pool_append(pool.handle, int(group), C.c_void_p(kp), C.c_void_p(vp_), int(n_tokens), stream))


def segment_select(pool: Pool, sel, sel_ptr, n_new: int) -> Plan:
    sel, sel_ptr = _i32(sel), _i32(sel_ptr)
    h = C.c_void_p()
    _check(load().segment_select(pool.handle, len(sel_ptr) - 1, _ip(sel), _ip(sel_ptr), n_new,
                                 C.byref(h)))
    return Plan(h, pool)


def segment_select_scored(pool: Pool, p, threshold: float, budget_tokens: int, n_new: int,
                          want_plan: bool = True) -> Tuple[np.ndarray, Optional[Plan]]:
    p = np.ascontiguousarray(p, dtype=np.float32)
    out = np.zeros(pool.desc.n_groups, dtype=np.int32)
    n = C.c_int32()
    h = C.c_void_p()
    _check(load().segment_select_scored(pool.handle, p.ctypes.data_as(C.POINTER(C.c_float)),
                                        C.c_float(threshold), C.c_int64(int(budget_tokens)), n_new,
                                        _ip(out), C.byref(n), C.byref(h) if want_plan else None))
    return out[:n.value].copy(), (Plan(h, pool) if want_plan else None)


def context_bytes(pool: Pool, plan: Plan) -> int:
    return int(load().en_context_bytes(pool.handle, plan.handle))


def workspace_bytes(pool: Pool, plan: Plan) -> int:
    return int(load().en_workspace_bytes(pool.handle, plan.handle))


def alloc_context(pool: Pool, plan: Plan):
    """Uninitialised context buffers (kc, vt) as flat byte tensors."""
    import torch
    n = context_bytes(pool, plan)
    dev = pool.k.device
    return (torch.empty(n, dtype=torch.uint8, device=dev), torch.empty(n, dtype=torch.uint8, device=dev))


def alloc_workspace(pool: Pool, plan: Plan):
    import torch
    return torch.empty(max(workspace_bytes(pool, plan), 256), dtype=torch.uint8, device=pool.k.device)


def gather_rope(pool: Pool, plan: Plan, k_new, v_new, kc, vt, stream=None):
    _check(load().gather_rope(pool.handle, plan.handle, k_new.data_ptr(), v_new.data_ptr(),
                              kc.data_ptr(), vt.data_ptr(), _stream(stream)))
    return kc, vt


def segmented_prefill_attention(pool: Pool, plan: Plan, q, kc, vt, out, ws=None, stream=None):
    _check(load().segmented_prefill_attention(
        pool.handle, plan.handle, q.data_ptr(), kc.data_ptr(), vt.data_ptr(), out.data_ptr(),
        ws.data_ptr() if ws is not None else None, ws.numel() * ws.element_size() if ws is not None else 0,
        _stream(stream)))
    return out


def gather_rope_queries(pool: Pool, plan: Plan, k_new, v_new, q, kc, vt, q_prep, stream=None):
    _check(load().gather_rope_queries(pool.handle, plan.handle, k_new.data_ptr(), v_new.data_ptr(), q.data_ptr(),
                                      kc.data_ptr(), vt.data_ptr(), q_prep.data_ptr(), _stream(stream)))
    return kc, vt, q_prep


def segmented_prefill_attention_prepared(pool: Pool, plan: Plan, q_prep, kc, vt, out, ws=None, mass_red_out=None,
                                         stream=None):
    _check(load().segmented_prefill_attention_prepared(
        pool.handle, plan.handle, q_prep.data_ptr(), kc.data_ptr(), vt.data_ptr(), out.data_ptr(),
        mass_red_out.data_ptr() if mass_red_out is not None else None,
        ws.data_ptr() if ws is not None else None, ws.numel() * ws.element_size() if ws is not None else 0,
        _stream(stream)))
    return out


def segment_attention_mass(pool: Pool, plan: Plan, ws, reduce: int, mass_out, stream=None):
    _check(load().segment_attention_mass(pool.handle, plan.handle, ws.data_ptr(), int(reduce),
                                         mass_out.data_ptr(), _stream(stream)))
    return mass_out


def segment_cluster_assign(pool: Pool, plan: Plan, ws, spans, score, assign=None, per_key: bool = False,
                           accumulate: bool = False, scale: float = 1.0, threshold: float = 0.0, stream=None):
    """spans: host int32 [n_obj+1]; score: float32 tensor [B, n_obj, Smax+1]; assign: int32 tensor
    [B, n_obj] or None. For host-only tests ws/score may be integers (opaque pointers)."""
    spans = _i32(spans)
    ptr = lambda t: C.c_void_p(t.data_ptr() if hasattr(t, "data_ptr") else t)
    _check(load().segment_cluster_assign(
        pool.handle, plan.handle, ptr(ws), len(spans) - 1, _ip(spans), int(per_key), int(accumulate),
        C.c_float(scale), C.c_float(threshold), ptr(score), ptr(assign) if assign is not None else None,
        _stream(stream) if hasattr(ws, "data_ptr") else C.c_void_p(0)))
    return score, assign


def segment_cluster_assign_rows(pool: Pool, plan: Plan, q_first: int, n_rows: int, ws, spans, score, assign=None,
                                per_key: bool = False, accumulate: bool = False, scale: float = 1.0,
                                threshold: float = 0.0, stream=None):
    """As segment_cluster_assign, from the scratch that segmented_decode_step(q_first, n_rows) left."""
    spans = _i32(spans)
    ptr = lambda t: C.c_void_p(t.data_ptr() if hasattr(t, "data_ptr") else t)
    _check(load().segment_cluster_assign_rows(
        pool.handle, plan.handle, int(q_first), int(n_rows), ptr(ws), len(spans) - 1, _ip(spans), int(per_key),
        int(accumulate), C.c_float(scale), C.c_float(threshold), ptr(score),
        ptr(assign) if assign is not None else None, _stream(stream) if hasattr(ws, "data_ptr") else C.c_void_p(0)))
    return score, assign


def decode_workspace_bytes(pool: Pool, plan: Plan, n_rows: int) -> int:
    return int(load().en_decode_workspace_bytes(pool.handle, plan.handle, int(n_rows)))


def segmented_decode_step(pool: Pool, plan: Plan, q_first: int, q, k_rows, v_rows, kc, vt, out, ws,
                          mass_out=None, stream=None):
    """q [B,n,Hq,D], k_rows/v_rows [B,n,Hkv,D], out [B,n,Hq,D]: contiguous torch tensors of the step."""
    n = int(q.shape[1])
    _check(load().segmented_decode_step(
        pool.handle, plan.handle, int(q_first), n, q.data_ptr(), k_rows.data_ptr(), v_rows.data_ptr(),
        kc.data_ptr(), vt.data_ptr(), out.data_ptr(), mass_out.data_ptr() if mass_out is not None else None,
        ws.data_ptr() if ws is not None else None, ws.numel() * ws.element_size() if ws is not None else 0,
        _stream(stream)))
    return out


def segmented_decode_step_static(pool: Pool, plan: Plan, q_first: int, q, k_rows, v_rows, kc, vt, out,
                                 mass_out=None, stream=None):
    """segmented_decode_step on the library's static device scratch: the call allocates nothing."""
    n = int(q.shape[1])
    _check(load().segmented_decode_step_static(
        pool.handle, plan.handle, int(q_first), n, q.data_ptr(), k_rows.data_ptr(), v_rows.data_ptr(),
        kc.data_ptr(), vt.data_ptr(), out.data_ptr(), mass_out.data_ptr() if mass_out is not None else None,
        _stream(stream)))
    return out


class Tier:
    """Handle of a residency tier. ``pool`` is the pool over the device slots (None for a tier that only
    keeps the books)."""

    def __init__(self, handle, pool: Optional[Pool], n_groups_total: int, desc: PoolDesc):
        self.handle, self.pool, self.n_groups_total, self.desc = handle, pool, n_groups_total, desc

    @property
    def stats(self) -> TierStats:
        st = TierStats()
        _check(load().kv_tier_get_stats(self.handle, C.byref(st)))
        return st

    def residency(self) -> np.ndarray:
        out = np.zeros(self.n_groups_total, dtype=np.int32)
        _check(load().kv_tier_residency(self.handle, _ip(out)))
        return out

    def close(self):
        if self.handle:
            if self.pool is not None:
                self.pool.close()
            load().kv_tier_destroy(self.handle)
            self.handle = None

    def __del__(self):
        if sys is None or sys.is_finalizing():
            return
        try:
            self.close()
        except Exception:
            pass


def kv_tier_slot_bytes(shape: Sequence[int], dtype: int) -> int:
    """Bytes of one device slot (K and V) for blocks [Hkv, C, D]."""
    Hkv, Cap, D = shape
    desc = PoolDesc(1, Cap, Hkv, Hkv, D, dtype, 1, 0, 1.0)
    return int(load().kv_tier_slot_bytes(C.byref(desc)))


def kv_tier_create(k_slots, v_slots, n_groups_total: int, n_q_heads: int, rope_base: float, max_ctx: int,
                   dtype: Optional[int] = None, shape: Optional[Sequence[int]] = None) -> Tier:
    """k_slots, v_slots: torch tensors [slots, Hkv, C, D] on the GPU, or None with ``shape`` and
    ``dtype`` for a tier that only keeps the books."""
    kp = vp_ = None
    if k_slots is not None:
        import torch
        assert k_slots.is_contiguous() and v_slots.is_contiguous() and k_slots.shape == v_slots.shape
        shape = tuple(k_slots.shape)
        dtype = EN_BF16 if k_slots.dtype == torch.bfloat16 else EN_F32
        kp, vp_ = k_slots.data_ptr(), v_slots.data_ptr()
    n_slots, Hkv, Cap, D = shape
    desc = PoolDesc(n_slots, Cap, Hkv, n_q_heads, D, dtype, max_ctx, 0, rope_base)
    h = C.c_void_p()
    _check(load().kv_tier_create(C.byref(desc), int(n_groups_total), C.c_void_p(kp), C.c_void_p(vp_), C.byref(h)))
    ph = load().kv_tier_pool(h)
    pool = Pool(C.c_void_p(ph), k_slots, v_slots, desc, owned=False) if ph else None
    return Tier(h, pool, int(n_groups_total), desc)


def kv_tier_put(tier: Tier, group: int, k_rows, v_rows, length: Optional[int] = None):
    """k_rows, v_rows: host arrays or CPU tensors [Hkv, len, D] in the tier's dtype (contiguous); for a
    tier that only keeps the books pass None and ``length``."""
    if k_rows is None:
        _check(load().kv_tier_put(tier.handle, int(group), None, None, int(length)))
        return
    assert k_rows.is_contiguous() and v_rows.is_contiguous() and k_rows.shape == v_rows.shape
    assert k_rows.device.type == "cpu" and v_rows.device.type == "cpu"
    length = int(k_rows.shape[1]) if length is None else int(length)
    _check(load().kv_tier_put(tier.handle, int(group), C.c_void_p(k_rows.data_ptr()),
                              C.c_void_p(v_rows.data_ptr()), length))


def kv_tier_append(tier: Tier, group: int, k_rows, v_rows, n_tokens: Optional[int] = None, stream=None):
    """k_rows, v_rows: torch tensors [n, Hkv, D] on the GPU (contiguous, tier dtype, keys unrotated); for a
    tier that only keeps the books pass None and n_tokens."""
    if k_rows is None:
        _check(load().kv_tier_append(tier.handle, int(group), None, None, int(n_tokens), C.c_void_p(0)))
        return
    assert k_rows.is_contiguous() and v_rows.is_contiguous() and k_rows.shape == v_rows.shape
    n_tokens = int(k_rows.shape[0]) if n_tokens is None else int(n_tokens)
    _check(load().kv_tier_append(tier.handle, int(group), C.c_void_p(k_rows.data_ptr()),
                                 C.c_void_p(v_rows.data_ptr()), n_tokens, _stream(stream)))


def kv_tier_select_scored(tier: Tier, p, threshold: float, budget_tokens: int) -> np.ndarray:
    p = np.ascontiguousarray(p, dtype=np.float32)
    assert p.shape == (tier.n_groups_total,)
    out = np.zeros(tier.n_groups_total, dtype=np.int32)
    n = C.c_int32()
    _check(load().kv_tier_select_scored(tier.handle, p.ctypes.data_as(C.POINTER(C.c_float)), C.c_float(threshold),
                                        C.c_int64(int(budget_tokens)), _ip(out), C.byref(n)))
    return out[:n.value].copy()


def kv_tier_fetch(tier: Tier, groups, stream=None) -> np.ndarray:
    """Make the groups resident; returns the slot of each (ids for segment_select on ``tier.pool``)."""
    groups = _i32(groups)
    slots = np.zeros(len(groups), dtype=np.int32)
    st = C.c_void_p(0) if tier.pool is None else _stream(stream)
    _check(load().kv_tier_fetch(tier.handle, _ip(groups), len(groups), _ip(slots), st))
    return slots


def kv_tier_fence(tier: Tier, stream=None):
    st = C.c_void_p(0) if tier.pool is None else _stream(stream)
    _check(load().kv_tier_fence(tier.handle, st))


def kv_tier_prefetch(tier: Tier, groups) -> int:
    groups = _i32(groups)
    n = C.c_int32()
    _check(load().kv_tier_prefetch(tier.handle, _ip(groups), len(groups), C.byref(n)))
    return n.value


def timing_enable(pool: Pool, n: int):
    _check(load().en_timing_enable(pool.handle, int(n)))


def timing_collect(pool: Pool, cap: int) -> np.ndarray:
    """Durations (ms) of the attention kernel launches on this pool recorded since
    the last collect."""
    ms = np.zeros(cap, dtype=np.float32)
    n = C.c_int32()
    _check(load().en_timing_collect(pool.handle, ms.ctypes.data_as(C.POINTER(C.c_float)), cap, C.byref(n)))
    return ms[:n.value].copy()


def ceiling_mfma_bf16(sink, n_workgroups: int, iters: int, constant_operands: bool, stream=None) -> float:
    """Enqueue the matrix-instruction-only loop; returns the operations of the launch."""
    flops = C.c_double()
    _check(load().en_ceiling_mfma_bf16(sink.data_ptr(), sink.numel() * sink.element_size(), int(n_workgroups),
                                       int(iters), int(bool(constant_operands)), C.byref(flops), _stream(stream)))
    return flops.value


def ceiling_read_stream(src, sink, n_workgroups: int, stream=None) -> int:
    """Enqueue the read-only stream over `src`; returns the bytes one launch reads."""
    nbytes = src.numel() * src.element_size()
    _check(load().en_ceiling_read_stream(src.data_ptr(), nbytes, sink.data_ptr(), sink.numel() * sink.element_size(),
                                         int(n_workgroups), _stream(stream)))
    return nbytes
