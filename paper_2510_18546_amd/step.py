"""One planning step on the GPU: upload a workload, then call the library's
five entry points in order. Plumbing shared by the tests, the smoke check and
the benchmark; it holds no arithmetic of the method.
"""
from __future__ import annotations

from typing import Optional

import numpy as np

from . import binding as B
from . import inputs as I


def _to_device(x: np.ndarray, bf16: bool, device):
    import torch
    if bf16:
        return torch.from_numpy(I.bf16_bits(x).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device)


def _to_host(t) -> np.ndarray:
    import torch
    if t.dtype == torch.bfloat16:
        return I.bf16_bits_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16))
    return t.cpu().numpy()


class PlanningStep:
    """Device-resident state of one workload: pool, plan, inputs, buffers."""

    def __init__(self, w: I.Workload, device: str = "cuda:0", n_splits: Optional[int] = None,
                 max_ctx: Optional[int] = None, prepared: Optional[bool] = None,
                 values_from_pool: bool = False):
        """prepared: the queries are prepared in the gather launch and the reduced masses come out
        of the attention call (gather_rope_queries + segmented_prefill_attention_prepared), where the
        library offers that (bf16 contexts, steps of more than 32 query rows per KV head): the
        default. False: the five calls gather_rope / segmented_prefill_attention /
        segment_attention_mass.
        values_from_pool: the plan leaves the values where they are (en_plan_values_from_pool)."""
        import torch
        cfg = w.cfg
        self.w, self.cfg = w, cfg
        self.bf16 = cfg.dtype == I.BF16
        self.device = torch.device(device)
        self.k_pool = _to_device(w.k_pool, self.bf16, self.device)
        self.v_pool = _to_device(w.v_pool, self.bf16, self.device)
        self.q = _to_device(w.q, self.bf16, self.device)
        self.k_new = _to_device(w.k_new, self.bf16, self.device)
        self.v_new = _to_device(w.v_new, self.bf16, self.device)
        if max_ctx is None:
            max_ctx = cfg.n_sel * cfg.capacity + cfg.n_new
            if len(w.sel_ptr) > 1:
                max_ctx = max(max_ctx, int(np.max(np.diff(w.sel_ptr))) * cfg.capacity + cfg.n_new)
        self.pool = B.kv_pool_create(self.k_pool, self.v_pool, w.lens, cfg.n_q_heads, cfg.rope_base,
                                     max_ctx)
        can_prepare = self.bf16 and (cfg.n_q_heads // cfg.n_kv_heads) * cfg.n_new > 32
        self.prepared = can_prepare if prepared is None else (prepared and can_prepare)
        self.q_prep = torch.empty_like(self.q) if self.prepared else None
        self.values_from_pool = values_from_pool
        self.plan = None
        self.select(n_splits)
        self.out = torch.empty((cfg.n_agents, cfg.n_new, cfg.n_q_heads, cfg.head_dim),
                               dtype=torch.bfloat16 if self.bf16 else torch.float32,
                               device=self.device)

    # -- the five entry points, in path order --------------------------------
    def select(self, n_splits: Optional[int] = None):
        import torch
        if self.plan is not None:
            self.plan.close()
        self.plan = B.segment_select(self.pool, self.w.sel, self.w.sel_ptr, self.cfg.n_new)
        if n_splits is not None:
            self.plan.set_splits(n_splits)
        if self.values_from_pool:
            self.plan.values_from_pool(True)
        inf = self.plan.info
        self.info = inf
        if getattr(self, "_ctx_bytes", -1) != B.context_bytes(self.pool, self.plan):
            self.kc, self.vt = B.alloc_context(self.pool, self.plan)
            self._ctx_bytes = B.context_bytes(self.pool, self.plan)
        if getattr(self, "_ws_bytes", -1) != B.workspace_bytes(self.pool, self.plan):
            self.ws = B.alloc_workspace(self.pool, self.plan)
            self._ws_bytes = B.workspace_bytes(self.pool, self.plan)
        S1 = inf.max_segments + 1
        if getattr(self, "_S1", -1) != S1:
            self.mass = torch.empty((self.cfg.n_agents, self.cfg.n_new, self.cfg.n_q_heads, S1),
                                    dtype=torch.float32, device=self.device)
            self.mass_red = torch.empty((self.cfg.n_agents, S1), dtype=torch.float32,
                                        device=self.device)
            self._S1 = S1
        return self.plan

    def gather(self):
        if self.prepared:
            B.gather_rope_queries(self.pool, self.plan, self.k_new, self.v_new, self.q, self.kc, self.vt, self.q_prep)
        else:
            B.gather_rope(self.pool, self.plan, self.k_new, self.v_new, self.kc, self.vt)

    def attention(self, reduced_mass: bool = False):
        """reduced_mass (prepared form only): the reduced masses come out of this call too."""
        if self.prepared:
            B.segmented_prefill_attention_prepared(self.pool, self.plan, self.q_prep, self.kc, self.vt, self.out,
                                                   self.ws, self.mass_red if reduced_mass else None)
        else:
            assert not reduced_mass
            B.segmented_prefill_attention(self.pool, self.plan, self.q, self.kc, self.vt, self.out, self.ws)

    def masses(self, reduce: int):
        B.segment_attention_mass(self.pool, self.plan, self.ws, reduce,
                                 self.mass_red if reduce else self.mass)

    def run(self, full_mass: bool = True, reduced_mass: bool = True):
        self.gather()
        self.attention(reduced_mass and self.prepared)
        if full_mass:
            self.masses(0)
        if reduced_mass and not self.prepared:
            self.masses(1)

    # -- read-back ------------------------------------------------------------
    def out_host(self) -> np.ndarray:
        return _to_host(self.out).astype(np.float64)

    def mass_host(self) -> np.ndarray:
        return self.mass.cpu().numpy().astype(np.float64)

    def mass_red_host(self) -> np.ndarray:
        return self.mass_red.cpu().numpy().astype(np.float64)

    def context_host(self, b: int):
        """(Kc, V) of agent b as float32 [Hkv, L, D] decoded from the context
        buffers' documented layout (V un-transposed, columns un-permuted)."""
        import torch
        cfg, inf = self.cfg, self.info
        T, D, H = inf.ctx_stride, cfg.head_dim, cfg.n_kv_heads
        L = int(self.plan.offsets(b)[-1]) + cfg.n_new
        if self.bf16:
            kc = _to_host(self.kc.view(torch.bfloat16).view(cfg.n_agents, H, T, D)[b])
            vt = _to_host(self.vt.view(torch.bfloat16).view(cfg.n_agents, H, D, T)[b])
            j = np.arange(T)
            col = (j & ~0xC) | ((j & 4) << 1) | ((j & 8) >> 1)
            v = np.transpose(vt[:, :, col], (0, 2, 1))
        else:
            kc = _to_host(self.kc.view(torch.float32).view(cfg.n_agents, H, T, D)[b])
            v = _to_host(self.vt.view(torch.float32).view(cfg.n_agents, H, T, D)[b])
        return kc[:, :L], v[:, :L], kc[:, L:], v[:, L:]
