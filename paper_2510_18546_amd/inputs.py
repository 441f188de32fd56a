"""Seeded synthetic workloads for the segmented-attention planning step.

This module only draws random tensors and index lists with the shapes of the
benchmark configurations. It contains none of the method's arithmetic
(no RoPE, no softmax, no prefix sums) so that both the HIP path and the CPU
oracle can be fed from it without sharing any computation.

The inputs stand in for the paper's navigation workload (Section 4: HM3D
episodes with map-description prompts, which cannot be shipped): many small
per-group K/V blocks of ragged length (Appendix B shows a handful of
{object, position} entries per group), a retrieved subset in arbitrary order,
a short instruction + trajectory query block (Appendix B, planning prompt)
and one-token decode steps (Section 3.2: about 40 per plan), on a
Llama-3.2-11B-shaped layer (Appendix C, Table 7).

Draw order is fixed: len[G] -> K_pool -> V_pool -> per-agent sel -> Q ->
K_new -> V_new, all from one numpy Generator(PCG64(seed)).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np

F32 = 0
BF16 = 1


@dataclass(frozen=True)
class Config:
    name: str
    seed: int
    dtype: int            # F32 or BF16 (storage type of Q/K/V/out)
    n_agents: int         # B
    n_q_heads: int        # Hq
    n_kv_heads: int       # Hkv
    head_dim: int         # D
    n_groups: int         # G
    capacity: int         # C, token slots per group
    len_lo: int           # group lengths uniform in [len_lo, len_hi]
    len_hi: int
    n_sel: int            # S, groups selected per agent
    n_new: int            # N_q, new prompt tokens per agent
    rope_base: float
    act_scale: float = 1.0          # multiplies every activation tensor
    fixed_sel: Optional[tuple] = None
    planted: bool = False           # concentrate attention on one segment


CONFIGS: Dict[str, Config] = {
    # tiny fp32 layer, explicit selection [1,3,4,6]
    "c0": Config("c0", 0, F32, 1, 4, 1, 64, 8, 32, 32, 32, 4, 64, 10000.0,
                 fixed_sel=(1, 3, 4, 6)),
    # Llama-3.2-11B-shaped layer, ragged groups, activations scaled by 128^-1/2
    "c1": Config("c1", 1, BF16, 1, 32, 8, 128, 64, 128, 64, 128, 16, 256,
                 500000.0, act_scale=128.0 ** -0.5),
    # large map: 32 x 256 = 8192 cached tokens + 512 new
    "c2": Config("c2", 2, BF16, 1, 32, 8, 128, 256, 256, 256, 256, 32, 512,
                 500000.0),
    # 16 agents sharing one pool, ragged
    "c3": Config("c3", 3, BF16, 16, 32, 8, 128, 512, 128, 32, 128, 24, 128,
                 500000.0),
    # decode: 64 agents, one new token, 16K-token contexts
    "c4": Config("c4", 4, BF16, 64, 32, 8, 128, 1024, 256, 256, 256, 64, 1,
                 500000.0),
    # the large map of c2 on a layer of the paper's largest planner (Appendix C, Table 7: LLaVA-34b,
    # hidden size 7168 = 56 heads of 128). The paper does not give the head split; 8 KV heads is
    # the published configuration of that backbone family and is taken as the reading here.
    "c5": Config("c5", 5, BF16, 1, 56, 8, 128, 256, 256, 256, 256, 32, 512,
                 5000000.0),
}


def variant(cfg: Config, **kw) -> Config:
    """A config with some fields replaced (used for reduced-size parity cases)."""
    return replace(cfg, **kw)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), returned as
    float32. NaN stays NaN."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    out = (r & 0xFFFFFFFF).astype(np.uint32).view(np.float32)
    return np.where(np.isnan(x), np.float32(np.nan), out).astype(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


@dataclass
class Workload:
    cfg: Config
    lens: np.ndarray          # int32 [G]
    k_pool: np.ndarray        # float32 [G,Hkv,C,D], rows t >= len are NaN
    v_pool: np.ndarray        # float32 [G,Hkv,C,D], rows t >= len are NaN
    sel: np.ndarray           # int32, all agents' lists concatenated
    sel_ptr: np.ndarray       # int32 [B+1]
    q: np.ndarray             # float32 [B,Nq,Hq,D]
    k_new: np.ndarray         # float32 [B,Nq,Hkv,D]
    v_new: np.ndarray         # float32 [B,Nq,Hkv,D]
    meta: dict = field(default_factory=dict)

    def agent_sel(self, b: int) -> np.ndarray:
        return self.sel[self.sel_ptr[b]:self.sel_ptr[b + 1]]


def _draw(rng: np.random.Generator, shape, scale: float, bf16: bool) -> np.ndarray:
    x = rng.standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    if bf16:
        x = round_to_bf16(x)
    return x


def make_workload(cfg: Config, poison: bool = True,
                  sel_lists: Optional[List[List[int]]] = None) -> Workload:
    """Draw one workload. With ``poison`` the unused rows of every group
    (t >= len) hold NaN so that any over-read shows up in the result."""
    rng = np.random.default_rng(cfg.seed)
    G, H, C, D = cfg.n_groups, cfg.n_kv_heads, cfg.capacity, cfg.head_dim
    B, Nq, Hq = cfg.n_agents, cfg.n_new, cfg.n_q_heads
    bf = cfg.dtype == BF16

    lens = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=G, dtype=np.int64).astype(np.int32)
    k_pool = _draw(rng, (G, H, C, D), cfg.act_scale, bf)
    v_pool = _draw(rng, (G, H, C, D), cfg.act_scale, bf)
    if poison:
        t = np.arange(C, dtype=np.int32)[None, :] >= lens[:, None]      # [G,C]
        mask = np.broadcast_to(t[:, None, :, None], k_pool.shape)
        k_pool[mask] = np.nan
        v_pool[mask] = np.nan

    lists = []
    for b in range(B):
        if sel_lists is not None:
            lists.append(np.asarray(sel_lists[b], dtype=np.int32))
        elif cfg.fixed_sel is not None:
            lists.append(np.asarray(cfg.fixed_sel, dtype=np.int32))
        else:
            lists.append(rng.choice(G, size=cfg.n_sel, replace=False).astype(np.int32))
    sel_ptr = np.zeros(B + 1, dtype=np.int32)
    sel_ptr[1:] = np.cumsum([len(l) for l in lists])
    sel = (np.concatenate(lists) if lists else np.zeros(0)).astype(np.int32)

    q = _draw(rng, (B, Nq, Hq, D), cfg.act_scale, bf)
    k_new = _draw(rng, (B, Nq, H, D), cfg.act_scale, bf)
    v_new = _draw(rng, (B, Nq, H, D), cfg.act_scale, bf)

    meta = {}
    if cfg.planted:
        # One selected segment per agent receives keys that share a common
        # component with every query, so attention mass concentrates there
        # (the situation of Fig. 4: a few relevant entries in a large map).
        # The shared direction lives in the slowest-rotating coordinates of the
        # first half so that position encoding leaves the alignment intact.
        u = np.zeros(D, dtype=np.float32)
        u[3 * D // 8:D // 2] = 1.0
        u /= np.linalg.norm(u)
        alpha = np.float32((8.0 * np.sqrt(D)) ** 0.5)
        q = q + alpha * u
        for b in range(B):
            g = int(lists[b][len(lists[b]) // 2]) if len(lists[b]) else -1
            meta.setdefault("planted_group", []).append(g)
            if g >= 0:
                n = int(lens[g])
                k_pool[g, :, :n, :] = 0.25 * k_pool[g, :, :n, :] + alpha * u
        if bf:
            q = round_to_bf16(q)
            k_pool = round_to_bf16(k_pool)

    return Workload(cfg, lens, k_pool, v_pool, sel, sel_ptr, q, k_new, v_new, meta)



def drifting_scores(seed: int, n_groups: int, n_steps: int, rho: float = 0.95) -> np.ndarray:
    """Relevance scores of ``n_groups`` groups over ``n_steps`` planning steps, float32
    [n_steps, n_groups]: a stationary first-order autoregression per group with unit variance,
    s[t] = rho * s[t-1] + sqrt(1 - rho^2) * noise. Stands in for the similarity between the goal
    and each group's description along an episode (Section 3.4), which changes little between
    adjacent planning steps (Section 4, cache hit rate): rho sets how little."""
    rng = np.random.Generator(np.random.PCG64(seed))
    s = np.empty((n_steps, n_groups), dtype=np.float64)
    s[0] = rng.standard_normal(n_groups)
    for t in range(1, n_steps):
        s[t] = rho * s[t - 1] + np.sqrt(1.0 - rho * rho) * rng.standard_normal(n_groups)
    return s.astype(np.float32)
