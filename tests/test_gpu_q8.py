"""8-bit pools (an option beside the paper's method) through the C ABI against the oracle: the gather
turns codes and scales into the same bf16 contexts as for a bf16 pool, the attention over them matches the
oracle run on the dequantised values, and an append quantises exactly as the oracle does."""
import numpy as np
import pytest

from paper_2510_18546_amd import inputs as I
from test_gpu_parity import announce, check_mass, check_out, small, step_mod  # noqa: F401

pytestmark = pytest.mark.gpu


def quantised_pool(oracle, w):
    """(codes, scales, dequantised values) of both pool arrays; rows beyond a group's length keep a NaN
    scale so that reading one shows up."""
    out = []
    for a in (w.k_pool, w.v_pool):
        used = np.isfinite(a).all(-1)
        q, s = oracle.quantize_rows(np.where(used[..., None], a, 0.0))
        s = np.where(used, s, np.float32(np.nan)).astype(np.float32)
        out.append((q, s, oracle.dequantize_rows(q, np.where(used, s, 0.0))))
    return out


class Q8Step:
    """A planning step over an EN_I8 pool (plumbing, like step.PlanningStep)."""

    def __init__(self, S, B, w, kq, vq, n_splits=None, max_ctx=None):
        import torch
        cfg = w.cfg
        self.cfg, self.w = cfg, w
        dev = torch.device("cuda:0")
        self.k_codes = torch.from_numpy(kq[0]).to(dev)
        self.v_codes = torch.from_numpy(vq[0]).to(dev)
        self.k_scale = torch.from_numpy(kq[1]).to(dev)
        self.v_scale = torch.from_numpy(vq[1]).to(dev)
        self.q = S._to_device(w.q, True, dev)
        self.k_new = S._to_device(w.k_new, True, dev)
        self.v_new = S._to_device(w.v_new, True, dev)
        max_ctx = max_ctx or cfg.n_groups * cfg.capacity + cfg.n_new
        self.pool = B.kv_pool_create(self.k_codes, self.v_codes, w.lens, cfg.n_q_heads, cfg.rope_base, max_ctx)
        assert self.pool.desc.dtype == B.EN_I8
        B.kv_pool_set_scales(self.pool, self.k_scale, self.v_scale)
        self.plan = B.segment_select(self.pool, w.sel, w.sel_ptr, cfg.n_new)
        if n_splits:
            self.plan.set_splits(n_splits)
        self.info = self.plan.info
        self.kc, self.vt = B.alloc_context(self.pool, self.plan)
        self.ws = B.alloc_workspace(self.pool, self.plan)
        self.out = torch.empty((cfg.n_agents, cfg.n_new, cfg.n_q_heads, cfg.head_dim), dtype=torch.bfloat16, device=dev)
        self.mass = torch.empty((cfg.n_agents, cfg.n_new, cfg.n_q_heads, self.info.max_segments + 1),
                                dtype=torch.float32, device=dev)
        self.B, self.S = B, S

    def run(self):
        B = self.B
        self.ws.fill_(0xFF)
        B.gather_rope(self.pool, self.plan, self.k_new, self.v_new, self.kc, self.vt)
        B.segmented_prefill_attention(self.pool, self.plan, self.q, self.kc, self.vt, self.out, self.ws)
        B.segment_attention_mass(self.pool, self.plan, self.ws, 0, self.mass)


@pytest.mark.parametrize("d,n_new,splits", [(128, 70, None), (64, 70, 3), (128, 2, None), (128, 1, 5)])
def test_q8_pool_step_matches_oracle_on_dequantised_values(step_mod, oracle, d, n_new, splits):
    import torch
    from paper_2510_18546_amd import binding as B
    cfg = small(f"q8-{d}-{n_new}", 1200 + d + n_new, n_agents=2, len_lo=0, n_sel=6, n_new=n_new, head_dim=d,
                rope_base=5e5 if d == 128 else 1e4)
    announce(f"8-bit pool: D={d} Nq={n_new} splits={splits}")
    w = I.make_workload(cfg)
    kq, vq = quantised_pool(oracle, w)
    st = Q8Step(step_mod, B, w, kq, vq, n_splits=splits)
    st.kc.fill_(0xFF)
    st.vt.fill_(0xFF)
    st.run()
    torch.cuda.synchronize()
    # the gathered context: values are the dequantised ones rounded to bf16, keys those rotated
    T, Hkv = st.info.ctx_stride, cfg.n_kv_heads
    for b in range(cfg.n_agents):
        L = int(st.plan.offsets(b)[-1]) + cfg.n_new
        kc = step_mod._to_host(st.kc.view(torch.bfloat16).view(cfg.n_agents, Hkv, T, d)[b])[:, :L]
        vt = step_mod._to_host(st.vt.view(torch.bfloat16).view(cfg.n_agents, Hkv, d, T)[b])
        j = np.arange(T)
        col = (j & ~0xC) | ((j & 4) << 1) | ((j & 8) >> 1)
        v = np.transpose(vt[:, :, col], (0, 2, 1))[:, :L]
        rk, rv = oracle.gather_rope(kq[2], vq[2], w.lens, w.agent_sel(b), w.k_new[b], w.v_new[b], cfg.rope_base)
        assert np.array_equal(v, I.round_to_bf16(rv.astype(np.float32))), "values: dequantised, rounded to bf16 once"
        ulp = np.maximum(np.abs(rk), 2.0 ** -126) * 2.0 ** -8
        assert (np.abs(kc - rk) <= 1.01 * ulp + 1e-7).all(), "keys: dequantised, rotated, rounded once"
    # attention over it against the oracle on the dequantised pool
    ref_out, ref_mass = oracle.attention(kq[2], vq[2], w.lens, w.sel, w.sel_ptr, w.q, w.k_new, w.v_new, cfg.rope_base)
    check_out(cfg, step_mod._to_host(st.out).astype(np.float64), ref_out)
    m = st.mass.cpu().numpy().astype(np.float64)
    check_mass(cfg, m, ref_mass)
    np.testing.assert_allclose(m.sum(-1), 1.0, atol=1e-4)


@pytest.mark.parametrize("d", [128, 64])
def test_q8_append_quantises_like_the_oracle(step_mod, oracle, d):
    import torch
    from paper_2510_18546_amd import binding as B
    cfg = small(f"q8-append-{d}", 1300 + d, n_agents=1, len_lo=10, len_hi=60, n_sel=4, n_new=9, head_dim=d,
                rope_base=5e5 if d == 128 else 1e4)
    announce(f"8-bit pool append: D={d}")
    w = I.make_workload(cfg)
    kq, vq = quantised_pool(oracle, w)
    st = Q8Step(step_mod, B, w, kq, vq)
    g = int(w.agent_sel(0)[1])
    n = 7
    rng = np.random.default_rng(3)
    rows_k = I.round_to_bf16(rng.standard_normal((n, cfg.n_kv_heads, d)).astype(np.float32) * 3)
    rows_v = I.round_to_bf16(rng.standard_normal((n, cfg.n_kv_heads, d)).astype(np.float32) * 0.01)
    rows_k[2, 0] = 0.0                       # a row of zeros: scale 0, codes 0
    B.kv_pool_append(st.pool, g, step_mod._to_device(rows_k, True, "cuda:0"), step_mod._to_device(rows_v, True, "cuda:0"))
    torch.cuda.synchronize()
    first = int(w.lens[g])
    for rows, codes, scale in ((rows_k, st.k_codes, st.k_scale), (rows_v, st.v_codes, st.v_scale)):
        q, s = oracle.quantize_rows(np.transpose(rows, (1, 0, 2)))          # [Hkv, n, D]
        assert np.array_equal(codes[g, :, first:first + n].cpu().numpy(), q), "codes are decided in float32 on both sides"
        assert np.array_equal(scale[g, :, first:first + n].cpu().numpy(), s)
    # and a step over the longer group
    kd, vd = kq[2].copy(), vq[2].copy()
    kd[g, :, first:first + n] = oracle.dequantize_rows(*oracle.quantize_rows(np.transpose(rows_k, (1, 0, 2))))
    vd[g, :, first:first + n] = oracle.dequantize_rows(*oracle.quantize_rows(np.transpose(rows_v, (1, 0, 2))))
    lens = w.lens.copy()
    lens[g] += n
    st.plan.close()
    st.plan = B.segment_select(st.pool, w.sel, w.sel_ptr, cfg.n_new)
    st.info = st.plan.info
    st.kc, st.vt = B.alloc_context(st.pool, st.plan)
    st.ws = B.alloc_workspace(st.pool, st.plan)
    st.run()
    torch.cuda.synchronize()
    ref_out, ref_mass = oracle.attention(kd, vd, lens, w.sel, w.sel_ptr, w.q, w.k_new, w.v_new, cfg.rope_base)
    check_out(cfg, step_mod._to_host(st.out).astype(np.float64), ref_out)
    check_mass(cfg, st.mass.cpu().numpy().astype(np.float64), ref_mass)
