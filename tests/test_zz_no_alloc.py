"""segmented_decode_step_static: the decode step on the library's static device scratch, for
callers that cannot allocate. Through the C ABI, against segmented_decode_step with a workspace of
the caller's: the two run the same kernels over the same scratch layout, so outputs and masses are
compared bit for bit (tighter than the bf16 tolerance); the first case is also checked against the
oracle's prefill rows. Two calls in a row, the second on a smaller plan: the scratch keeps what the
first left in it."""
import sys

import numpy as np
import pytest

from paper_2510_18546_amd import inputs as I


def announce(msg):
    sys.__stderr__.write(f"[gpu-case] {msg}\n")
    sys.__stderr__.flush()


def _case(cfg, n_rows, tag):
    import torch
    from paper_2510_18546_amd import binding as B
    from paper_2510_18546_amd import step as S
    announce(f"static scratch {tag}: B={cfg.n_agents} Hq={cfg.n_q_heads} Hkv={cfg.n_kv_heads} D={cfg.head_dim} "
             f"S={cfg.n_sel} len={cfg.len_lo}..{cfg.len_hi} Nq={cfg.n_new} rows per step={n_rows} seed={cfg.seed}")
    w = I.make_workload(cfg)
    st = S.PlanningStep(w)
    st.gather()                                   # creates the rotary table and the plan's block
    S1 = st.info.max_segments + 1
    ws = torch.empty(max(B.decode_workspace_bytes(st.pool, st.plan, n_rows), 256), dtype=torch.uint8, device="cuda:0")
    results = []
    for q_first in range(0, cfg.n_new - n_rows + 1, n_rows):
        sl = slice(q_first, q_first + n_rows)
        q, k, v = (t[:, sl].contiguous() for t in (st.q, st.k_new, st.v_new))
        out_a, out_b = torch.empty_like(q), torch.empty_like(q)
        mass_a = torch.full((cfg.n_agents, n_rows, cfg.n_q_heads, S1), -1.0, dtype=torch.float32, device="cuda:0")
        mass_b = mass_a.clone()
        ws.fill_(0xA5)
        B.segmented_decode_step(st.pool, st.plan, q_first, q, k, v, st.kc, st.vt, out_a, ws, mass_out=mass_a)
        B.segmented_decode_step_static(st.pool, st.plan, q_first, q, k, v, st.kc, st.vt, out_b, mass_out=mass_b)
        torch.cuda.synchronize()
        assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16)), f"outputs differ at row {q_first}"
        assert torch.equal(mass_a.view(torch.int32), mass_b.view(torch.int32)), f"masses differ at row {q_first}"
        results.append((q_first, S._to_host(out_b).astype(np.float64), mass_b.cpu().numpy().astype(np.float64)))
    return w, results


@pytest.mark.gpu
def test_static_scratch_decode_equals_workspace_decode(oracle):
    big = I.Config("static-big", 71, I.BF16, 2, 8, 2, 128, 40, 96, 40, 96, 30, 8, 500000.0)
    w, results = _case(big, 4, "first call")
    # ... and against the oracle: rows of the step are rows of a prefill over all tokens up to them
    ref_out, ref_mass = oracle.attention(w.k_pool, w.v_pool, w.lens, w.sel, w.sel_ptr, w.q, w.k_new, w.v_new,
                                         big.rope_base)
    for q_first, out, mass in results:
        n = out.shape[1]
        assert np.abs(out - ref_out[:, q_first:q_first + n]).max() <= 2e-2
        # a step's last bucket holds the new tokens visible to the row, as the prefill's does
        assert np.abs(mass - ref_mass[:, q_first:q_first + n]).max() <= 1e-2
    # the second call: a smaller plan, fewer splits, one row; the scratch still holds the first call's data
    small = I.Config("static-small", 72, I.BF16, 1, 8, 2, 128, 6, 64, 10, 64, 3, 3, 500000.0)
    _case(small, 1, "second call, smaller")


def test_static_scratch_refusals_without_device():
    """Host-side checks come first: a step whose scratch exceeds the static array is refused with
    CAPACITY, a plan that has not been through gather_rope with INVALID_ARG; nothing is launched."""
    from paper_2510_18546_amd import binding as B
    lens = np.full(64, 128, np.int32)
    pool = B.kv_pool_create(None, None, lens, n_q_heads=32, rope_base=1e4, max_ctx=64 * 128 + 8, dtype=B.EN_BF16,
                            k_ptr=0x1000, v_ptr=0x2000, shape=(64, 8, 128, 128))
    n_agents = 400                                  # 400 agents x 32 heads x 65 buckets x 2 splits: above 8 MiB
    sel = np.tile(np.arange(64, dtype=np.int32), n_agents)
    ptr = np.arange(n_agents + 1, dtype=np.int32) * 64
    plan = B.segment_select(pool, sel, ptr, 1)
    assert B.decode_workspace_bytes(pool, plan, 1) > 8 << 20
    lib = B.load()
    fake = 0x10000
    rc = lib.segmented_decode_step_static(pool.handle, plan.handle, 0, 1, fake, fake, fake, fake, fake, fake, None, None)
    assert rc == 4 and b"static" in lib.en_last_error()
    one = B.segment_select(pool, np.arange(4, dtype=np.int32), [0, 4], 1)
    assert B.decode_workspace_bytes(pool, one, 1) <= 8 << 20
    rc = lib.segmented_decode_step_static(pool.handle, one.handle, 0, 1, fake, fake, fake, fake, fake, fake, None, None)
    assert rc == 1 and b"gather_rope" in lib.en_last_error()
    rc = lib.segmented_decode_step_static(pool.handle, one.handle, 0, 0, fake, fake, fake, fake, fake, fake, None, None)
    assert rc == 2
