"""Random sweeps of the HIP path against the oracle, on top of the hand-picked cases: shapes, head
ratios, ragged and empty segments, split counts (also more splits than an agent has key tiles), planted
dominant keys, decode steps of random sizes, clustering spans. Seeds are fixed; the scratch is filled
with a NaN pattern before every run so that anything read without having been written shows up.
Two sweeps like these, run for thousands of cases, found the two defects that
test_agent_with_fewer_tiles_than_splits and test_bf16_dominant_key_among_tiny_segments now pin."""
import numpy as np
import pytest

from paper_2510_18546_amd import inputs as I
from test_gpu_parity import announce, check_mass, check_out, oracle_full, run_case, step_mod  # noqa: F401

pytestmark = pytest.mark.gpu


def seeds(*fixed):
    """The fixed seeds of a sweep, plus EN_SWEEP_EXTRA_SEEDS more (an integer) for a longer run by hand."""
    import os
    extra = int(os.environ.get("EN_SWEEP_EXTRA_SEEDS", "0"))
    return list(fixed) + [10007 * (i + 1) + fixed[0] for i in range(extra)]


@pytest.mark.parametrize("seed", seeds(101, 202))
def test_random_planning_steps(step_mod, oracle, seed, monkeypatch):
    orig = step_mod.PlanningStep.run

    def run(self, *a, **k):
        self.ws.fill_(0xFF)
        return orig(self, *a, **k)
    monkeypatch.setattr(step_mod.PlanningStep, "run", run)
    rng = np.random.default_rng(seed)
    for case in range(150):
        dtype = I.BF16 if rng.random() < 0.7 else I.F32
        hkv = int(rng.choice([1, 2, 4]))
        r = int(rng.choice([1, 2, 3, 4, 7]))
        d = int(rng.choice([64, 128]))
        cap = int(rng.choice([9, 33, 64, 96, 130]))
        len_lo = int(rng.integers(0, cap + 1))
        len_hi = int(rng.integers(len_lo, cap + 1))
        n_groups = int(rng.integers(2, 40))
        n_sel = int(rng.integers(0, n_groups + 1))
        n_new = int(rng.choice([1, 2, 5, 17, 33, 64, 70, 129]))
        n_agents = int(rng.choice([1, 1, 2, 3]))
        splits = rng.choice([None, 1, 2, 3, 5, 9, 13])
        splits = None if splits is None else int(splits)
        cfg = I.Config(f"sweep{seed}-{case}", seed * 1000 + case, dtype, n_agents, hkv * r, hkv, d, n_groups, cap,
                       len_lo, len_hi, n_sel, n_new, 1e4 if d == 64 else 5e5,
                       act_scale=float(rng.choice([1.0, 1.0, 0.3])),
                       planted=bool(rng.random() < 0.2 and n_sel > 0))
        run_case(step_mod, oracle, cfg, n_splits=splits)


@pytest.mark.parametrize("seed", seeds(303))
def test_random_decode_steps_and_clustering(step_mod, oracle, seed):
    import torch
    from paper_2510_18546_amd import binding as B
    rng = np.random.default_rng(seed)
    for case in range(120):
        dtype = I.BF16 if rng.random() < 0.7 else I.F32
        hkv = int(rng.choice([1, 2, 4]))
        r = int(rng.choice([1, 2, 4, 7]))
        d = int(rng.choice([64, 128]))
        cap = int(rng.choice([9, 33, 64, 130]))
        len_lo = int(rng.integers(0, cap + 1))
        len_hi = int(rng.integers(len_lo, cap + 1))
        n_groups = int(rng.integers(2, 30))
        n_sel = int(rng.integers(0, n_groups + 1))
        n_new = int(rng.choice([3, 8, 17, 40, 70]))
        n_agents = int(rng.choice([1, 2, 3]))
        cfg = I.Config(f"dsweep{seed}-{case}", seed * 1000 + case, dtype, n_agents, hkv * r, hkv, d, n_groups, cap,
                       len_lo, len_hi, n_sel, n_new, 1e4 if d == 64 else 5e5,
                       planted=bool(rng.random() < 0.3 and n_sel > 0))
        announce(f"decode / cluster sweep {cfg}")
        w = I.make_workload(cfg)
        st = step_mod.PlanningStep(w)
        ref_out, ref_mass = oracle_full(oracle, w)
        S1 = st.info.max_segments + 1
        # decode steps of random sizes over a context gathered once equal the prefill rows
        B.gather_rope(st.pool, st.plan, torch.zeros_like(st.k_new), torch.zeros_like(st.v_new), st.kc, st.vt)
        q0 = 0
        while q0 < n_new:
            n = int(min(n_new - q0, rng.choice([1, 1, 2, 5, 16, 40])))
            q = st.q[:, q0:q0 + n].contiguous()
            k = st.k_new[:, q0:q0 + n].contiguous()
            v = st.v_new[:, q0:q0 + n].contiguous()
            out = torch.empty_like(q)
            mass = torch.empty((cfg.n_agents, n, cfg.n_q_heads, S1), dtype=torch.float32, device=st.device)
            ws = torch.empty(max(B.decode_workspace_bytes(st.pool, st.plan, n), 256), dtype=torch.uint8,
                             device=st.device)
            ws.fill_(0xFF)
            B.segmented_decode_step(st.pool, st.plan, q0, q, k, v, st.kc, st.vt, out, ws, mass_out=mass)
            torch.cuda.synchronize()
            check_out(cfg, step_mod._to_host(out).astype(np.float64), ref_out[:, q0:q0 + n])
            m = mass.cpu().numpy().astype(np.float64)
            check_mass(cfg, m, ref_mass[:, q0:q0 + n])
            np.testing.assert_allclose(m.sum(-1), 1.0, atol=1e-4 if dtype == I.BF16 else 2e-5)
            assert m.min() >= -1e-6
            q0 += n
        # clustering scores and decisions on a prefill over the same plan, random spans
        st.ws.fill_(0xFF)
        st.gather()
        st.attention()
        cuts = np.unique(np.concatenate([[0, n_new], rng.integers(0, n_new + 1, size=int(rng.integers(0, 5)))]))
        cuts = cuts.astype(np.int32)
        tol = 1e-2 if dtype == I.BF16 else 1e-5
        for per_key in (False, True):
            score = torch.full((cfg.n_agents, len(cuts) - 1, S1), 7.0, dtype=torch.float32, device=st.device)
            assign = torch.full((cfg.n_agents, len(cuts) - 1), -7, dtype=torch.int32, device=st.device)
            thr = float(rng.choice([0.0, 0.05, 0.3]))
            B.segment_cluster_assign(st.pool, st.plan, st.ws, cuts, score, assign, per_key=per_key, threshold=thr)
            torch.cuda.synchronize()
            got, got_a = score.cpu().numpy().astype(np.float64), assign.cpu().numpy()
            for b in range(cfg.n_agents):
                lens = [int(w.lens[g]) for g in w.agent_sel(b)]
                ref = oracle.cluster_scores(ref_mass[b], lens, cuts, per_key)
                colt = np.full(ref.shape[1], tol)       # the new tokens' own bucket stays a mass
                if per_key:
                    for s_, l_ in enumerate(lens):
                        colt[s_] = tol / max(l_, 1)
                assert (np.abs(got[b][:, :ref.shape[1]] - ref) <= colt[None, :]).all()
                mine = oracle.cluster_assign(score[b].cpu().numpy(), lens, np.float32(thr))
                assert np.array_equal(got_a[b], mine)
        del st


@pytest.mark.parametrize("seed", seeds(404))
def test_random_steps_with_values_left_in_the_pool(step_mod, seed):
    """en_plan_values_from_pool on random shapes: the same bits as the gathered form (which the sweeps
    above hold against the oracle), whatever the segments' lengths, the tail of the last tile, the
    number of agents and splits, and whether the queries were prepared in the gather launch."""
    import torch
    rng = np.random.default_rng(seed)
    done = 0
    while done < 100:
        hkv = int(rng.choice([1, 2, 4]))
        r = int(rng.choice([1, 2, 3, 4, 7]))
        n_new = int(rng.choice([9, 17, 33, 64, 70, 129, 200]))
        if r * n_new <= 32:
            continue                  # such a step runs in the decode kernel, which reads gathered values
        cap = int(rng.choice([9, 33, 64, 96, 130]))
        len_lo = int(rng.integers(0, cap + 1))
        len_hi = int(rng.integers(len_lo, cap + 1))
        n_groups = int(rng.integers(2, 40))
        n_sel = int(rng.integers(0, n_groups + 1))
        n_agents = int(rng.choice([1, 1, 2, 3, 6]))
        splits = rng.choice([None, 1, 2, 3, 5, 9])
        splits = None if splits is None else int(splits)
        prepared = bool(rng.random() < 0.7)
        d = int(rng.choice([64, 128]))
        cfg = I.Config(f"vsweep{seed}-{done}", seed * 1000 + done, I.BF16, n_agents, hkv * r, hkv, d, n_groups, cap,
                       len_lo, len_hi, n_sel, n_new, 1e4 if d == 64 else 5e5, act_scale=float(rng.choice([1.0, 0.3])),
                       planted=bool(rng.random() < 0.2 and n_sel > 0))
        announce(f"values from the pool sweep {cfg} splits={splits} prepared={prepared}")
        w = I.make_workload(cfg)
        a = step_mod.PlanningStep(w, n_splits=splits, prepared=prepared, values_from_pool=True)
        b = step_mod.PlanningStep(w, n_splits=splits, prepared=prepared)
        a.vt.view(torch.int16).fill_(0x7fc0)
        for st in (a, b):
            st.ws.fill_(0xFF)
            st.run()
        torch.cuda.synchronize()
        assert torch.equal(a.out.view(torch.int16), b.out.view(torch.int16))
        assert torch.equal(a.mass.view(torch.int32), b.mass.view(torch.int32))
        assert np.array_equal(a.mass_red_host(), b.mass_red_host())
        assert np.isfinite(a.out_host()).all()
        del a, b
        done += 1
