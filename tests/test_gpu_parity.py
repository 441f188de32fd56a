"""Parity of the HIP path (through the C ABI) with the float64 CPU oracle on the
same seeded inputs. Needs a real MI355X: every test is marked gpu.

Tolerances (per the benchmark contract):
  fp32 path : |d| <= 1e-5 * max(|ref|, max|ref row|) for outputs,
              |d| <= 1e-5 * max(ref, 1e-3) for masses
  bf16 path : outputs 2e-2 absolute, masses 1e-2 absolute
  integers (plan offsets, gathered V bits, padding) : exact
"""
import sys

import numpy as np
import pytest

from paper_2510_18546_amd import inputs as I

pytestmark = pytest.mark.gpu


def announce(msg):
    sys.__stderr__.write(f"[gpu-case] {msg}\n")
    sys.__stderr__.flush()


@pytest.fixture(scope="module")
def step_mod():
    import torch
    assert torch.cuda.is_available(), "gpu tests need a GPU"
    from paper_2510_18546_amd import step
    return step


def oracle_full(O, w, rows=None):
    return O.attention(w.k_pool, w.v_pool, w.lens, w.sel, w.sel_ptr, w.q, w.k_new, w.v_new,
                       w.cfg.rope_base, rows=rows)


def check_out(cfg, got, ref):
    if cfg.dtype == I.F32:
        scale = np.maximum(np.abs(ref), np.abs(ref).max(axis=-1, keepdims=True))
        bad = np.abs(got - ref) > 1e-5 * scale + 1e-30
        assert not bad.any(), f"fp32 out: max rel {np.max(np.abs(got - ref) / scale):.3e}"
    else:
        err = np.abs(got - ref).max()
        assert err <= 2e-2, f"bf16 out: max abs err {err:.3e}"


def check_mass(cfg, got, ref):
    if cfg.dtype == I.F32:
        bad = np.abs(got - ref) > 1e-5 * np.maximum(ref, 1e-3)
        assert not bad.any(), f"fp32 mass: max err {np.abs(got - ref).max():.3e}"
    else:
        err = np.abs(got - ref).max()
        assert err <= 1e-2, f"bf16 mass: max abs err {err:.3e}"


def run_case(step_mod, O, cfg, n_splits=None, sel_lists=None, rows=None, name=""):
    announce(f"{name or cfg.name}: dtype={cfg.dtype} B={cfg.n_agents} Hq={cfg.n_q_heads} "
             f"Hkv={cfg.n_kv_heads} D={cfg.head_dim} G={cfg.n_groups}x{cfg.capacity} "
             f"S={cfg.n_sel} Nq={cfg.n_new} seed={cfg.seed} splits={n_splits}")
    import torch
    w = I.make_workload(cfg, sel_lists=sel_lists)
    st = step_mod.PlanningStep(w, n_splits=n_splits)
    # plan integers, bit-exact
    for b in range(cfg.n_agents):
        assert np.array_equal(st.plan.offsets(b), O.plan(w.lens, w.agent_sel(b)))
    st.run()
    torch.cuda.synchronize()
    out, mass, red = st.out_host(), st.mass_host(), st.mass_red_host()
    assert np.isfinite(out).all() and np.isfinite(mass).all() and np.isfinite(red).all()
    if rows is None:
        ref_out, ref_mass = oracle_full(O, w)
        check_out(cfg, out, ref_out)
        check_mass(cfg, mass, ref_mass)
        ref_red, red_agents = O.reduce_mass(ref_mass), np.arange(cfg.n_agents)
    else:
        ref_out, ref_mass = oracle_full(O, w, rows=rows)
        sel_out = np.stack([out[b, i, h] for b, i, h in rows])
        sel_mass = np.stack([mass[b, i, h] for b, i, h in rows])
        check_out(cfg, sel_out, ref_out)
        check_mass(cfg, sel_mass, ref_mass)
        # agents of which `rows` holds every (query, head) pair: their reduced masses have a reference too
        full = [b for b in np.unique(rows[:, 0])
                if len({(i, h) for bb, i, h in rows if bb == b}) == cfg.n_new * cfg.n_q_heads]
        red_agents = np.array(full, dtype=np.int64)
        ref_red = np.stack([ref_mass[rows[:, 0] == b].sum(axis=0) for b in full]) if full else None
    # properties that hold at any size
    # every block of keys gives the same total to the row's sum and to its buckets, whatever the
    # rounding of the probabilities: the masses of a row add up to 1 to fp32 rounding, none is negative
    np.testing.assert_allclose(mass.sum(-1), 1.0, atol=1e-4 if cfg.dtype == I.BF16 else 2e-5)
    assert mass.min() >= -1e-6, f"negative mass {mass.min():.3e}"
    np.testing.assert_allclose(red, mass.sum(axis=(1, 2)), rtol=1e-4, atol=1e-3)
    if ref_red is not None:
        # Reduced masses [B, S+1]: a bucket is a sum of Nq * Hq masses whose errors (roundings of K, Q and P
        # to bf16; fp32 sums) have no common sign, so the sum's error grows like the square root of
        # their number: the per-mass tolerance times sqrt(Nq * Hq). A dropped head, query block or
        # split is off by the mass it held and fails this.
        # (fp32: the per-mass bound is relative, 1e-5 of the mass, and so is the sum's.)
        # Where many rows lean on the same keys (the planted variant: one component shared by all queries
        # and by a segment's keys) the second rounding of the rotated keys and of the prepared queries to
        # bf16 (2^-9 relative) moves their masses the same way: a relative term of 1e-3 of the bucket's
        # mass on top (a random sweep found 6e-4 with two planted segments sharing the mass).
        n_terms = cfg.n_new * cfg.n_q_heads
        if cfg.dtype == I.BF16:
            tol = 1e-2 * np.sqrt(n_terms) + 1e-3 * ref_red
            err = np.abs(red[red_agents] - ref_red)
        else:
            tol = 1e-5 * np.ones_like(ref_red)
            err = np.abs(red[red_agents] - ref_red) / np.maximum(ref_red, 1.0)
        worst = np.unravel_index(np.argmax(err - tol), err.shape)
        announce(f"{name or cfg.name}: reduced masses of {len(red_agents)} agents, max |err| {err.max():.3e} "
                 f"(closest to its tolerance: {err[worst]:.3e} of {tol[worst]:.3e})")
        assert (err <= tol).all(), f"reduced mass: abs err {err[worst]:.3e} > {tol[worst]:.3e}"
    return st, w, out, mass


def small(name, seed, dtype=I.BF16, **kw):
    base = dict(name=name, seed=seed, dtype=dtype, n_agents=1, n_q_heads=8, n_kv_heads=2,
                head_dim=128, n_groups=12, capacity=96, len_lo=20, len_hi=96, n_sel=5, n_new=70,
                rope_base=500000.0)
    base.update(kw)
    return I.Config(**base)


# ---------------------------------------------------------------------------
# fp32 path
# ---------------------------------------------------------------------------
def test_c0_fp32(step_mod, oracle):
    run_case(step_mod, oracle, I.CONFIGS["c0"])


@pytest.mark.parametrize("splits", [1, 2, 3])
def test_fp32_ragged_splits(step_mod, oracle, splits):
    cfg = small("f32-ragged", 100 + splits, dtype=I.F32, head_dim=64, n_q_heads=4, n_kv_heads=2,
                len_lo=0, len_hi=96, n_sel=6, n_new=37, n_agents=2, rope_base=1e4)
    run_case(step_mod, oracle, cfg, n_splits=splits)


def test_fp32_d128_no_selection(step_mod, oracle):
    cfg = small("f32-S0", 110, dtype=I.F32, n_sel=0, n_new=33, n_q_heads=2, n_kv_heads=2)
    run_case(step_mod, oracle, cfg)


def test_fp32_single_query(step_mod, oracle):
    cfg = small("f32-decode", 111, dtype=I.F32, head_dim=64, n_new=1, n_agents=3, n_sel=4)
    run_case(step_mod, oracle, cfg, n_splits=2)


# ---------------------------------------------------------------------------
# bf16 matrix-core path, reduced sizes, full comparison
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("splits", [1, 2, 5])
def test_bf16_ragged_splits(step_mod, oracle, splits):
    cfg = small("bf16-ragged", 200 + splits, n_agents=2, len_lo=0, n_sel=7)
    run_case(step_mod, oracle, cfg, n_splits=splits)


@pytest.mark.parametrize("residue", range(0, 64, 7))
def test_bf16_every_tail_residue(step_mod, oracle, residue):
    """Context lengths hitting different (L_c + N_q) mod 64 and len mod 64."""
    cfg = small("bf16-residue", 300 + residue, len_lo=64 + residue, len_hi=64 + residue,
                capacity=128, n_sel=3, n_new=33 + residue)
    run_case(step_mod, oracle, cfg)


def test_bf16_aligned_segments_like_c2(step_mod, oracle):
    cfg = small("bf16-aligned", 210, n_q_heads=8, n_kv_heads=2, n_groups=10, capacity=256,
                len_lo=256, len_hi=256, n_sel=6, n_new=128)
    run_case(step_mod, oracle, cfg, n_splits=1)
    run_case(step_mod, oracle, cfg, n_splits=4)


def test_bf16_planted_mass(step_mod, oracle):
    cfg = small("bf16-planted", 220, planted=True, n_sel=6)
    st, w, out, mass = run_case(step_mod, oracle, cfg)
    s = list(w.agent_sel(0)).index(w.meta["planted_group"][0])
    assert mass[0, :, :, s].mean() > 0.5


@pytest.mark.parametrize("splits", [1, 3])
def test_bf16_reference_moves_mid_stream(step_mod, oracle, splits):
    """One key of a LATE segment gets a logit of about +80 (agent 1) or +110 (agent 0, whose
    exponential overflows to infinity against the reference chosen at the first block): the
    kernel must move the softmax reference mid-stream and rescale what it has accumulated.
    The key dominates with a wide margin, so the case is well conditioned in bf16."""
    cfg = small("bf16-reref", 225 + splits, planted=True, n_sel=6, n_new=70, n_agents=2, len_lo=40)
    announce(f"reference move, splits={splits}")
    w = I.make_workload(cfg)
    D = cfg.head_dim
    u = np.zeros(D, np.float32)
    u[3 * D // 8:D // 2] = 1.0
    u /= np.linalg.norm(u)
    alpha = np.float32((8.0 * np.sqrt(D)) ** 0.5)        # the generator's shared component
    toks = []
    for b, gamma in ((0, 14.0), (1, 10.0)):
        g = w.meta["planted_group"][b]
        t = int(w.lens[g]) - 3
        w.k_pool[g, :, t, :] = I.round_to_bf16(np.float32(gamma) * alpha * u)
        toks.append((g, t))
    import torch
    st = step_mod.PlanningStep(w, n_splits=splits)
    st.run()
    torch.cuda.synchronize()
    out, mass = st.out_host(), st.mass_host()
    assert np.isfinite(out).all() and np.isfinite(mass).all()
    ref_out, ref_mass = oracle_full(oracle, w)
    check_out(cfg, out, ref_out)
    check_mass(cfg, mass, ref_mass)
    for b, (g, t) in enumerate(toks):
        s_idx = list(w.agent_sel(b)).index(g)
        assert mass[b, :, :, s_idx].min() > 0.999
        r = cfg.n_q_heads // cfg.n_kv_heads
        for hq in range(cfg.n_q_heads):
            np.testing.assert_allclose(out[b, :, hq], np.broadcast_to(w.v_pool[g, hq // r, t], out[b, :, hq].shape),
                                       atol=2e-2)


def test_bf16_scaled_activations_like_c1(step_mod, oracle):
    cfg = small("bf16-scaled", 230, act_scale=128.0 ** -0.5, n_sel=8)
    run_case(step_mod, oracle, cfg, n_splits=2)


@pytest.mark.parametrize("hq,hkv", [(2, 2), (4, 2), (8, 1), (6, 2)])
def test_bf16_head_ratios(step_mod, oracle, hq, hkv):
    cfg = small(f"bf16-gqa{hq}:{hkv}", 240 + hq, n_q_heads=hq, n_kv_heads=hkv, n_new=45)
    run_case(step_mod, oracle, cfg, n_splits=2)


def test_bf16_head_dim_64(step_mod, oracle):
    cfg = small("bf16-d64", 250, head_dim=64, n_q_heads=4, n_kv_heads=1, rope_base=1e4)
    run_case(step_mod, oracle, cfg, n_splits=1)
    run_case(step_mod, oracle, cfg, n_splits=3)


def test_bf16_no_selection(step_mod, oracle):
    cfg = small("bf16-S0", 260, n_sel=0, n_new=100)
    run_case(step_mod, oracle, cfg)


def test_bf16_single_query_decode(step_mod, oracle):
    cfg = small("bf16-decode", 270, n_new=1, n_agents=3, n_sel=6)
    run_case(step_mod, oracle, cfg, n_splits=1)
    run_case(step_mod, oracle, cfg, n_splits=4)


@pytest.mark.parametrize("nq,hq,hkv,d", [(4, 8, 2, 128), (8, 4, 1, 128), (3, 6, 2, 64), (1, 8, 8, 128),
                                         (32, 2, 2, 128)])
def test_bf16_few_query_rows_decode_kernel(step_mod, oracle, nq, hq, hkv, d):
    """r * N_q <= 32: all rows of a KV head are columns of one wave (decode kernel),
    including its causal mask among several new tokens and ragged segments."""
    cfg = small(f"bf16-decode-nq{nq}", 500 + nq + hq, n_new=nq, n_q_heads=hq, n_kv_heads=hkv,
                head_dim=d, n_agents=2, len_lo=0, n_sel=7, rope_base=1e4 if d == 64 else 5e5)
    run_case(step_mod, oracle, cfg, n_splits=1)
    run_case(step_mod, oracle, cfg, n_splits=3)


@pytest.mark.parametrize("dtype,splits", [(I.BF16, 9), (I.BF16, 30), (I.BF16, None), (I.F32, 11),
                                          (I.BF16, 33), (I.BF16, 61), (I.F32, 45)])
def test_many_splits_are_merged_by_lane_groups(step_mod, oracle, dtype, splits):
    """More than eight KV splits (one agent decoding over a long context): the merge of the splits
    is shared by four lanes per output chunk, more than 32 by sixteen."""
    cfg = small(f"many-splits-{dtype}-{splits}", 520 + (splits or 0), dtype=dtype, n_groups=40, capacity=128,
                len_lo=90, len_hi=128, n_sel=36, n_new=3 if dtype == I.BF16 else 5,
                head_dim=128 if dtype == I.BF16 else 64)
    run_case(step_mod, oracle, cfg, n_splits=splits)


def test_bf16_decode_over_long_context(step_mod, oracle):
    """A reduced c4: 4 agents, one new token, 16 x 256 cached tokens, default splits."""
    cfg = I.Config("c4-small", 44, I.BF16, 4, 32, 8, 128, 64, 256, 256, 256, 16, 1, 500000.0)
    run_case(step_mod, oracle, cfg)


def test_bf16_agents_with_different_selections(step_mod, oracle):
    cfg = small("bf16-ragged-agents", 280, n_agents=3, len_lo=0)
    run_case(step_mod, oracle, cfg, sel_lists=[[3, 1, 7, 9, 0, 2], [], [5]], n_splits=2)


def test_bf16_tiny_segments(step_mod, oracle):
    """Many buckets inside one 64-key tile, including empty ones."""
    cfg = small("bf16-tiny-seg", 290, capacity=9, len_lo=0, len_hi=9, n_groups=40, n_sel=30, n_new=20)
    run_case(step_mod, oracle, cfg)


@pytest.mark.parametrize("nq,splits,len_hi", [(1, 1, 9), (4, 2, 9), (2, 5, 40), (3, None, 9)])
def test_bf16_two_waves_share_a_unit(step_mod, oracle, nq, splits, len_hi):
    """A step with so few (agent, KV head, split) units that two waves share each unit's tiles, each
    taking every other 32-key block and leaving partial results of its own. Segments shorter than a
    block, some empty: buckets lie wholly inside the other wave's blocks, or straddle two waves'
    blocks and two splits. Outputs, per-row masses and per-head sums against the oracle."""
    cfg = small(f"bf16-two-waves-nq{nq}-{splits}", 530 + nq, capacity=max(len_hi, 9), len_lo=0, len_hi=len_hi,
                n_groups=48, n_sel=44, n_new=nq)
    run_case(step_mod, oracle, cfg, n_splits=splits)


@pytest.mark.parametrize("dtype,n_agents", [(I.BF16, 1), (I.BF16, 9), (I.F32, 2)])
def test_more_segments_than_lanes(step_mod, oracle, dtype, n_agents):
    """More than 62 selected segments per agent: the bucket bounds no longer fit one per lane, and
    with nine agents the plan's tables no longer travel inside the gather launch's arguments."""
    cfg = small(f"many-seg-{dtype}-{n_agents}", 295 + n_agents, dtype=dtype, capacity=9, len_lo=0, len_hi=9,
                n_groups=120, n_sel=90, n_new=70, n_agents=n_agents, head_dim=128 if dtype == I.BF16 else 64)
    run_case(step_mod, oracle, cfg)
    run_case(step_mod, oracle, cfg, n_splits=3)


@pytest.mark.parametrize("dtype", [I.BF16, I.F32])
def test_more_segments_than_the_gather_stages(step_mod, oracle, dtype):
    """More than 254 selected segments: the gather no longer stages the agent's tables in LDS and
    searches them where they are."""
    cfg = small(f"very-many-seg-{dtype}", 297, dtype=dtype, capacity=5, len_lo=0, len_hi=5, n_groups=330,
                n_sel=300, n_new=33, n_agents=2, head_dim=128 if dtype == I.BF16 else 64)
    run_case(step_mod, oracle, cfg)


@pytest.mark.parametrize("dtype,n_new", [(I.BF16, 40), (I.BF16, 2), (I.F32, 5)])
def test_agent_with_fewer_tiles_than_splits(step_mod, oracle, dtype, n_new):
    """The split count follows the longest context; an agent with a short one leaves some splits
    without keys. Nothing is written for those, and nothing may be read from them (the scratch is
    filled with a NaN pattern first)."""
    import torch
    cfg = small(f"short-agent-{dtype}-{n_new}", 940 + n_new, dtype=dtype, n_agents=3, n_groups=14, capacity=128,
                len_lo=100, len_hi=128, n_sel=0, n_new=n_new, head_dim=128 if dtype == I.BF16 else 64)
    sel_lists = [[0, 1, 2, 3, 4, 5, 6, 7, 8, 9], [11], [12, 13]]
    w = I.make_workload(cfg, sel_lists=sel_lists)
    st = step_mod.PlanningStep(w, n_splits=13)
    st.ws.fill_(0xFF)
    st.run()
    torch.cuda.synchronize()
    ref_out, ref_mass = oracle_full(oracle, w)
    check_out(cfg, st.out_host(), ref_out)
    check_mass(cfg, st.mass_host(), ref_mass)
    red = st.mass_red_host()
    assert np.isfinite(red).all()
    np.testing.assert_allclose(red, oracle.reduce_mass(ref_mass), atol=1e-2 * cfg.n_new * cfg.n_q_heads)


@pytest.mark.parametrize("splits", [None, 1, 3])
def test_bf16_dominant_key_among_tiny_segments(step_mod, oracle, splits):
    """A key that carries almost all of a row's weight, inside a 32-key block in which several
    segments end, one of them exactly at the end of a KV split: the rounding of that key's
    probability must not leak into a neighbouring bucket (a negative mass) or get lost."""
    cfg = I.Config(name="tiny-planted", seed=1772, dtype=I.BF16, n_agents=3, n_q_heads=12, n_kv_heads=4,
                   head_dim=64, n_groups=26, capacity=33, len_lo=4, len_hi=5, n_sel=16, n_new=64,
                   rope_base=10000.0, planted=True)
    run_case(step_mod, oracle, cfg, n_splits=splits)


# ---------------------------------------------------------------------------
# gather_rope on its own: indices and values bit-exact, rotation to 1 bf16 ulp
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
def test_gather_rope_layout(step_mod, oracle, dtype):
    import torch
    cfg = small("gather", 400 + dtype, dtype=dtype, n_agents=2, len_lo=0, n_sel=6, n_new=19,
                head_dim=64 if dtype == I.F32 else 128)
    announce(f"gather_rope dtype={dtype}")
    w = I.make_workload(cfg)
    st = step_mod.PlanningStep(w)
    st.kc.fill_(0xFF)
    st.vt.fill_(0xFF)                    # NaN patterns: every byte must be overwritten
    st.gather()
    torch.cuda.synchronize()
    for b in range(cfg.n_agents):
        kc, v, kpad, vpad = st.context_host(b)
        rk, rv = oracle.gather_rope(w.k_pool, w.v_pool, w.lens, w.agent_sel(b), w.k_new[b],
                                    w.v_new[b], cfg.rope_base)
        assert np.array_equal(v.astype(np.float64), rv), "gathered values must be bit-exact copies"
        if dtype == I.F32:
            assert np.abs(kc - rk).max() <= 1e-6 * max(1.0, np.abs(rk).max())
        else:
            ulp = np.maximum(np.abs(rk), 2.0 ** -126) * 2.0 ** -8
            assert (np.abs(kc - rk) <= 1.01 * ulp + 1e-7).all()
        L = kc.shape[1]
        pad_to = -(-L // 64) * 64
        assert (kpad[:, :pad_to - L] == 0).all() and (vpad[:, :pad_to - L] == 0).all()


# ---------------------------------------------------------------------------
# the two forms of a step: queries prepared in the gather launch and reduced masses out of the
# attention call (what run_case and the benchmark use where the library offers it), against the
# five separate calls
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("case", ["ragged", "one-split", "d64", "c1"])
def test_prepared_step_equals_the_five_calls(step_mod, oracle, case):
    import torch
    cfg = {"ragged": small("prep-ragged", 900, n_agents=2, len_lo=0, n_sel=7),
           "one-split": small("prep-one-split", 901, n_agents=3, n_new=40),
           "d64": small("prep-d64", 902, head_dim=64, n_q_heads=4, n_kv_heads=1, n_new=45),
           "c1": I.CONFIGS["c1"]}[case]
    splits = {"ragged": 3, "one-split": 1, "d64": 2, "c1": None}[case]
    announce(f"prepared vs five calls: {cfg.name} splits={splits}")
    w = I.make_workload(cfg)
    a = step_mod.PlanningStep(w, n_splits=splits, prepared=True)
    b = step_mod.PlanningStep(w, n_splits=splits, prepared=False)
    assert a.prepared and not b.prepared
    a.mass_red.fill_(float("nan"))            # the attention launch must start the sums at zero itself
    a.run()
    b.run()
    torch.cuda.synchronize()
    # same arithmetic on the queries, wherever it is done: the same bits
    assert torch.equal(a.out.view(torch.int16), b.out.view(torch.int16))
    assert torch.equal(a.mass.view(torch.int32), b.mass.view(torch.int32))
    # reduced masses: an exact integer sum of the heads' sums against the float sum of the mass call
    ra, rb = a.mass_red_host(), b.mass_red_host()
    assert np.isfinite(ra).all()
    np.testing.assert_allclose(ra, rb, rtol=2e-6, atol=1e-5)
    # ... and a second run starts from zero again, not from the first run's sums, and gives the same
    # bits: the heads' sums are added as integers, whatever order they arrive in
    a.run()
    torch.cuda.synchronize()
    assert np.array_equal(a.mass_red_host(), ra)
    # the mass call after a prepared attention call gives the fixed-order sums
    a.masses(1)
    torch.cuda.synchronize()
    assert np.array_equal(a.mass_red_host(), rb)
    ref_out, ref_mass = oracle_full(oracle, w)
    check_out(cfg, a.out_host(), ref_out)
    check_mass(cfg, a.mass_host(), ref_mass)


def test_prepared_form_refusals(step_mod):
    from paper_2510_18546_amd import binding as B
    w32 = I.make_workload(small("prep-f32", 903, dtype=I.F32, head_dim=64, n_new=40))
    st = step_mod.PlanningStep(w32)
    assert not st.prepared
    with pytest.raises(B.EnError) as e:
        B.gather_rope_queries(st.pool, st.plan, st.k_new, st.v_new, st.q, st.kc, st.vt, st.q)
    assert e.value.code == 5
    wd = I.make_workload(small("prep-decode", 904, n_new=2))       # 4 heads per KV head x 2 rows: the decode kernel's
    sd = step_mod.PlanningStep(wd)
    assert not sd.prepared
    sd.gather()
    with pytest.raises(B.EnError) as e:
        B.segmented_prefill_attention_prepared(sd.pool, sd.plan, sd.q, sd.kc, sd.vt, sd.out, sd.ws)
    assert e.value.code == 5


# ---------------------------------------------------------------------------
# values left where they are (en_plan_values_from_pool): the attention kernel fetches the value rows
# from the pool's blocks and the new tokens through a table of row addresses. Same values into the
# same products in the same order: the same bits as the gathered form.
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("case", ["ragged", "one-split", "tail-1", "tail-37", "agents", "five-calls", "d64",
                                  "d64-five-calls", "c1", "c2", "c3"])
def test_values_from_pool_equals_the_gathered_form(step_mod, oracle, case):
    import torch
    cfg = {"ragged": small("vp-ragged", 910, n_agents=2, len_lo=0, n_sel=7),
           "one-split": small("vp-one-split", 911, n_agents=3, n_new=40),
           "tail-1": small("vp-tail-1", 912, len_lo=64, len_hi=64, capacity=64, n_sel=4, n_new=65),
           "tail-37": small("vp-tail-37", 913, len_lo=50, len_hi=50, capacity=64, n_sel=3, n_new=79),
           "agents": small("vp-agents", 914, n_agents=5, n_groups=40, len_lo=1, len_hi=30, capacity=32, n_sel=11,
                           n_new=33),
           "five-calls": small("vp-five-calls", 915, n_agents=2),
           "d64": small("vp-d64", 920, head_dim=64, n_agents=2, len_lo=0, n_sel=7, n_q_heads=4, n_kv_heads=1, n_new=77),
           "d64-five-calls": small("vp-d64-five-calls", 921, head_dim=64, n_q_heads=6, n_kv_heads=2, n_new=45),
           "c1": I.CONFIGS["c1"], "c2": I.CONFIGS["c2"], "c3": I.CONFIGS["c3"]}[case]
    splits = {"ragged": 3, "one-split": 1, "tail-1": 2, "tail-37": 1, "agents": 2, "d64": 2}.get(case)
    prepared = False if case.endswith("five-calls") else None
    announce(f"values from the pool vs gathered: {cfg.name} splits={splits} prepared={prepared}")
    w = I.make_workload(cfg)             # rows of a group beyond its length hold NaN
    a = step_mod.PlanningStep(w, n_splits=splits, prepared=prepared, values_from_pool=True)
    b = step_mod.PlanningStep(w, n_splits=splits, prepared=prepared)
    a.vt.view(torch.int16).fill_(0x7fc0)  # NaN where the gathered form would have values
    a.run()
    b.run()
    torch.cuda.synchronize()
    assert torch.equal(a.out.view(torch.int16), b.out.view(torch.int16))
    assert torch.equal(a.mass.view(torch.int32), b.mass.view(torch.int32))
    assert np.array_equal(a.mass_red_host(), b.mass_red_host())
    # the keys are gathered as ever
    for ag in range(cfg.n_agents):
        assert np.array_equal(a.context_host(ag)[0], b.context_host(ag)[0])
    # a second step on the same plan, and one after the plan goes back to gathered values
    a.out.zero_()
    a.run()
    torch.cuda.synchronize()
    assert torch.equal(a.out.view(torch.int16), b.out.view(torch.int16))
    a.plan.values_from_pool(False)
    a.out.zero_()
    a.run()
    torch.cuda.synchronize()
    assert torch.equal(a.out.view(torch.int16), b.out.view(torch.int16))
    for ag in range(cfg.n_agents):        # ... which gathers the values again
        for x, y in zip(a.context_host(ag)[:2], b.context_host(ag)[:2]):      # keys and values of the context
            assert np.array_equal(x, y)
    if case not in ("c2", "c3"):          # (their gathered form has its own full-size comparison)
        ref_out, ref_mass = oracle_full(oracle, w)
        check_out(cfg, a.out_host(), ref_out)
        check_mass(cfg, a.mass_host(), ref_mass)


def test_values_from_pool_refusals(step_mod):
    import torch
    from paper_2510_18546_amd import binding as B

    def code_of(fn):
        with pytest.raises(B.EnError) as e:
            fn()
        return e.value.code

    # fp32 pools keep their gathered values
    s32 = step_mod.PlanningStep(I.make_workload(small("vp-f32", 916, dtype=I.F32, head_dim=64, n_new=40)))
    assert code_of(lambda: s32.plan.values_from_pool(True)) == 5
    # so few rows that the attention runs in the decode kernel
    sd = step_mod.PlanningStep(I.make_workload(small("vp-decode", 918, n_new=2)))
    assert code_of(lambda: sd.plan.values_from_pool(True)) == 5
    # the flag is 0 or 1
    st = step_mod.PlanningStep(I.make_workload(small("vp-flag", 919)))
    with pytest.raises(B.EnError) as e:
        B._check(B.load().en_plan_values_from_pool(st.plan.handle, 2))
    assert e.value.code == 1
    # a change between the gather and the attention call is caught; a new gather clears it
    st.gather()
    st.plan.values_from_pool(True)
    assert code_of(lambda: st.attention()) == 1
    st.gather()
    st.attention()
    # the decode steps read gathered values
    ws = torch.empty(B.decode_workspace_bytes(st.pool, st.plan, 1), dtype=torch.uint8, device=st.device)
    assert code_of(lambda: B.segmented_decode_step(st.pool, st.plan, 0, st.q[:, :1].contiguous(),
                                                   st.k_new[:, :1].contiguous(), st.v_new[:, :1].contiguous(),
                                                   st.kc, st.vt, st.out[:, :1].contiguous(), ws)) == 5
    # the new tokens' value rows are fetched as 256-byte rows: aligned
    raw = torch.empty(st.v_new.numel() + 64, dtype=st.v_new.dtype, device=st.device)
    v_mis = raw[64:].view(st.v_new.shape)
    v_mis.copy_(st.v_new)
    assert code_of(lambda: B.gather_rope(st.pool, st.plan, st.k_new, v_mis, st.kc, st.vt)) == 1
    torch.cuda.synchronize()


# ---------------------------------------------------------------------------
# full benchmark sizes, in the launch configuration the benchmark times
# (default split choice): every output row, every mass and the reduced masses
# against the oracle
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c5"])
def test_full_size_prefill_configs(step_mod, oracle, name):
    """All rows of all agents: a wrong work decode of one workgroup slot fails."""
    run_case(step_mod, oracle, I.CONFIGS[name])


def test_full_size_c1_unscaled_and_planted(step_mod, oracle):
    cfg = I.variant(I.CONFIGS["c1"], act_scale=1.0, planted=True, name="c1-planted")
    run_case(step_mod, oracle, cfg)


def test_full_size_decode_c4(step_mod, oracle):
    """Every head of 16 of the 64 agents, spread over the launch (first, last, every fourth or
    so); the oracle gathers each of them once (16 K tokens)."""
    cfg = I.CONFIGS["c4"]
    agents = [0, 3, 7, 12, 16, 21, 25, 30, 34, 39, 43, 48, 52, 57, 61, 63]
    rows = np.array([(b, 0, h) for b in agents for h in range(cfg.n_q_heads)], dtype=np.int32)
    run_case(step_mod, oracle, cfg, rows=rows)


# ---------------------------------------------------------------------------
# boundary behaviour on the device side
# ---------------------------------------------------------------------------
def test_scored_selection_end_to_end(step_mod, oracle):
    """Retrieval form: knapsack over scores -> plan -> gather -> attention, checked
    against the oracle run on the oracle's own selection."""
    import torch
    from paper_2510_18546_amd import binding as B
    cfg = small("scored", 600, n_groups=20, n_sel=0)
    announce("segment_select_scored end to end")
    w = I.make_workload(cfg)
    rng = np.random.default_rng(1)
    p = rng.random(cfg.n_groups).astype(np.float32)
    budget = int(w.lens.sum()) // 3
    want = oracle.knapsack(p, w.lens, 0.4, budget)
    w.sel = np.asarray(want, np.int32)
    w.sel_ptr = np.array([0, len(want)], np.int32)
    st = step_mod.PlanningStep(w, max_ctx=cfg.n_groups * cfg.capacity + cfg.n_new)
    got, plan = B.segment_select_scored(st.pool, p, 0.4, budget, cfg.n_new)
    assert got.tolist() == want
    assert np.array_equal(plan.offsets(0), oracle.plan(w.lens, want))
    st.plan.close()
    st.plan = plan
    st.info = plan.info
    st.run()
    torch.cuda.synchronize()
    ref_out, ref_mass = oracle_full(oracle, w)
    check_out(cfg, st.out_host(), ref_out)
    check_mass(cfg, st.mass_host(), ref_mass)


def test_device_side_errors_and_timing_aid(step_mod):
    import torch
    from paper_2510_18546_amd import binding as B
    cfg = small("errors", 610)
    announce("error paths and timing aid")
    w = I.make_workload(cfg)
    st = step_mod.PlanningStep(w, n_splits=2)
    st.gather()
    small_ws = torch.empty(256, dtype=torch.uint8, device=st.device)
    with pytest.raises(B.EnError) as e:
        B.segmented_prefill_attention(st.pool, st.plan, st.q, st.kc, st.vt, st.out, small_ws)
    assert e.value.code == 4                                  # workspace too small
    with pytest.raises(B.EnError) as e:
        B.segmented_prefill_attention(st.pool, st.plan, st.q, st.kc, st.vt, st.out, None)
    assert e.value.code == 1                                  # splits need a workspace
    other = step_mod.PlanningStep(w)
    with pytest.raises(B.EnError) as e:
        B.gather_rope(other.pool, st.plan, st.k_new, st.v_new, st.kc, st.vt)
    assert e.value.code == 1                                  # plan of another pool
    # the timing aid belongs to a pool: calls on another pool leave no record in this one
    B.timing_enable(st.pool, 3)
    other.gather()
    other.attention()
    for _ in range(5):
        st.attention()
    torch.cuda.synchronize()
    ms = B.timing_collect(st.pool, 8)
    assert len(B.timing_collect(other.pool, 8)) == 0
    B.timing_enable(st.pool, 0)
    assert len(ms) == 3 and (ms > 0).all() and (ms < 50).all()


def test_pool_destroyed_before_its_plan(step_mod):
    """Handles released in the wrong order (as a garbage collector may do): the plan, which holds a
    device block by now, is still destroyed cleanly."""
    import torch
    from paper_2510_18546_amd import binding as B
    announce("destroy order: pool first, then a plan that was used on the device")
    w = I.make_workload(small("destroy-order", 930))
    st = step_mod.PlanningStep(w)
    st.run()
    torch.cuda.synchronize()
    lib = B.load()
    plan_handle, pool_handle = st.plan.handle, st.pool.handle
    st.plan.handle = None                 # the wrappers must not release them again
    st.pool.handle = None
    assert lib.kv_pool_destroy(pool_handle) == 0
    assert lib.en_plan_destroy(plan_handle) == 0


def test_no_workspace_single_split(step_mod, oracle):
    """n_splits == 1 and no masses wanted: the attention call works without scratch."""
    import torch
    from paper_2510_18546_amd import binding as B
    cfg = small("no-ws", 620)
    announce("attention without workspace")
    w = I.make_workload(cfg)
    st = step_mod.PlanningStep(w, n_splits=1)
    st.gather()
    B.segmented_prefill_attention(st.pool, st.plan, st.q, st.kc, st.vt, st.out, None)
    torch.cuda.synchronize()
    ref_out, _ = oracle_full(oracle, w)
    check_out(cfg, st.out_host(), ref_out)


def test_plan_reuse_and_repeatability(step_mod, oracle):
    """The same plan run twice gives bit-identical results (no state leaks through the scratch);
    a second plan on the same pool reuses the descriptor block."""
    import torch
    cfg = small("repeat", 630, n_agents=2)
    announce("repeatability")
    w = I.make_workload(cfg)
    st = step_mod.PlanningStep(w, n_splits=3)
    st.run()
    torch.cuda.synchronize()
    o1, m1, r1 = st.out_host(), st.mass_host(), st.mass_red_host()
    st.ws.fill_(0xFF)
    st.select(3)
    st.run()
    torch.cuda.synchronize()
    assert np.array_equal(o1, st.out_host()) and np.array_equal(m1, st.mass_host())
    assert np.array_equal(r1, st.mass_red_host())


# ---------------------------------------------------------------------------
# append (next row of the scope table): cache lifecycle
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [I.BF16, I.F32])
def test_append_then_attend(step_mod, oracle, dtype):
    """kv_pool_append through the C ABI: the pool arrays equal the oracle's append bit for bit
    (every group, NaN poison included); a plan made afterwards attends over the appended group."""
    import torch
    from paper_2510_18546_amd import binding as B
    cfg = small("append", 640, dtype=dtype, n_groups=10, capacity=96, len_lo=10, len_hi=60, n_sel=4,
                n_new=40, head_dim=128 if dtype == I.BF16 else 64, rope_base=5e5 if dtype == I.BF16 else 1e4)
    announce(f"kv_pool_append dtype={dtype}")
    w = I.make_workload(cfg)
    st = step_mod.PlanningStep(w, max_ctx=5 * cfg.capacity + cfg.n_new)
    g = next(i for i in range(cfg.n_groups) if i not in set(w.agent_sel(0).tolist()))
    # the group is emptied, then receives the step's new tokens in two pieces
    B.kv_pool_set_len(st.pool, g, 0)
    lens = w.lens.copy()
    lens[g] = 0
    kp, vp = w.k_pool, w.v_pool
    for lo, hi in ((0, 13), (13, 40)):
        B.kv_pool_append(st.pool, g, st.k_new[0, lo:hi].contiguous(), st.v_new[0, lo:hi].contiguous())
        kp, vp, lens = oracle.append(kp, vp, lens, g, w.k_new[0, lo:hi], w.v_new[0, lo:hi])
    torch.cuda.synchronize()

    def bits(t):
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy().view(np.uint32)

    def ref_bits(x):
        return I.bf16_bits(x) if dtype == I.BF16 else np.ascontiguousarray(x, np.float32).view(np.uint32)
    assert np.array_equal(bits(st.k_pool), ref_bits(kp))
    assert np.array_equal(bits(st.v_pool), ref_bits(vp))
    # attend over [old selection, the appended group]
    sel = np.concatenate([w.agent_sel(0), [g]]).astype(np.int32)
    w.k_pool, w.v_pool, w.lens = kp, vp, lens
    w.sel, w.sel_ptr = sel, np.array([0, len(sel)], np.int32)
    st.select()
    assert np.array_equal(st.plan.offsets(0), oracle.plan(lens, sel))
    st.run()
    torch.cuda.synchronize()
    ref_out, ref_mass = oracle_full(oracle, w)
    check_out(cfg, st.out_host(), ref_out)
    check_mass(cfg, st.mass_host(), ref_mass)
    with pytest.raises(B.EnError) as e:
        B.kv_pool_append(st.pool, g, st.k_new[0].contiguous(), st.v_new[0].contiguous(), 57)   # 40 + 57 > 96
    assert e.value.code == 4


# ---------------------------------------------------------------------------
# clustering signal and decision (next row of the scope table)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,splits", [(I.BF16, 1), (I.BF16, 3), (I.F32, 2)])
def test_cluster_scores_and_assignment(step_mod, oracle, dtype, splits):
    """segment_cluster_assign through the C ABI against the oracle: scores to the mass tolerance;
    the decision compared where it is decided in the same precision (recomputed from the GPU's own
    scores, bit for bit) and against the oracle's where the margin exceeds the tolerance."""
    import torch
    from paper_2510_18546_amd import binding as B
    cfg = small("cluster", 650 + splits, dtype=dtype, planted=True, n_agents=2, n_sel=5, n_new=48,
                head_dim=128 if dtype == I.BF16 else 64, rope_base=5e5 if dtype == I.BF16 else 1e4,
                n_q_heads=8 if dtype == I.BF16 else 4)
    announce(f"segment_cluster_assign dtype={dtype} splits={splits}")
    w = I.make_workload(cfg)
    st = step_mod.PlanningStep(w, n_splits=splits)
    st.gather()
    st.attention()
    spans = np.array([0, 5, 6, 30, 48], np.int32)
    n_obj = len(spans) - 1
    S1 = st.info.max_segments + 1
    tol = 1e-2 if dtype == I.BF16 else 1e-5
    _, ref_mass = oracle_full(oracle, w)
    for per_key in (False, True):
        score = torch.full((cfg.n_agents, n_obj, S1), 7.0, dtype=torch.float32, device=st.device)
        assign = torch.full((cfg.n_agents, n_obj), -7, dtype=torch.int32, device=st.device)
        thr = 0.25 if not per_key else 0.004
        B.segment_cluster_assign(st.pool, st.plan, st.ws, spans, score, assign, per_key=per_key, threshold=thr)
        torch.cuda.synchronize()
        got, got_a = score.cpu().numpy().astype(np.float64), assign.cpu().numpy()
        for b in range(cfg.n_agents):
            lens = [int(w.lens[g]) for g in w.agent_sel(b)]
            ref = oracle.cluster_scores(ref_mass[b], lens, spans, per_key)
            assert np.abs(got[b] - ref).max() <= tol * (1.0 if not per_key else 1.0 / min(lens))
            # the same decision rule applied to the GPU's own fp32 scores
            mine = oracle.cluster_assign(score[b].cpu().numpy(), lens, np.float32(thr))
            assert np.array_equal(got_a[b], mine)
            ref_a = oracle.cluster_assign(ref, lens, thr)
            for o in range(n_obj):
                top = np.sort(ref[o, :len(lens)])[::-1]
                clear = (top[0] - top[1] > 4 * tol) and abs(top[0] - thr) > 4 * tol
                if not per_key and clear:
                    assert got_a[b, o] == ref_a[o]
        if not per_key:
            # what the objects join is a planted segment (the pool is shared: an agent may have
            # selected the other agent's planted group as well)
            for b in range(cfg.n_agents):
                joined = {int(w.agent_sel(b)[p]) for p in got_a[b]}
                assert -1 not in got_a[b] and joined <= set(w.meta["planted_group"])
    # layer averaging: two accumulated calls, decision on half the sum = the single-call decision
    score2 = torch.zeros((cfg.n_agents, n_obj, S1), dtype=torch.float32, device=st.device)
    assign2 = torch.empty((cfg.n_agents, n_obj), dtype=torch.int32, device=st.device)
    B.segment_cluster_assign(st.pool, st.plan, st.ws, spans, score2, None, accumulate=True)
    B.segment_cluster_assign(st.pool, st.plan, st.ws, spans, score2, assign2, accumulate=True, scale=0.5,
                             threshold=0.25)
    score1 = torch.empty_like(score2)
    assign1 = torch.empty_like(assign2)
    B.segment_cluster_assign(st.pool, st.plan, st.ws, spans, score1, assign1, threshold=0.25)
    torch.cuda.synchronize()
    assert torch.equal(score2, 2 * score1) and torch.equal(assign1, assign2)


# ---------------------------------------------------------------------------
# decode steps over a context gathered once (next row of the scope table)
# ---------------------------------------------------------------------------
def _decode_case(step_mod, dtype, seed, n_new=11):
    cfg = small("decode-loop", seed, dtype=dtype, n_agents=2, n_sel=5, n_new=n_new, len_lo=10,
                n_q_heads=8, n_kv_heads=2, head_dim=128 if dtype == I.BF16 else 64,
                rope_base=5e5 if dtype == I.BF16 else 1e4)
    w = I.make_workload(cfg)
    return cfg, w, step_mod.PlanningStep(w)


@pytest.mark.parametrize("dtype", [I.BF16, I.F32])
def test_decode_steps_equal_prefill_rows(step_mod, oracle, dtype):
    """The context is gathered once with placeholder rows for the new tokens; steps of 1, 1, 3, 1 and 5
    tokens then append their keys/values and attend. Outputs and masses of every step equal the rows
    of one prefill over all tokens (the oracle); the context ends up as a plain gather makes it."""
    import torch
    from paper_2510_18546_amd import binding as B
    cfg, w, st = _decode_case(step_mod, dtype, 660)
    announce(f"segmented_decode_step dtype={dtype}")
    ref_out, ref_mass = oracle_full(oracle, w)
    B.gather_rope(st.pool, st.plan, torch.zeros_like(st.k_new), torch.zeros_like(st.v_new), st.kc, st.vt)
    S1 = st.info.max_segments + 1
    q0 = 0
    for n in (1, 1, 3, 1, 5):
        q = st.q[:, q0:q0 + n].contiguous()
        k = st.k_new[:, q0:q0 + n].contiguous()
        v = st.v_new[:, q0:q0 + n].contiguous()
        out = torch.empty_like(q)
        mass = torch.empty((cfg.n_agents, n, cfg.n_q_heads, S1), dtype=torch.float32, device=st.device)
        ws = torch.empty(max(B.decode_workspace_bytes(st.pool, st.plan, n), 256), dtype=torch.uint8,
                         device=st.device)
        B.segmented_decode_step(st.pool, st.plan, q0, q, k, v, st.kc, st.vt, out, ws, mass_out=mass)
        torch.cuda.synchronize()
        got = step_mod._to_host(out).astype(np.float64)
        check_out(cfg, got, ref_out[:, q0:q0 + n])
        check_mass(cfg, mass.cpu().numpy().astype(np.float64), ref_mass[:, q0:q0 + n])
        q0 += n
    # the context now holds what a plain gather with the real rows writes
    kc_steps, vt_steps = st.kc.clone(), st.vt.clone()
    st.gather()
    torch.cuda.synchronize()
    assert torch.equal(vt_steps, st.vt)                          # values are copies: bit for bit
    if dtype == I.F32:
        a, b_ = kc_steps.view(torch.float32), st.kc.view(torch.float32)
    else:
        a, b_ = kc_steps.view(torch.bfloat16).float(), st.kc.view(torch.bfloat16).float()
    assert (a - b_).abs().max().item() <= (2e-6 if dtype == I.F32 else 4e-2)   # rotated keys: rounding order only
    with pytest.raises(B.EnError) as e:
        B.segmented_decode_step(st.pool, st.plan, 9, st.q[:, :3].contiguous(), st.k_new[:, :3].contiguous(),
                                st.v_new[:, :3].contiguous(), st.kc, st.vt, torch.empty_like(st.q[:, :3]), None)
    assert e.value.code == 2


@pytest.mark.parametrize("name,n_new", [("c2", 6), ("c3", 3)])
def test_full_size_decode_steps(step_mod, oracle, name, n_new):
    """One-token steps over full-size contexts (c2: one agent, 8192 cached tokens, as many KV splits as
    the plan allows, the step's K/V written by the attention kernel itself; c3: 16 agents, ragged
    segments): every step's output and masses against the oracle's rows of the same prefill."""
    import torch
    from paper_2510_18546_amd import binding as B
    cfg = I.variant(I.CONFIGS[name], name=f"{name}-decode", n_new=n_new)
    w = I.make_workload(cfg)
    st = step_mod.PlanningStep(w)
    announce(f"full-size decode steps {name}: {n_new} tokens")
    ref_out, ref_mass = oracle_full(oracle, w)
    B.gather_rope(st.pool, st.plan, torch.zeros_like(st.k_new), torch.zeros_like(st.v_new), st.kc, st.vt)
    S1 = st.info.max_segments + 1
    ws = torch.empty(max(B.decode_workspace_bytes(st.pool, st.plan, 1), 256), dtype=torch.uint8, device=st.device)
    ws.fill_(0xFF)
    for i in range(n_new):
        q, k, v = (t[:, i:i + 1].contiguous() for t in (st.q, st.k_new, st.v_new))
        out = torch.empty_like(q)
        mass = torch.empty((cfg.n_agents, 1, cfg.n_q_heads, S1), dtype=torch.float32, device=st.device)
        B.segmented_decode_step(st.pool, st.plan, i, q, k, v, st.kc, st.vt, out, ws, mass_out=mass)
        torch.cuda.synchronize()
        check_out(cfg, step_mod._to_host(out).astype(np.float64), ref_out[:, i:i + 1])
        got_mass = mass.cpu().numpy().astype(np.float64)
        check_mass(cfg, got_mass, ref_mass[:, i:i + 1])
        np.testing.assert_allclose(got_mass.sum(-1), 1.0, atol=1e-4)


def test_decode_steps_in_a_graph(step_mod, oracle):
    """Eight one-token steps captured into one HIP graph (the steps allocate nothing and only launch
    kernels); three replays, each after an eager re-gather, reproduce the eager results bit for bit."""
    import torch
    from paper_2510_18546_amd import binding as B
    cfg, w, st = _decode_case(step_mod, I.BF16, 670, n_new=8)
    announce("segmented_decode_step in a graph")
    zk, zv = torch.zeros_like(st.k_new), torch.zeros_like(st.v_new)
    qs = [st.q[:, i:i + 1].contiguous() for i in range(cfg.n_new)]
    ks = [st.k_new[:, i:i + 1].contiguous() for i in range(cfg.n_new)]
    vs = [st.v_new[:, i:i + 1].contiguous() for i in range(cfg.n_new)]
    outs = [torch.empty_like(q) for q in qs]
    ws = torch.empty(max(B.decode_workspace_bytes(st.pool, st.plan, 1), 256), dtype=torch.uint8, device=st.device)

    def steps():
        for i in range(cfg.n_new):
            B.segmented_decode_step(st.pool, st.plan, i, qs[i], ks[i], vs[i], st.kc, st.vt, outs[i], ws)
    B.gather_rope(st.pool, st.plan, zk, zv, st.kc, st.vt)
    steps()
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    ref_out, _ = oracle_full(oracle, w)
    check_out(cfg, np.concatenate([step_mod._to_host(o) for o in eager], 1).astype(np.float64), ref_out)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            steps()
    torch.cuda.synchronize()
    for _ in range(3):
        for o in outs:
            o.fill_(7.0)
        B.gather_rope(st.pool, st.plan, zk, zv, st.kc, st.vt)     # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, e in zip(outs, eager):
            assert torch.equal(o, e)


@pytest.mark.parametrize("case", ["one-split", "three-splits", "values-from-pool"])
def test_planning_step_in_a_graph(step_mod, case):
    """The launches of a planning step (gather with the queries prepared, attention with the reduced
    masses, per-row masses) captured into one HIP graph: they allocate nothing once the plan has been
    used, and nothing in them clears memory with a memset node (the accumulators of the reduced masses
    are set to zero by the kernels themselves). Three replays, with eager work on the same buffers
    between them, reproduce the eager step bit for bit."""
    import torch
    cfg = small(f"graph-{case}", 930, n_agents=3 if case == "one-split" else 2, len_lo=0, n_sel=7)
    splits = {"one-split": 1, "three-splits": 3, "values-from-pool": 2}[case]
    announce(f"planning step in a graph: {cfg.name} splits={splits}")
    w = I.make_workload(cfg)
    st = step_mod.PlanningStep(w, n_splits=splits, values_from_pool=case == "values-from-pool")
    assert st.prepared
    st.run()                                  # first use: the plan's descriptors go to the device here
    torch.cuda.synchronize()
    eager = [t.clone() for t in (st.out, st.mass, st.mass_red)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            st.run()
    torch.cuda.synchronize()
    for _ in range(3):
        for t in (st.out, st.mass, st.mass_red):
            t.fill_(7.0)
        st.ws.fill_(0xFF)                     # eager work between the replays, on the step's own scratch
        st.kc.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, e in zip((st.out, st.mass, st.mass_red), eager):
            assert torch.equal(t.view(torch.int32) if t.dtype == torch.float32 else t.view(torch.int16),
                               e.view(torch.int32) if e.dtype == torch.float32 else e.view(torch.int16))
