"""Residency tier on the GPU, through the C ABI: the blocks a fetch loads are bit-exact copies of the
store; a planning step over fetched slots equals, bit for bit, the same step over a pool that holds
every group, and the oracle to the usual tolerance; loads that run beside the previous step's kernels
(fence + prefetch) disturb nothing. Needs a real MI355X."""
import sys

import numpy as np
import pytest

from oracle.residency import Residency
from paper_2510_18546_amd import inputs as I

pytestmark = pytest.mark.gpu


def announce(msg):
    sys.__stderr__.write(f"[gpu-case] {msg}\n")
    sys.__stderr__.flush()


@pytest.fixture(scope="module")
def mods():
    import torch
    assert torch.cuda.is_available(), "gpu tests need a GPU"
    from paper_2510_18546_amd import binding, step
    return binding, step


def host_blocks(w, bf16):
    """Per group, (K, V) as CPU tensors [Hkv, len, D] in the storage type (unused rows cut off)."""
    import torch
    out = []
    for g in range(w.cfg.n_groups):
        n = int(w.lens[g])
        pair = []
        for a in (w.k_pool, w.v_pool):
            x = np.ascontiguousarray(a[g, :, :n, :])
            if bf16:
                pair.append(torch.from_numpy(I.bf16_bits(x).view(np.int16)).view(torch.bfloat16))
            else:
                pair.append(torch.from_numpy(x.astype(np.float32)))
        out.append(tuple(pair))
    return out


def make_tier(B, cfg, w, n_slots, max_ctx):
    import torch
    dt = torch.bfloat16 if cfg.dtype == I.BF16 else torch.float32
    shape = (n_slots, cfg.n_kv_heads, cfg.capacity, cfg.head_dim)
    # slots start as NaN: a row that is read without having been loaded shows up in the result
    k_slots = torch.full(shape, float("nan"), dtype=dt, device="cuda:0")
    v_slots = torch.full(shape, float("nan"), dtype=dt, device="cuda:0")
    tier = B.kv_tier_create(k_slots, v_slots, cfg.n_groups, cfg.n_q_heads, cfg.rope_base, max_ctx)
    blocks = host_blocks(w, cfg.dtype == I.BF16)
    for g, (k, v) in enumerate(blocks):
        B.kv_tier_put(tier, g, k, v)
    return tier, blocks


def bits(t):
    import torch
    return t.contiguous().view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu().numpy()


@pytest.mark.parametrize("base,lo", [("c1", 1), ("c0", 0)])
def test_fetched_blocks_are_bit_exact_copies(mods, base, lo):
    import torch
    B, _ = mods
    cfg = I.variant(I.CONFIGS[base], n_groups=12, len_lo=lo, seed=21, n_sel=4, fixed_sel=None)
    w = I.make_workload(cfg)
    n_slots = 5
    announce(f"tier copies: {base} dtype={cfg.dtype} G=12 slots={n_slots} C={cfg.capacity} len>={lo}")
    tier, blocks = make_tier(B, cfg, w, n_slots, 4096)
    ref = Residency(n_slots)
    rng = np.random.default_rng(4)
    for step in range(12):
        groups = rng.permutation(cfg.n_groups)[:int(rng.integers(1, n_slots + 1))]
        slots = B.kv_tier_fetch(tier, groups)
        assert slots.tolist() == ref.fetch(groups.tolist())[0]
        torch.cuda.synchronize()
        for g, s in zip(groups, slots):
            n = int(w.lens[g])
            for dev, host in ((tier.pool.k, blocks[g][0]), (tier.pool.v, blocks[g][1])):
                assert np.array_equal(bits(dev[s, :, :n, :]), bits(host)), (step, g, s)
    st = tier.stats
    assert (st.hits, st.misses, st.loads, st.evictions) == (ref.hits, ref.misses, ref.loads, ref.evictions)
    assert st.bytes_loaded > 0
    tier.close()


def one_step(B, pool, slots_or_groups, w, dev, n_new, tier=None, prefetch=None):
    """select + gather + attention + reduced mass over the given pool ids; returns (out, mass) bits."""
    import torch
    cfg = w.cfg
    plan = B.segment_select(pool, slots_or_groups, [0, len(slots_or_groups)], n_new)
    kc, vt = B.alloc_context(pool, plan)
    ws = B.alloc_workspace(pool, plan)
    out = torch.empty((1, n_new, cfg.n_q_heads, cfg.head_dim), dtype=dev["q"].dtype, device="cuda:0")
    mass = torch.empty((1, plan.info.max_segments + 1), dtype=torch.float32, device="cuda:0")
    B.gather_rope(pool, plan, dev["k_new"], dev["v_new"], kc, vt)
    if tier is not None:
        B.kv_tier_fence(tier)             # the slots are not read after this point
        if prefetch is not None:
            B.kv_tier_prefetch(tier, prefetch)     # runs beside the attention kernels
    B.segmented_prefill_attention(pool, plan, dev["q"], kc, vt, out, ws)
    B.segment_attention_mass(pool, plan, ws, 1, mass)
    return plan, out, mass, (kc, vt, ws)


@pytest.mark.parametrize("base,n_slots,ahead", [("c1", 20, False), ("c1", 20, True), ("c1", 40, True),
                                                ("c0", 5, True)])
def test_steps_over_fetched_slots_equal_steps_over_a_full_pool(mods, oracle, base, n_slots, ahead):
    import torch
    B, S = mods
    cfg = I.variant(I.CONFIGS[base], seed=33, fixed_sel=None) if base == "c0" else I.CONFIGS[base]
    w = I.make_workload(cfg)
    bf16 = cfg.dtype == I.BF16
    n_sel = min(cfg.n_sel, n_slots - 1)
    announce(f"tier steps: {base} dtype={cfg.dtype} G={cfg.n_groups} slots={n_slots} S={n_sel} "
             f"Nq={cfg.n_new} prefetch={ahead}")
    max_ctx = n_sel * cfg.capacity + cfg.n_new
    full = S.PlanningStep(w, max_ctx=max_ctx)          # every group resident
    dev = {"q": full.q[:1].contiguous(), "k_new": full.k_new[:1].contiguous(),
           "v_new": full.v_new[:1].contiguous()}
    tier, _ = make_tier(B, cfg, w, n_slots, max_ctx)
    # selections that drift: each step replaces a few groups of the previous one
    rng = np.random.default_rng(8)
    sels = [rng.permutation(cfg.n_groups)[:n_sel]]
    for t in range(5):
        nxt = sels[-1].copy()
        others = np.setdiff1d(np.arange(cfg.n_groups), nxt)
        swap = rng.permutation(n_sel)[:max(1, n_sel // 4)]
        nxt[swap] = rng.permutation(others)[:len(swap)]
        sels.append(rng.permutation(nxt))
    keep = []
    for t, groups in enumerate(sels):
        slots = B.kv_tier_fetch(tier, groups)
        nxt = sels[t + 1] if ahead and t + 1 < len(sels) else None
        plan, out, mass, bufs = one_step(B, tier.pool, slots, w, dev, cfg.n_new, tier, nxt)
        keep.append((plan, out, mass, bufs))
    torch.cuda.synchronize()
    st = tier.stats
    assert st.requested == n_sel * len(sels) and st.hits + st.prefetched + st.misses == st.requested
    if ahead and n_slots >= 2 * n_sel:
        assert st.prefetched > 0 and st.misses == n_sel       # after the first step nothing is loaded late
    for t, groups in enumerate(sels):
        plan_f, out_f, mass_f, bufs_f = one_step(B, full.pool, groups, w, dev, cfg.n_new)
        torch.cuda.synchronize()
        plan, out, mass, _ = keep[t]
        assert np.array_equal(plan.offsets(0), plan_f.offsets(0))
        assert np.array_equal(bits(out), bits(out_f)), f"step {t}: output differs from the full pool's"
        assert np.array_equal(bits(mass), bits(mass_f)), f"step {t}: masses differ from the full pool's"
    # and the last step against the oracle
    groups = sels[-1]
    ref_out, ref_mass = oracle.attention(w.k_pool, w.v_pool, w.lens, groups.astype(np.int32),
                                         np.array([0, n_sel], dtype=np.int32), w.q[:1], w.k_new[:1],
                                         w.v_new[:1], cfg.rope_base)[:2]
    got = S._to_host(keep[-1][1]).astype(np.float64)
    tol = 2e-2 if bf16 else 1e-5 * np.abs(ref_out).max()
    assert np.abs(got - ref_out).max() <= tol
    tier.close()


def test_put_replaces_a_resident_group(mods):
    import torch
    B, _ = mods
    cfg = I.variant(I.CONFIGS["c1"], n_groups=6, seed=5, n_sel=2)
    w = I.make_workload(cfg)
    announce("tier put: c1 G=6 slots=3")
    tier, blocks = make_tier(B, cfg, w, 3, 4096)
    s0 = B.kv_tier_fetch(tier, [2, 4])
    torch.cuda.synchronize()
    k_new = (blocks[2][0][:, :7, :] * 2).contiguous()
    v_new = (blocks[2][1][:, :7, :] * 2).contiguous()
    B.kv_tier_put(tier, 2, k_new, v_new)
    assert tier.residency()[2] == -1 and tier.residency()[4] == s0[1]
    s1 = B.kv_tier_fetch(tier, [2])
    torch.cuda.synchronize()
    assert np.array_equal(bits(tier.pool.k[s1[0], :, :7, :]), bits(k_new))
    assert np.array_equal(bits(tier.pool.v[s1[0], :, :7, :]), bits(v_new))
    plan = B.segment_select(tier.pool, s1, [0, 1], 4)
    assert plan.offsets(0).tolist() == [0, 7]          # the slot carries the new length
    tier.close()


@pytest.mark.parametrize("base", ["c1", "c0"])
def test_append_reaches_the_store_and_the_resident_copy(mods, base):
    """Section 3.2: the KV of objects that join a group is saved at the end of the group's cache. With a
    tier that is the store's block and, if the group is resident, its slot; a group that is displaced
    and loaded again comes back with the appended rows."""
    import torch
    B, _ = mods
    cfg = I.variant(I.CONFIGS[base], n_groups=4, seed=17, n_sel=2, fixed_sel=None,
                    len_lo=5, len_hi=I.CONFIGS[base].capacity - 9)
    w = I.make_workload(cfg)
    announce(f"tier append: {base} dtype={cfg.dtype} G=4 slots=2 lens={w.lens.tolist()}")
    tier, blocks = make_tier(B, cfg, w, 2, 4096)
    dt = blocks[0][0].dtype
    gen = torch.Generator().manual_seed(3)
    new = {g: (torch.randn((n, cfg.n_kv_heads, cfg.head_dim), generator=gen).to(dt),
               torch.randn((n, cfg.n_kv_heads, cfg.head_dim), generator=gen).to(dt))
           for g, n in ((0, 7), (2, 3))}

    def expect(g):
        k, v = blocks[g]
        if g in new:
            k = torch.cat([k, new[g][0].permute(1, 0, 2)], dim=1)
            v = torch.cat([v, new[g][1].permute(1, 0, 2)], dim=1)
        return k, v

    def check(groups, slots):
        torch.cuda.synchronize()
        for g, s in zip(groups, slots):
            k, v = expect(g)
            n = k.shape[1]
            assert tier.pool.desc.capacity >= n
            assert np.array_equal(bits(tier.pool.k[s, :, :n, :]), bits(k)), g
            assert np.array_equal(bits(tier.pool.v[s, :, :n, :]), bits(v)), g
            plan = B.segment_select(tier.pool, [s], [0, 1], 4)
            assert plan.offsets(0).tolist() == [0, n]
            plan.close()

    s01 = B.kv_tier_fetch(tier, [0, 1])
    for g in (0, 2):                       # 0 is resident, 2 is not
        B.kv_tier_append(tier, g, new[g][0].cuda(), new[g][1].cuda())
    check([0, 1], s01)
    s23 = B.kv_tier_fetch(tier, [2, 3])     # displaces 0 and 1; 2 comes from the store with its new rows
    check([2, 3], s23)
    s01 = B.kv_tier_fetch(tier, [1, 0])     # 0 comes back from the store with its new rows
    check([1, 0], s01)
    with pytest.raises(B.EnError) as e:
        B.kv_tier_append(tier, 1, torch.zeros((cfg.capacity, cfg.n_kv_heads, cfg.head_dim), dtype=dt).cuda(),
                         torch.zeros((cfg.capacity, cfg.n_kv_heads, cfg.head_dim), dtype=dt).cuda())
    assert e.value.code == 4
    tier.close()


def test_random_tier_traces_keep_the_data_right(mods):
    """Random traces of fetch / prefetch / fence / put / append on tiers of random sizes: the slots a fetch
    hands out equal the bookkeeping oracle's, and what they hold equals what was put and appended."""
    import torch
    B, _ = mods
    rng = np.random.default_rng(5)
    for case in range(40):
        base = "c1" if rng.random() < 0.6 else "c0"
        G = int(rng.integers(3, 14))
        n_slots = int(rng.integers(1, G + 1))
        capc = I.CONFIGS[base].capacity
        cfg = I.variant(I.CONFIGS[base], n_groups=G, seed=7000 + case, n_sel=1, fixed_sel=None, len_lo=0,
                        len_hi=capc - 12)
        w = I.make_workload(cfg)
        announce(f"tier trace {case}: {base} G={G} slots={n_slots}")
        tier, blocks = make_tier(B, cfg, w, n_slots, 4096)
        dt = blocks[0][0].dtype
        cur = {g: [blocks[g][0].clone(), blocks[g][1].clone()] for g in range(G)}
        ref = Residency(n_slots)
        for step in range(40):
            op = rng.choice(["fetch", "fetch", "fetch", "prefetch", "fence", "put", "append"])
            if op in ("fetch", "prefetch"):
                groups = rng.permutation(G)[:int(rng.integers(0, n_slots + 1))]
                if op == "prefetch":
                    assert B.kv_tier_prefetch(tier, groups) == ref.prefetch(groups.tolist())
                    continue
                slots = B.kv_tier_fetch(tier, groups)
                assert slots.tolist() == ref.fetch(groups.tolist())[0]
                torch.cuda.synchronize()
                for g, s in zip(groups, slots):
                    n = cur[g][0].shape[1]
                    assert np.array_equal(bits(tier.pool.k[s, :, :n, :]), bits(cur[g][0])), (case, step, g)
                    assert np.array_equal(bits(tier.pool.v[s, :, :n, :]), bits(cur[g][1])), (case, step, g)
            elif op == "fence":
                B.kv_tier_fence(tier)
                ref.fence()
            elif op == "put":
                g, n = int(rng.integers(0, G)), int(rng.integers(0, capc - 12))
                k = torch.randn((cfg.n_kv_heads, n, cfg.head_dim)).to(dt)
                v = torch.randn((cfg.n_kv_heads, n, cfg.head_dim)).to(dt)
                B.kv_tier_put(tier, g, k, v)
                ref.put(g)
                cur[g] = [k, v]
            else:
                g = int(rng.integers(0, G))
                n = int(rng.integers(0, min(capc - cur[g][0].shape[1], 5) + 1))
                k = torch.randn((n, cfg.n_kv_heads, cfg.head_dim)).to(dt)
                v = torch.randn((n, cfg.n_kv_heads, cfg.head_dim)).to(dt)
                B.kv_tier_append(tier, g, k.cuda(), v.cuda(), n_tokens=n)
                cur[g] = [torch.cat([cur[g][0], k.permute(1, 0, 2)], 1).contiguous(),
                          torch.cat([cur[g][1], v.permute(1, 0, 2)], 1).contiguous()]
            assert tier.residency().tolist() == [ref.slot_of(g) for g in range(G)], (case, step, op)
        torch.cuda.synchronize()
        tier.close()
