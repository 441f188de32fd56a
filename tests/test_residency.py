"""Residency bookkeeping: the oracle (oracle/residency.py) against what the mathematics of
least-recently-used replacement fixes, and the library's host logic against the oracle, decision by
decision. No GPU: the library's tier is created without device memory, where it only keeps the books."""
import numpy as np
import pytest

from oracle.residency import Residency
from paper_2510_18546_amd import binding as B
from paper_2510_18546_amd import inputs


def _faults(n_slots, refs):
    r = Residency(n_slots)
    for g in refs:
        r.fetch([g])
    return r.misses


# The worked page-replacement example found in operating-systems textbooks (reference string of 20
# pages over 8 distinct ones): least-recently-used replacement takes 12 faults with 3 frames and 8 with 4.
TEXTBOOK = [7, 0, 1, 2, 0, 3, 0, 4, 2, 3, 0, 3, 2, 1, 2, 0, 1, 7, 0, 1]


def test_oracle_textbook_reference_string():
    assert _faults(3, TEXTBOOK) == 12
    assert _faults(4, TEXTBOOK) == 8
    assert _faults(8, TEXTBOOK) == 6 == len(set(TEXTBOOK))     # only the compulsory ones
    assert _faults(1, TEXTBOOK) == 20 - 0                      # no page repeats back to back


def test_oracle_cyclic_sweep_never_hits():
    # n+1 groups asked for in a cycle with n slots: the one needed next is always the one just displaced
    for n in (1, 2, 5):
        assert _faults(n, list(range(n + 1)) * 6) == 6 * (n + 1)
        assert _faults(n + 1, list(range(n + 1)) * 6) == n + 1


def test_oracle_inclusion_property():
    # least-recently-used is a stack algorithm: with one more slot the resident set only grows, so
    # the hits never drop (first-in-first-out, or displacing the newest, breaks this on some trace)
    rng = np.random.default_rng(5)
    for trial in range(30):
        refs = rng.integers(0, 9, size=80).tolist()
        tiers = [Residency(n) for n in range(1, 9)]
        for g in refs:
            for r in tiers:
                r.fetch([g])
            for small, big in zip(tiers, tiers[1:]):
                assert small.resident() <= big.resident()
        hits = [r.hits for r in tiers]
        assert hits == sorted(hits)


def test_oracle_set_requests_invariants():
    rng = np.random.default_rng(11)
    for trial in range(40):
        n_slots = int(rng.integers(2, 9))
        G = int(rng.integers(n_slots, 3 * n_slots + 1))
        r = Residency(n_slots)
        for step in range(40):
            k = int(rng.integers(0, n_slots + 1))
            groups = rng.permutation(G)[:k].tolist()
            before = r.resident()
            age_before = {g: r.age[r.slot_of(g)] for g in before}
            slots, kinds = r.fetch(groups)
            assert len(set(slots)) == len(slots) and all(0 <= s < n_slots for s in slots)
            assert set(groups) <= r.resident() and len(r.resident()) <= n_slots
            assert [k == "miss" for k in kinds] == [g not in before for g in groups]
            # a resident group gives way only if every group that stayed and was not asked for
            # was used more recently or is equally old
            gone = before - r.resident()
            stayed = (before & r.resident()) - set(groups)
            assert not (gone & set(groups))
            if gone and stayed:
                assert max(age_before[g] for g in gone) <= min(age_before[g] for g in stayed)
        assert r.hits + r.misses + r.prefetched == r.requested


def test_oracle_victim_is_the_least_recently_used():
    r = Residency(3)
    r.fetch([10, 11, 12])          # slots 0 1 2, all used at step 1
    r.fetch([11])                  # 11 newer
    r.fetch([12])                  # 12 newest
    slots, kinds = r.fetch([13])   # 10 is the oldest
    assert kinds == ["miss"] and slots == [0] and r.resident() == {11, 12, 13}
    slots, kinds = r.fetch([14, 12])     # 12 is asked for in the same step: it must not give way
    assert kinds == ["miss", "hit"] and r.resident() == {12, 13, 14} and slots[0] == 1
    # equally old slots: the lowest number first
    r = Residency(4)
    r.fetch([1, 2, 3, 4])
    assert r.fetch([5, 6])[0] == [0, 1]


def test_oracle_prefetch_and_fence():
    r = Residency(4)
    r.fetch([0, 1])                                   # slots 0, 1
    assert r.prefetch([2, 3, 4]) == 2                 # no fence yet: only the two unused slots
    assert r.resident() == {0, 1, 2, 3}
    slots, kinds = r.fetch([2, 0, 5])                 # 2 came by prefetch, 0 by a fetch, 5 is new
    assert kinds == ["prefetched", "hit", "miss"]
    assert 3 not in r.resident() or 1 not in r.resident()     # 5 displaced one of the idle ones
    r.fence()
    assert r.prefetch([7]) == 1                       # now a used slot may be taken
    slots, kinds = r.fetch([7])
    assert kinds == ["prefetched"]
    slots, kinds = r.fetch([7])
    assert kinds == ["hit"]                           # only the first use counts as prefetched
    r.put(7)
    assert 7 not in r.resident()
    assert r.fetch([7])[1] == ["miss"]


# ---------------------------------------------------------------------------------------------
# the library's bookkeeping against the oracle
# ---------------------------------------------------------------------------------------------
SHAPE = (8, 16, 64)     # Hkv, C, D of a block; irrelevant to the bookkeeping


def test_oracle_unfenced_fetch_fences_for_itself_hand_worked():
    """Four steps worked by hand, no library involved. Three slots, no explicit fence anywhere.
    The rule under test: a fetch that has to load while the last fence is older than the previous
    step first waits for everything queued so far (there is nothing else it could wait for), and
    that wait covers every reader of the slots handed out in earlier steps, so from then on those
    slots count as fenced, exactly as after fence(). Slots used by the CURRENT step are not covered.

      step 1  fetch A B C   all miss                        slots [A B C]  ages [1 1 1]  fenced never
      step 2  fetch A D     A hit (age 2); D must load: fences for itself -> fenced = 1;
                            D takes the oldest slot not used in step 2: slots 1 and 2 are both age 1,
                            the lower number wins            slots [A D C]  ages [2 2 1]
              prefetch E    may take slots with age <= fenced = 1 only: slot 2 (C) -> E, 1 loaded;
                            without the rule nothing would be fenced and 0 would be loaded
                                                            slots [A D E]  ages [2 2 1]
              prefetch F    slot 2 now holds a prefetched group as old as the fence: it is the only
                            candidate again, F displaces E   slots [A D F]
      step 3  fetch F A     F was prefetched, A hit          ages [3 2 3]
      step 4  fetch C       miss; fences for itself -> fenced = 3; oldest slot is 1 (D, age 2)
                                                            slots [A C F]  ages [3 4 3]
    """
    A, B_, C, D, E, F = range(6)
    r = Residency(3)
    assert r.fetch([A, B_, C]) == ([0, 1, 2], ["miss", "miss", "miss"])
    assert r.fenced == -1
    assert r.fetch([A, D]) == ([0, 1], ["hit", "miss"])
    assert r.fenced == 1
    assert r.prefetch([E]) == 1 and r.slot_of(E) == 2 and r.slot_of(C) == -1
    assert r.prefetch([F]) == 1 and r.slot_of(F) == 2 and r.slot_of(E) == -1
    assert r.fetch([F, A]) == ([2, 0], ["prefetched", "hit"])
    assert r.fetch([C]) == ([1], ["miss"])
    assert r.fenced == 3
    assert [r.group_in[s] for s in range(3)] == [A, C, F]
    assert (r.hits, r.prefetched, r.misses, r.loads, r.evictions, r.requested) == (2, 1, 5, 7, 4, 8)
    # and with an explicit fence in its place the same trace gives the same slots
    q = Residency(3)
    q.fetch([A, B_, C])
    q.fence()
    q.fetch([A, D])
    assert q.prefetch([E]) == 1 and q.slot_of(E) == 2


def _tier(n_slots, G):
    t = B.kv_tier_create(None, None, G, 32, 1e4, 4096, dtype=B.EN_BF16, shape=(n_slots,) + SHAPE)
    for g in range(G):
        B.kv_tier_put(t, g, None, None, 1 + g % 16)
    return t


def test_tier_matches_oracle_on_random_traces():
    rng = np.random.default_rng(3)
    for trial in range(60):
        n_slots = int(rng.integers(1, 10))
        G = int(rng.integers(n_slots, 3 * n_slots + 2))
        t, r = _tier(n_slots, G), Residency(n_slots)
        for step in range(60):
            op = rng.choice(["fetch", "fetch", "fetch", "prefetch", "fence", "put"])
            if op in ("fetch", "prefetch"):
                k = int(rng.integers(0, n_slots + 1))
                groups = rng.permutation(G)[:k].tolist()
                if op == "fetch":
                    assert B.kv_tier_fetch(t, groups).tolist() == r.fetch(groups)[0], (trial, step)
                else:
                    assert B.kv_tier_prefetch(t, groups) == r.prefetch(groups), (trial, step)
            elif op == "fence":
                B.kv_tier_fence(t)
                r.fence()
            else:
                g = int(rng.integers(0, G))
                B.kv_tier_put(t, g, None, None, 3)
                r.put(g)
            assert t.residency().tolist() == [r.slot_of(g) for g in range(G)], (trial, step, op)
            st = t.stats
            assert (st.requested, st.hits, st.prefetched, st.misses, st.loads, st.evictions) == \
                (r.requested, r.hits, r.prefetched, r.misses, r.loads, r.evictions), (trial, step, op)
        t.close()


def test_tier_textbook_reference_string():
    for n, want in ((3, 12), (4, 8)):
        t = _tier(n, 8)
        for g in TEXTBOOK:
            B.kv_tier_fetch(t, [g])
        assert t.stats.misses == want and t.stats.hits == len(TEXTBOOK) - want
        t.close()


def test_tier_bytes_and_slot_size():
    t = _tier(2, 4)                      # lengths 1, 2, 3, 4
    B.kv_tier_fetch(t, [3, 1])
    Hkv, Cap, D = SHAPE
    assert t.stats.bytes_loaded == 2 * Hkv * D * 2 * (4 + 2)
    assert B.kv_tier_slot_bytes(SHAPE, B.EN_BF16) == 2 * Hkv * Cap * D * 2
    assert B.kv_tier_slot_bytes(SHAPE, B.EN_F32) == 2 * Hkv * Cap * D * 4
    t.close()


def test_tier_error_codes():
    t = B.kv_tier_create(None, None, 6, 32, 1e4, 4096, dtype=B.EN_BF16, shape=(3,) + SHAPE)
    for g in range(5):
        B.kv_tier_put(t, g, None, None, 4)
    for groups, code in (([0, 1, 2, 3], 4), ([0, 0], 3), ([6], 2), ([-1], 2), ([5], 2)):
        for call in (B.kv_tier_fetch, B.kv_tier_prefetch):
            with pytest.raises(B.EnError) as e:
                call(t, groups)
            assert e.value.code == code, (groups, call.__name__)
    with pytest.raises(B.EnError) as e:
        B.kv_tier_put(t, 0, None, None, SHAPE[1] + 1)
    assert e.value.code == 2
    with pytest.raises(B.EnError) as e:
        B.kv_tier_put(t, 6, None, None, 1)
    assert e.value.code == 2
    assert t.stats.requested == 0 and (t.residency() == -1).all()      # a refused call changes nothing
    t.close()
    with pytest.raises(B.EnError) as e:
        B.kv_tier_create(None, None, 0, 32, 1e4, 4096, dtype=B.EN_BF16, shape=(3,) + SHAPE)
    assert e.value.code == 1


def test_tier_scored_selection_matches_oracle_knapsack():
    from oracle import oracle as O
    rng = np.random.default_rng(9)
    G = 14
    t = B.kv_tier_create(None, None, G, 32, 1e4, 4096, dtype=B.EN_BF16, shape=(4,) + SHAPE)
    lens = rng.integers(1, 17, size=G)
    lens[5] = 0
    never = {2, 9}
    for g in range(G):
        if g not in never:
            B.kv_tier_put(t, g, None, None, int(lens[g]))
    for trial in range(20):
        p = rng.random(G).astype(np.float32)
        budget = int(rng.integers(0, 60))
        got = B.kv_tier_select_scored(t, p, 0.3, budget).tolist()
        cand = [g for g in range(G) if g not in never]
        want = O.knapsack(p[cand], lens[cand], 0.3, budget)
        assert got == [cand[i] for i in want], trial
    t.close()


def test_hit_rate_grows_with_the_budget_on_drifting_scores():
    # Section 4 (cache hit rate): with scores that change little between adjacent steps, the hit
    # rate rises with the device budget and is high once the budget holds the selection plus its churn
    G, n_sel, steps = 64, 8, 120
    scores = inputs.drifting_scores(1, G, steps, rho=0.95)
    rates = []
    for n_slots in (8, 12, 16, 32, 64):
        t = _tier(n_slots, G)
        for s in scores:
            groups = np.argsort(-s, kind="stable")[:n_sel]
            B.kv_tier_fetch(t, np.sort(groups))
        rates.append(t.stats.hits / t.stats.requested)
        t.close()
    assert rates == sorted(rates)
    assert rates[-1] > 0.9 and rates[0] < rates[-1]


def test_tier_append_bookkeeping():
    t = B.kv_tier_create(None, None, 3, 32, 1e4, 4096, dtype=B.EN_BF16, shape=(2,) + SHAPE)
    B.kv_tier_put(t, 0, None, None, 4)
    B.kv_tier_put(t, 1, None, None, SHAPE[1] - 1)
    B.kv_tier_append(t, 0, None, None, 5)
    B.kv_tier_fetch(t, [0])
    Hkv, Cap, D = SHAPE
    assert t.stats.bytes_loaded == 2 * Hkv * D * 2 * 9           # the appended rows are part of the block
    B.kv_tier_append(t, 1, None, None, 1)
    for group, n, code in ((1, 1, 4), (2, 1, 2), (3, 1, 2), (0, -1, 1)):
        with pytest.raises(B.EnError) as e:
            B.kv_tier_append(t, group, None, None, n)
        assert e.value.code == code, (group, n)
    assert B.kv_tier_select_scored(t, np.array([1, 1, 1], np.float32), 0.0, 9).tolist() == [0]
    t.close()
