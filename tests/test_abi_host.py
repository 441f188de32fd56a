"""Host side of the C ABI, no GPU: the library loads, exports every symbol the
header declares, and the planner / knapsack agree bit-exactly with the oracle.
Pool device pointers are opaque non-null tokens here; no kernel is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2510_18546_amd import binding as B
from paper_2510_18546_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = dict(k_ptr=0x1000, v_ptr=0x2000)


def host_pool(lens, cap=8, hkv=2, hq=4, d=64, dtype=B.EN_BF16, max_ctx=4096, base=1e4):
    return B.kv_pool_create(None, None, lens, hq, base, max_ctx, dtype=dtype,
                            shape=(len(lens), hkv, cap, d), **FAKE)


def test_library_exports_every_declared_symbol():
    lib = B.load()
    hdr = open(os.path.join(ROOT, "include", "efficientnav.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\(", hdr)
    names = sorted(set(n for n in names if not n.startswith("defined")))
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_plan_offsets_bit_exact_vs_oracle(oracle):
    rng = np.random.default_rng(0)
    for _ in range(50):
        G = int(rng.integers(1, 40))
        cap = int(rng.integers(1, 300))
        lens = rng.integers(0, cap + 1, G).astype(np.int32)
        Bn = int(rng.integers(1, 5))
        lists = [rng.choice(G, size=int(rng.integers(0, G + 1)), replace=False).astype(np.int32)
                 for _ in range(Bn)]
        ptr = np.concatenate([[0], np.cumsum([len(l) for l in lists])]).astype(np.int32)
        sel = np.concatenate(lists).astype(np.int32) if ptr[-1] else np.zeros(0, np.int32)
        nq = int(rng.integers(1, 70))
        pool = host_pool(lens, cap=cap, max_ctx=G * cap + nq)
        plan = B.segment_select(pool, sel, ptr, nq)
        inf = plan.info
        worst = 0
        pairs = 0
        for b in range(Bn):
            want = oracle.plan(lens, lists[b])
            got = plan.offsets(b)
            assert got.dtype == np.int32 and np.array_equal(got, want)
            worst = max(worst, int(want[-1]) + nq)
            pairs += nq * int(want[-1]) + nq * (nq + 1) // 2
        assert inf.n_agents == Bn and inf.n_new == nq
        assert inf.max_ctx_len == worst and inf.ctx_stride % 64 == 0 and inf.ctx_stride >= worst
        assert inf.total_pairs == pairs
        assert inf.max_segments == max(len(l) for l in lists)
        assert B.context_bytes(pool, plan) == Bn * 2 * inf.ctx_stride * 64 * 2
        assert B.workspace_bytes(pool, plan) > 0


def test_c0_plan_matches_golden():
    w = I.make_workload(I.CONFIGS["c0"], poison=False)
    pool = host_pool(w.lens, cap=32, hkv=1, hq=4, d=64, dtype=B.EN_F32, max_ctx=192)
    plan = B.segment_select(pool, w.sel, w.sel_ptr, 64)
    assert plan.offsets(0).tolist() == [0, 32, 64, 96, 128]
    assert plan.info.max_ctx_len == 192


def test_error_codes():
    lens = np.array([3, 0, 5, 8], np.int32)
    pool = host_pool(lens, max_ctx=20)
    with pytest.raises(B.EnError) as e:
        B.segment_select(pool, [0, 4], [0, 2], 4)
    assert e.value.code == 2                                   # id out of range
    with pytest.raises(B.EnError) as e:
        B.segment_select(pool, [0, -1], [0, 2], 4)
    assert e.value.code == 2
    with pytest.raises(B.EnError) as e:
        B.segment_select(pool, [2, 0, 2], [0, 3], 4)
    assert e.value.code == 3                                   # duplicate
    B.segment_select(pool, [2, 0, 2, 3], [0, 2, 4], 4)         # same id in two agents is fine
    with pytest.raises(B.EnError) as e:
        B.segment_select(pool, [0, 2, 3], [0, 3], 5)           # 16 + 5 > 20
    assert e.value.code == 4
    B.segment_select(pool, [0, 2, 3], [0, 3], 4)               # 16 + 4 == 20 fits
    with pytest.raises(B.EnError) as e:
        B.segment_select(pool, [0], [0, 1], 0)
    assert e.value.code == 1
    with pytest.raises(B.EnError) as e:
        host_pool(np.array([9], np.int32), cap=8)
    assert e.value.code == 2                                   # len > capacity
    with pytest.raises(B.EnError) as e:
        host_pool(lens, d=96)
    assert e.value.code == 5
    with pytest.raises(B.EnError) as e:
        host_pool(lens, hkv=3, hq=4)
    assert e.value.code == 5
    with pytest.raises(B.EnError) as e:
        B.kv_pool_create(None, None, lens, 4, 1e4, 64, dtype=B.EN_BF16, shape=(4, 2, 8, 64),
                         k_ptr=0, v_ptr=0x10)
    assert e.value.code == 1                                   # null device pointer
    assert b"null" in B.load().en_last_error()
    with pytest.raises(B.EnError) as e:
        B.kv_pool_set_len(pool, 1, 9)
    assert e.value.code == 2


def test_empty_selection_and_empty_groups():
    lens = np.array([3, 0, 5], np.int32)
    pool = host_pool(lens)
    plan = B.segment_select(pool, [], [0, 0], 7)
    assert plan.offsets(0).tolist() == [0] and plan.info.max_ctx_len == 7
    plan = B.segment_select(pool, [1, 2, 0], [0, 3], 2)
    assert plan.offsets(0).tolist() == [0, 0, 5, 8]


def test_set_len_affects_later_plans_only():
    lens = np.array([3, 4], np.int32)
    pool = host_pool(lens)
    p1 = B.segment_select(pool, [0, 1], [0, 2], 1)
    B.kv_pool_set_len(pool, 0, 6)
    p2 = B.segment_select(pool, [0, 1], [0, 2], 1)
    assert p1.offsets(0).tolist() == [0, 3, 7] and p2.offsets(0).tolist() == [0, 6, 10]


def test_set_splits_clamps():
    pool = host_pool(np.full(16, 8, np.int32), max_ctx=1024)
    plan = B.segment_select(pool, np.arange(16), [0, 16], 10)      # 138 keys -> 3 tiles
    plan.set_splits(100)
    assert plan.info.n_splits == 3
    plan.set_splits(1)
    assert plan.info.n_splits == 1
    long_pool = host_pool(np.full(40, 250, np.int32), cap=256, max_ctx=16384)
    long_plan = B.segment_select(long_pool, np.arange(40), [0, 40], 1)  # 10001 keys -> 157 tiles
    long_plan.set_splits(100)
    assert long_plan.info.n_splits == 64


@pytest.mark.parametrize("n_groups,tiles,expect", [(7, 28, 28), (17, 67, 34), (25, 98, 49), (34, 133, 64),
                                                   (41, 161, 54)])
def test_split_choice_of_a_one_token_step(n_groups, tiles, expect):
    """Host logic, 256 compute units assumed without a device, 2 KV heads, one agent: as many KV splits
    as there are key tiles up to 64; then the fewest splits that keep the longest split as short (67
    tiles: 2 per split either way, so 34 splits; 161 tiles: 54 x 3) unless fewer than an eighth of the
    splits are three tiles or longer (133 tiles over 64 splits: five of them)."""
    pool = host_pool(np.full(n_groups, 250, np.int32), cap=256, max_ctx=16384)
    plan = B.segment_select(pool, np.arange(n_groups), [0, n_groups], 1)
    assert (plan.info.max_ctx_len + 63) // 64 == tiles
    assert plan.info.n_splits == expect


def test_scored_selection_matches_oracle(oracle):
    rng = np.random.default_rng(5)
    for trial in range(120):
        G = int(rng.integers(1, 15)) if trial < 90 else int(rng.integers(17, 60))
        cap = 12
        lens = rng.integers(0, cap + 1, G).astype(np.int32)
        p = rng.random(G).astype(np.float32)
        if trial % 2:
            p = (np.round(p * 8) / 8).astype(np.float32)
        budget = int(rng.integers(0, max(2, int(lens.sum()) + 3)))
        pool = host_pool(lens, cap=cap, max_ctx=G * cap + 4)
        got, plan = B.segment_select_scored(pool, p, 0.375, budget, 4)
        want = oracle.knapsack(p, lens, 0.375, budget)
        assert got.tolist() == want
        assert plan.offsets(0).tolist() == oracle.plan(lens, want).tolist()
        assert int(lens[got].sum()) <= budget


def test_scored_selection_edges():
    lens = np.array([4, 1, 3, 3], np.int32)
    pool = host_pool(lens)
    p = np.array([0.9, 0.2, 0.6, 0.55], np.float32)
    assert B.segment_select_scored(pool, p, 0.5, 0, 1, want_plan=False)[0].tolist() == []
    assert B.segment_select_scored(pool, p, 0.5, 10 ** 12, 1, want_plan=False)[0].tolist() == [0, 2, 3]
    with pytest.raises(B.EnError) as e:
        B.segment_select_scored(pool, p, 0.5, -1, 1)
    assert e.value.code == 1


def test_scored_selection_refuses_what_it_cannot_hold_or_compare():
    """Nothing crosses the C ABI as a C++ exception: a knapsack table beyond the stated limit is
    refused with a status, and so is a score or threshold that is not a finite number."""
    # 2000 candidates x a budget of 5e6 tokens: 2000 * 5e6 / 8 bytes = 1.25 GB of take bits > 1 GiB
    G, cap = 2000, 5000
    lens = np.full(G, cap, np.int32)
    pool = host_pool(lens, cap=cap, max_ctx=2 ** 31 - 1)
    p = np.linspace(0.6, 0.9, G).astype(np.float32)
    with pytest.raises(B.EnError) as e:
        B.segment_select_scored(pool, p, 0.5, 5_000_000, 1, want_plan=False)
    assert e.value.code == 4 and "limit" in str(e.value)
    # the same candidates under a budget that admits them all need no table
    got = B.segment_select_scored(pool, p, 0.5, G * cap, 1, want_plan=False)[0]
    assert got.tolist() == list(range(G))
    small_pool = host_pool(np.array([4, 1, 3, 3], np.int32))
    for bad in (np.nan, np.inf, -np.inf):
        p4 = np.array([0.9, bad, 0.6, 0.55], np.float32)
        with pytest.raises(B.EnError) as e:
            B.segment_select_scored(small_pool, p4, 0.5, 5, 1, want_plan=False)
        assert e.value.code == 1
        with pytest.raises(B.EnError) as e:
            B.segment_select_scored(small_pool, np.array([0.9, 0.2, 0.6, 0.55], np.float32), bad, 5, 1,
                                    want_plan=False)
        assert e.value.code == 1
    # a tier's selection goes through the same checks
    t = B.kv_tier_create(None, None, 4, 4, 1e4, 64, dtype=B.EN_BF16, shape=(2, 2, 8, 64))
    for g in range(4):
        B.kv_tier_put(t, g, None, None, 3)
    with pytest.raises(B.EnError) as e:
        B.kv_tier_select_scored(t, np.array([0.9, np.nan, 0.6, 0.55], np.float32), 0.5, 6)
    assert e.value.code == 1
    t.close()


def test_append_checks_without_device():
    """Range and capacity checks of kv_pool_append come before any device work;
    a rejected append leaves the length as it was."""
    lens = np.array([3, 8, 0, 5], np.int32)
    pool = B.kv_pool_create(None, None, lens, n_q_heads=4, rope_base=1e4, max_ctx=64, dtype=B.EN_BF16,
                            k_ptr=0x1000, v_ptr=0x2000, shape=(4, 2, 8, 64))
    with pytest.raises(B.EnError) as e:
        B.kv_pool_append(pool, 4, 0x3000, 0x4000, 1)
    assert e.value.code == 2
    with pytest.raises(B.EnError) as e:
        B.kv_pool_append(pool, 1, 0x3000, 0x4000, 1)          # group 1 is full
    assert e.value.code == 4
    with pytest.raises(B.EnError) as e:
        B.kv_pool_append(pool, 0, 0x3000, 0x4000, 6)          # 3 + 6 > 8
    assert e.value.code == 4
    with pytest.raises(B.EnError) as e:
        B.kv_pool_append(pool, 0, 0x3000, 0x4000, -1)
    assert e.value.code == 1
    with pytest.raises(B.EnError) as e:
        B.kv_pool_append(pool, 0, 0, 0x4000, 2)
    assert e.value.code == 1
    B.kv_pool_append(pool, 0, 0, 0, 0)                        # nothing to do
    plan = B.segment_select(pool, [0, 3], [0, 2], 4)
    assert plan.offsets(0).tolist() == [0, 3, 8]


def test_pool_destroyed_before_its_plans_host_side():
    lib = B.load()
    pool = B.kv_pool_create(None, None, [3, 4, 5], 4, 1e4, 64, dtype=B.EN_F32, k_ptr=8, v_ptr=8,
                            shape=(3, 1, 8, 64))
    p1 = B.segment_select(pool, [0, 2], [0, 2], 4)
    p2 = B.segment_select(pool, [1], [0, 1], 4)
    p1.close()                            # one leaves the pool's list the ordinary way
    h_pool, h_plan = pool.handle, p2.handle
    pool.handle = p2.handle = None
    assert lib.kv_pool_destroy(h_pool) == 0
    assert lib.en_plan_destroy(h_plan) == 0


def test_binding_closes_plans_before_their_pool():
    """Whatever order the garbage collector picks, a plan is never destroyed after its pool."""
    lens = np.array([3, 8, 0, 5], np.int32)
    pool = B.kv_pool_create(None, None, lens, n_q_heads=4, rope_base=1e4, max_ctx=64, dtype=B.EN_BF16,
                            k_ptr=0x1000, v_ptr=0x2000, shape=(4, 2, 8, 64))
    p1 = B.segment_select(pool, [0, 3], [0, 2], 4)
    p2 = B.segment_select(pool, [1], [0, 1], 2)
    pool.close()
    assert p1.handle is None and p2.handle is None
    p1.close()
    p2.close()
    pool.close()


def test_cluster_assign_checks_without_device():
    lens = np.array([3, 8, 0, 5], np.int32)
    pool = B.kv_pool_create(None, None, lens, n_q_heads=4, rope_base=1e4, max_ctx=64, dtype=B.EN_BF16,
                            k_ptr=0x1000, v_ptr=0x2000, shape=(4, 2, 8, 64))
    plan = B.segment_select(pool, [0, 3], [0, 2], 6)
    for spans in ([0, 0, 3], [2, 1], [0, 7], [-1, 2]):
        with pytest.raises(B.EnError) as e:
            B.segment_cluster_assign(pool, plan, 0x5000, spans, 0x6000, None)
        assert e.value.code == 1, spans
    with pytest.raises(B.EnError) as e:
        B.segment_cluster_assign(pool, plan, 0x5000, list(range(0, 7)) * 50, 0x6000, None)
    assert e.value.code in (1, 5)


def test_product_and_oracle_do_not_import_each_other():
    """The oracle is test infrastructure: nothing under the package imports it, and the oracle imports
    nothing of the package; only the seeded input generators serve both."""
    import ast
    import glob
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

    def imported(path):
        names = set()
        for node in ast.walk(ast.parse(open(path).read())):
            if isinstance(node, ast.Import):
                names.update(a.name.split(".")[0] for a in node.names)
            elif isinstance(node, ast.ImportFrom) and node.level == 0 and node.module:
                names.add(node.module.split(".")[0])
        return names
    for path in glob.glob(os.path.join(root, "paper_2510_18546_amd", "*.py")):
        assert "oracle" not in imported(path), path
    for path in glob.glob(os.path.join(root, "oracle", "*.py")):
        assert "paper_2510_18546_amd" not in imported(path), path
    # the C sources of the two sides include nothing of each other
    for path in glob.glob(os.path.join(root, "paper_2510_18546_amd", "csrc", "*")):
        assert "oracle" not in open(path).read().lower(), path
    assert "efficientnav.h" not in open(os.path.join(root, "oracle", "en_oracle.c")).read()


def test_header_is_plain_c_and_links_from_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 (and as C++), and a C program that links
    the library can build a plan with host calls only."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    inc = os.path.join(root, "include")
    src = tmp_path / "abi.c"
    src.write_text('''
#include <stdio.h>
#include <stdint.h>
#include "efficientnav.h"
int main(void) {
    en_pool_desc d = {0};
    int32_t len[3] = {3, 4, 5}, sel[2] = {2, 0}, ptr[2] = {0, 2}, off[3] = {0, 0, 0}, n = 0;
    en_pool *pool = NULL; en_plan *plan = NULL; en_plan_info info;
    d.n_groups = 3; d.capacity = 8; d.n_kv_heads = 1; d.n_q_heads = 4; d.head_dim = 64; d.dtype = EN_F32;
    d.max_ctx = 64; d.rope_base = 10000.0;
    if (kv_pool_create(&d, (void *)8, (void *)8, len, &pool) != EN_OK) return 1;
    if (segment_select(pool, 1, sel, ptr, 4, &plan) != EN_OK) return 2;
    if (en_plan_query(plan, 0, off, &n) != EN_OK || n != 2 || off[1] != 5 || off[2] != 8) return 3;
    if (en_plan_get_info(plan, &info) != EN_OK || info.total_cached != 8) return 4;
    if (segment_select(pool, 1, sel, ptr, 100, &plan) != EN_ERR_CAPACITY) return 5;
    printf("%s\\n", en_last_error());
    en_plan_destroy(plan); kv_pool_destroy(pool);
    return 0;
}
''')
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc,
                           "-fsyntax-only", str(src)])
    subprocess.check_call(["g++", "-std=c++11", "-Wall", "-Wextra", "-I", inc, "-fsyntax-only", "-x", "c++", str(src)])
    exe = tmp_path / "abi"
    subprocess.check_call(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe), B._build.LIB_PATH,
                           "-Wl,-rpath," + os.path.dirname(B._build.LIB_PATH)])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, (out.returncode, out.stdout, out.stderr)
    assert "max_ctx" in out.stdout


def test_q8_pool_checks_without_device():
    pool = B.kv_pool_create(None, None, [3, 4], 4, 1e4, 64, dtype=B.EN_I8, k_ptr=8, v_ptr=8, shape=(2, 1, 8, 64))
    plan = B.segment_select(pool, [1, 0], [0, 2], 4)
    assert plan.offsets(0).tolist() == [0, 4, 7]
    # contexts of an 8-bit pool are bf16: 2 bytes per element, 64 rows of padding granularity
    assert B.context_bytes(pool, plan) == 1 * 1 * plan.info.ctx_stride * 64 * 2
    with pytest.raises(B.EnError) as e:      # no scales yet
        B.load().gather_rope.restype = C.c_int
        rc = B.load().gather_rope(pool.handle, plan.handle, C.c_void_p(8), C.c_void_p(8), C.c_void_p(8), C.c_void_p(8), None)
        B._check(rc)
    assert e.value.code == 1 and "kv_pool_set_scales" in str(e.value)
    with pytest.raises(B.EnError) as e:
        B.kv_pool_append(pool, 0, 8, 8, n_tokens=1)
    assert e.value.code == 1
    f32 = B.kv_pool_create(None, None, [3, 4], 4, 1e4, 64, dtype=B.EN_F32, k_ptr=8, v_ptr=8, shape=(2, 1, 8, 64))
    with pytest.raises(B.EnError) as e:
        B.kv_pool_set_scales(f32, 8, 8)
    assert e.value.code == 1
    with pytest.raises(B.EnError) as e:
        B.kv_tier_create(None, None, 4, 4, 1e4, 64, dtype=B.EN_I8, shape=(2, 1, 8, 64))
    assert e.value.code == 5


def test_values_from_pool_checks_without_device():
    """en_plan_values_from_pool is a host-side property of the plan: what it refuses needs no GPU."""
    def code_of(fn):
        with pytest.raises(B.EnError) as e:
            fn()
        return e.value.code

    lens = [5, 6, 7]
    ok = B.kv_pool_create(None, None, lens, 8, 1e4, 256, dtype=B.EN_BF16, k_ptr=0x1000, v_ptr=0x2000,
                          shape=(3, 2, 8, 128))
    plan = B.segment_select(ok, [2, 0], [0, 2], 40)
    plan.values_from_pool(True)
    plan.values_from_pool(False)
    assert code_of(lambda: B._check(B.load().en_plan_values_from_pool(plan.handle, 2))) == 1
    assert code_of(lambda: B._check(B.load().en_plan_values_from_pool(None, 1))) == 1
    # so few new tokens that the step runs in the decode kernel (4 heads per KV head x 2 rows fit one wave)
    few = B.segment_select(ok, [1], [0, 1], 2)
    assert code_of(lambda: few.values_from_pool(True)) == 5
    few.values_from_pool(False)             # switching it off is always allowed
    # float32 and 8-bit pools keep their gathered values
    for kw in (dict(dtype=B.EN_F32, shape=(3, 2, 8, 128)), dict(dtype=B.EN_I8, shape=(3, 2, 8, 128))):
        pool = B.kv_pool_create(None, None, lens, 8, 1e4, 256, k_ptr=0x1000, v_ptr=0x2000, **kw)
        p = B.segment_select(pool, [2, 0], [0, 2], 40)
        assert code_of(lambda: p.values_from_pool(True)) == 5
    # value rows are fetched whole: aligned to a row (256 bytes with 128-wide heads, 128 with 64-wide ones)
    odd = B.kv_pool_create(None, None, lens, 8, 1e4, 256, dtype=B.EN_BF16, k_ptr=0x1000, v_ptr=0x2080,
                           shape=(3, 2, 8, 128))
    p = B.segment_select(odd, [2, 0], [0, 2], 40)
    assert code_of(lambda: p.values_from_pool(True)) == 1
    d64 = B.kv_pool_create(None, None, lens, 8, 1e4, 256, dtype=B.EN_BF16, k_ptr=0x1000, v_ptr=0x2080,
                           shape=(3, 2, 8, 64))
    B.segment_select(d64, [2, 0], [0, 2], 40).values_from_pool(True)
    d64o = B.kv_pool_create(None, None, lens, 8, 1e4, 256, dtype=B.EN_BF16, k_ptr=0x1000, v_ptr=0x2040,
                            shape=(3, 2, 8, 64))
    p = B.segment_select(d64o, [2, 0], [0, 2], 40)
    assert code_of(lambda: p.values_from_pool(True)) == 1
