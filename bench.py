#!/usr/bin/env python3
"""Benchmark of the segmented-attention planning step on one MI355X.

A step is one pass of the whole hot path over one synthetic workload:
segment_select (host plan + descriptor upload) -> gather_rope ->
segmented_prefill_attention (+ split combine) -> segment_attention_mass
(reduced over heads and queries). Inputs are resident in HBM before the timed
region. Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2]

The default workload is the 8K-context configuration (32 segments x 256 cached
tokens + 512 new tokens, Llama-3.2-11B-shaped layer, bf16), the one the
matrix-core target is quoted on.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "segmented prefill attention TFLOP/s + µs per planning step, % bf16 MFMA peak"
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E

WORKLOAD_TEXT = {
    "c1": "c1: 32q/8kv heads, D=128, bf16; 16 ragged segments (64..128 tokens) of a 64-group pool + 256 new tokens",
    "c2": "c2: 32q/8kv heads, D=128, bf16; 32 segments x 256 cached tokens (8192) of a 256-group pool + 512 new tokens; mass summed over heads and queries",
    "c3": "c3: 16 agents sharing a 512-group pool; 24 ragged segments (32..128 tokens) + 128 new tokens each; 32q/8kv, D=128, bf16",
    "c5": "c5: c2's map on a LLaVA-34b-shaped layer: 56q/8kv heads, D=128, bf16; 32 segments x 256 cached tokens + 512 new tokens",
    "c4": "c4: decode, 64 agents x 1 new token over 64 segments x 256 tokens (16384) from a 1024-group pool; 32q/8kv, D=128, bf16",
}

# HBM bytes from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs, each scaled by what the same counter
# reads for a plain copy of known size: per launch of the dominant kernel, and per whole planning step
# (all its launches). Stored figures, re-measured when a kernel changes; the profile named holds the
# commands and the counters.
MEASURED_TRAFFIC = {
    "c2": {"kernel": 62.4e6, "step": 181.6e6, "source": "profiles/attn_bf16_c2_hbm_traffic.md"},
    "c4": {"kernel": 4.318e9, "step": None, "source": "profiles/attn_decode_c4_hbm_traffic.md"},
}


def algorithmic_flops(cfg, info) -> int:
    """4*Hq*D per visible (query, key) pair; causal triangle counted once."""
    return 4 * cfg.n_q_heads * cfg.head_dim * int(info.total_pairs)


def step_traffic(name, cfg, info):
    alg = algorithmic_bytes(cfg, info) + 2 * cfg.n_agents * cfg.n_new * cfg.n_kv_heads * cfg.head_dim * 2
    t = MEASURED_TRAFFIC.get(name, {})
    return {"algorithmic_bytes": alg, "measured_bytes": t.get("step"),
            "ratio": (t["step"] / alg) if t.get("step") else None, "source": t.get("source")}


def algorithmic_bytes(cfg, info) -> int:
    """Bytes the attention kernel must move once: gathered K and V^T of the
    visible context, Q in, O out (2-byte elements)."""
    es = 2 if cfg.dtype == 1 else 4
    kv = 2 * cfg.n_kv_heads * cfg.head_dim * (int(info.total_cached) + cfg.n_agents * cfg.n_new) * es
    qo = 2 * cfg.n_agents * cfg.n_new * cfg.n_q_heads * cfg.head_dim * es
    return kv + qo


def measure_ceilings(torch, B) -> dict:
    """Measured ceilings of this machine beside the nominal peaks. The library's own two kernels: a loop of bf16
    matrix instructions and nothing else (on operands with the bits of normal-distributed data and on constant
    operands: the chip's clock depends on how many bits toggle), and a read-only stream. For comparison the
    vendor's large bf16 GEMM on both kinds of data, and a plain device copy."""
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros(n_cu * 512, dtype=torch.float32, device="cuda:0")
    mfma = {}
    for label, const in (("normal_data", False), ("constant_data", True)):
        fl = B.ceiling_mfma_bf16(sink, n_cu, 2000, const)
        mfma[label] = fl / timed(lambda: B.ceiling_mfma_bf16(sink, n_cu, 2000, const), 20) / 1e12
    nb = 1 << 30
    src = torch.empty(nb, dtype=torch.uint8, device="cuda:0").fill_(3)
    t_read = timed(lambda: B.ceiling_read_stream(src, sink, n_cu * 8), 10)
    dst = torch.empty_like(src)
    t_copy = timed(lambda: dst.copy_(src), 10)
    del dst, src
    n = 8192
    a = torch.randn(n, n, device="cuda:0").to(torch.bfloat16)
    b = torch.randn(n, n, device="cuda:0").to(torch.bfloat16)
    c = torch.empty(n, n, device="cuda:0", dtype=torch.bfloat16)
    t_gemm = timed(lambda: torch.matmul(a, b, out=c), 20)
    ones = torch.ones(n, n, device="cuda:0", dtype=torch.bfloat16)
    t_gemm1 = timed(lambda: torch.matmul(ones, ones, out=c), 20)
    return {
        "mfma_only_bf16_tflops": mfma["normal_data"],
        "mfma_only_bf16_constant_operands_tflops": mfma["constant_data"],
        "read_stream_gbs": nb / t_read / 1e9,
        "vendor_gemm_bf16_8192_normal_data_tflops": 2.0 * n ** 3 / t_gemm / 1e12,
        "vendor_gemm_bf16_8192_constant_data_tflops": 2.0 * n ** 3 / t_gemm1 / 1e12,
        "copy_1GiB_read_plus_write_gbs": 2.0 * nb / t_copy / 1e9,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=sorted(WORKLOAD_TEXT))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the measured ceilings reported under 'ceilings' (the library's loop of matrix "
                         "instructions only and its read-only stream, the vendor's bf16 GEMM, a device copy)")
    ap.add_argument("--ceilings", action="store_true", help="print the measured ceilings only")
    ap.add_argument("--no-residency", action="store_true",
                    help="skip the residency-tier figures (hit rate against the device budget, planning "
                         "steps whose groups are loaded from the host store) reported under 'residency'")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="with the default workload, skip the brief figures of c1, c3, c4 and c5 reported under "
                         "'other_workloads'")
    ap.add_argument("--five-calls", action="store_true",
                    help="time the step as the five calls gather_rope / segmented_prefill_attention / "
                         "segment_attention_mass (queries rotated inside the attention kernel, reduced masses "
                         "by a launch of their own) instead of gather_rope_queries + "
                         "segmented_prefill_attention_prepared: the before/after of those two changes")
    ap.add_argument("--values-from-pool", action="store_true",
                    help="prefill-only form of the step: the values are not gathered, the attention kernel fetches "
                         "them from the pool's blocks (en_plan_values_from_pool); the decode phase that the line "
                         "also reports gathers its own context either way")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain device copy of known size instead (scales the FETCH_SIZE / "
                         "WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (every agent, head and segment of a planning "
                 "step lives on it); --gpus must be 1")

    import numpy as np
    import torch
    from paper_2510_18546_amd import binding as B
    from paper_2510_18546_amd import inputs as I
    from paper_2510_18546_amd import step

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.copy_calibration:
        n = 256 << 20
        src = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read_per_copy": n, "bytes_written_per_copy": n,
                          "copies": 5}))
        return
    if args.ceilings:
        print(json.dumps({"ceilings": measure_ceilings(torch, B)}))
        return
    def time_workload(name, steps, warmup, values_from_pool=args.values_from_pool):
        """K whole planning steps of one workload, inputs resident; the attention kernel's own
        duration from HIP events around its launches, on the stream it is launched on."""
        cfg = I.CONFIGS[name]
        w = I.make_workload(cfg)
        st = step.PlanningStep(w, prepared=False if args.five_calls else None,
                               values_from_pool=values_from_pool and cfg.n_new > 1)
        info = st.info
        flops = algorithmic_flops(cfg, info)
        hbm_bound = cfg.n_new == 1

        def one_step():
            st.select()
            st.gather()                       # with the queries prepared in the same launch (prefill workloads)
            if st.prepared:
                st.attention(True)            # ... and the reduced masses out of the attention call
            else:
                st.attention()
                st.masses(1)

        for _ in range(warmup):
            one_step()
        torch.cuda.synchronize()
        B.timing_enable(st.pool, steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            one_step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        kern_ms = B.timing_collect(st.pool, steps)
        B.timing_enable(st.pool, 0)
        sec_per_step = (t1 - t0) / steps
        kern_s = float(np.mean(kern_ms)) * 1e-3
        if hbm_bound:
            abytes = algorithmic_bytes(cfg, info)
            roof = {"bound": "hbm", "achieved": abytes / kern_s / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
        else:
            roof = {"bound": "mfma", "achieved": flops / kern_s / 1e12, "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s"}
        roof["frac"] = roof["achieved"] / roof["peak"]
        # HBM bytes per launch of this kernel: a stored figure from rocprofv3 --pmc runs (FETCH_SIZE and
        # WRITE_SIZE, each scaled by what it reads for a plain copy), not something this run measures
        roof["traffic"] = MEASURED_TRAFFIC.get(name, {}).get("kernel")
        roof["traffic_source"] = MEASURED_TRAFFIC.get(name, {}).get("source")
        roof["kernel"] = ("attn_decode_kernel<128, 1>" if hbm_bound else
                          "attn_bf16_kernel<128, %s, %s>" % ("true" if st.prepared else "false",
                                                             "true" if st.values_from_pool else "false"))
        roof["kernel_us"] = kern_s * 1e6
        roof["kernel_us_min"] = float(np.min(kern_ms)) * 1e3
        return cfg, w, st, info, flops, hbm_bound, sec_per_step, roof

    cfg, w, st, info, flops, hbm_bound, sec_per_step, roof = time_workload(args.workload, args.steps, args.warmup)
    value = flops / sec_per_step / 1e12

    res = {
        "metric": METRIC, "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": sec_per_step * 1e3,
        "us_per_planning_step": sec_per_step * 1e6,
        "pct_bf16_mfma_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.workload], "n_splits": int(info.n_splits),
                   "flops_per_step": flops, "cached_tokens": int(info.total_cached),
                   "new_tokens": cfg.n_new, "agents": cfg.n_agents,
                   "values": "left in the pool (en_plan_values_from_pool)" if st.values_from_pool else "gathered",
                   "entry_points": ("segment_select, gather_rope_queries, segmented_prefill_attention_prepared"
                                    if st.prepared else
                                    "segment_select, gather_rope, segmented_prefill_attention, "
                                    "segment_attention_mass")},
        "roofline": roof,
        # the whole step's HBM traffic (stored profile figure) against the bytes the method must move once:
        # selected K+V read once, Q, O, new K/V (2-byte elements)
        "step_traffic": step_traffic(args.workload, cfg, info),
        # the paper's own figures, other hardware, whole planner: context only, never a target
        "paper_context": "EfficientNav-11b (40-layer LLaMA-3.2-11b planner): 0.35 s planning latency per "
                         "navigation step on 1x RTX A6000 vs 3.07 s naive and 2.27 s vLLM (Table 3); prefill "
                         "time reduced about 20x by discrete memory caching (Fig. 9). This benchmark is one "
                         "attention layer of that step, not comparable in absolute terms.",
    }

    if not hbm_bound and st.prepared:
        # The step's GPU launches (gather with the queries, attention with the merge and the reduced masses) as one
        # HIP graph on the plan of the last step: what the launches cost without the host between them. The
        # selection, which is host work, stays outside; `value` above is the eager step with it.
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g_step = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g_step, stream=side):
                st.gather()
                st.attention(True)
        torch.cuda.synchronize()
        for _ in range(5):
            g_step.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(args.steps):
            g_step.replay()
        torch.cuda.synchronize()
        g1 = time.perf_counter()
        res["launches_as_a_graph"] = {"us_per_step": (g1 - g0) / args.steps * 1e6, "steps": args.steps,
                                      "what": "gather_rope_queries + segmented_prefill_attention_prepared on one plan"}
        del g_step

    if hbm_bound:
        # Decode-phase reuse as the paper runs it: the context is gathered ONCE, then 40 tokens are decoded
        # over it, each step appending its key/value and attending (segmented_decode_step); timed eagerly
        # and as one HIP graph of the 40 steps.
        n_dec = 40
        pool_d = B.kv_pool_create(st.k_pool, st.v_pool, w.lens, cfg.n_q_heads, cfg.rope_base,
                                  cfg.n_sel * cfg.capacity + n_dec)      # same arrays, room for 40 new tokens
        plan_d = B.segment_select(pool_d, w.sel, w.sel_ptr, n_dec)
        kc_d, vt_d = B.alloc_context(pool_d, plan_d)
        gen = torch.Generator(device="cuda:0").manual_seed(5)
        dt = torch.bfloat16
        qd = torch.randn((cfg.n_agents, n_dec, cfg.n_q_heads, cfg.head_dim), generator=gen, device="cuda:0").to(dt)
        kd = torch.randn((cfg.n_agents, n_dec, cfg.n_kv_heads, cfg.head_dim), generator=gen, device="cuda:0").to(dt)
        vd = torch.randn((cfg.n_agents, n_dec, cfg.n_kv_heads, cfg.head_dim), generator=gen, device="cuda:0").to(dt)
        qs = [qd[:, i:i + 1].contiguous() for i in range(n_dec)]
        ks = [kd[:, i:i + 1].contiguous() for i in range(n_dec)]
        vs = [vd[:, i:i + 1].contiguous() for i in range(n_dec)]
        od = [torch.empty_like(q) for q in qs]
        ws_d = torch.empty(max(B.decode_workspace_bytes(pool_d, plan_d, 1), 256), dtype=torch.uint8, device="cuda:0")
        B.gather_rope(pool_d, plan_d, torch.zeros_like(kd), torch.zeros_like(vd), kc_d, vt_d)

        def decode_all():
            for i in range(n_dec):
                B.segmented_decode_step(pool_d, plan_d, i, qs[i], ks[i], vs[i], kc_d, vt_d, od[i], ws_d)
        decode_all()
        torch.cuda.synchronize()
        B.timing_enable(pool_d, n_dec)
        d0 = time.perf_counter()
        decode_all()
        torch.cuda.synchronize()
        d1 = time.perf_counter()
        dec_kern_ms = B.timing_collect(pool_d, n_dec)
        B.timing_enable(pool_d, 0)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                decode_all()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        g1 = time.perf_counter()
        kv_bytes = 2 * cfg.n_kv_heads * cfg.head_dim * 2 * (int(info.total_cached) + cfg.n_agents * n_dec / 2)
        res["decode_reuse"] = {
            "tokens_decoded": n_dec, "context_gathered": "once",
            "us_per_decode_step_eager": (d1 - d0) / n_dec * 1e6,
            "us_per_decode_step_graph": (g1 - g0) / n_dec * 1e6,
            "attention_kernel_us": float(np.mean(dec_kern_ms)) * 1e3,
            "hbm_gbs_graph": kv_bytes / ((g1 - g0) / n_dec) / 1e9,
        }
        plan_d.close()
        pool_d.close()

    if not hbm_bound:
        # The decode phase that follows the prefill (Section 3.2: about 40 tokens per plan, over the KV that was
        # loaded once): the context holds the cached segments and the prompt tokens; each step appends its
        # key/value and attends (segmented_decode_step), eagerly and as one HIP graph of the 40 steps.
        n_dec = 40
        n_all = cfg.n_new + n_dec
        pool_d = B.kv_pool_create(st.k_pool, st.v_pool, w.lens, cfg.n_q_heads, cfg.rope_base,
                                  int(info.max_ctx_len) + n_dec)
        plan_d = B.segment_select(pool_d, w.sel, w.sel_ptr, n_all)
        kc_d, vt_d = B.alloc_context(pool_d, plan_d)
        dt = torch.bfloat16
        gen = torch.Generator(device="cuda:0").manual_seed(5)
        shp = (cfg.n_agents, n_dec, cfg.n_kv_heads, cfg.head_dim)
        qd = torch.randn((cfg.n_agents, n_dec, cfg.n_q_heads, cfg.head_dim), generator=gen, device="cuda:0").to(dt)
        kd = torch.randn(shp, generator=gen, device="cuda:0").to(dt)
        vd = torch.randn(shp, generator=gen, device="cuda:0").to(dt)
        B.gather_rope(pool_d, plan_d, torch.cat([st.k_new, torch.zeros_like(kd)], 1).contiguous(),
                      torch.cat([st.v_new, torch.zeros_like(vd)], 1).contiguous(), kc_d, vt_d)
        qs = [qd[:, i:i + 1].contiguous() for i in range(n_dec)]
        ks = [kd[:, i:i + 1].contiguous() for i in range(n_dec)]
        vs = [vd[:, i:i + 1].contiguous() for i in range(n_dec)]
        od = [torch.empty_like(q) for q in qs]
        ws_d = torch.empty(max(B.decode_workspace_bytes(pool_d, plan_d, 1), 256), dtype=torch.uint8, device="cuda:0")

        def decode_all():
            for i in range(n_dec):
                B.segmented_decode_step(pool_d, plan_d, cfg.n_new + i, qs[i], ks[i], vs[i], kc_d, vt_d, od[i], ws_d)
        decode_all()
        torch.cuda.synchronize()
        B.timing_enable(pool_d, n_dec)
        d0 = time.perf_counter()
        decode_all()
        torch.cuda.synchronize()
        d1 = time.perf_counter()
        dec_kern_ms = B.timing_collect(pool_d, n_dec)
        B.timing_enable(pool_d, 0)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                decode_all()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(5):
            graph.replay()
        torch.cuda.synchronize()
        g1 = time.perf_counter()
        # bytes a decoded token must read once: K and V of the context (the prompt and, on average, half of
        # the decoded tokens included), every KV head
        dec_bytes = 2 * cfg.n_kv_heads * cfg.head_dim * 2 * cfg.n_agents * (int(info.max_ctx_len) + n_dec / 2)
        us_graph = (g1 - g0) / 5 / n_dec * 1e6
        us_attn = float(np.mean(dec_kern_ms)) * 1e3
        res["decode_after_prefill"] = {
            "tokens_decoded": n_dec, "context_tokens": int(info.max_ctx_len),
            "us_per_decode_step_eager": (d1 - d0) / n_dec * 1e6,
            "us_per_decode_step_graph": us_graph,
            "attention_kernel_us": us_attn,
            "context_bytes_per_step": dec_bytes,
            "hbm_floor_us": dec_bytes / (PEAK_HBM_GBS * 1e9) * 1e6,
            "frac_of_hbm_peak_step": dec_bytes / (us_graph * 1e-6) / (PEAK_HBM_GBS * 1e9),
            "frac_of_hbm_peak_attention_kernel": dec_bytes / (us_attn * 1e-6) / (PEAK_HBM_GBS * 1e9),
            "us_prefill_step_plus_40_decode_steps": sec_per_step * 1e6 + (g1 - g0) / 5 * 1e6,
        }
        del graph
        plan_d.close()
        pool_d.close()

    # (on workloads whose groups all have the slot's length: with ragged groups the token budget of
    # Eq. (1) selects more groups than the workload's own plan, scratch and slots are sized for)
    if not hbm_bound and cfg.n_agents == 1 and cfg.len_lo == cfg.len_hi and not args.no_residency:
        # Residency tier (Section 3.2, Section 4 "cache hit rate"): every group's K/V lives in a pinned host
        # store, the device holds a budget of slots, a step loads only the selected groups that are not
        # there. Selections: Eq. (1) over relevance scores that drift slowly from step to step.
        G, n_sel, T = cfg.n_groups, cfg.n_sel, 120
        rho = 0.98
        scores = I.drifting_scores(cfg.seed + 100, G, T, rho=rho)
        blk = (cfg.n_kv_heads, cfg.capacity, cfg.head_dim)

        def book_tier(n_slots):
            t = B.kv_tier_create(None, None, G, cfg.n_q_heads, cfg.rope_base, 1, dtype=B.EN_BF16,
                                 shape=(n_slots,) + blk)
            for g in range(G):
                B.kv_tier_put(t, g, None, None, int(w.lens[g]))
            return t
        t0_ = book_tier(n_sel)
        sels = [B.kv_tier_select_scored(t0_, scores[t], -8.0, n_sel * cfg.capacity) for t in range(T)]
        t0_.close()
        slot_mb = B.kv_tier_slot_bytes(blk, B.EN_BF16) / 1e6
        curve = []
        for n_slots in sorted({n_sel, n_sel * 5 // 4, n_sel * 3 // 2, n_sel * 2, n_sel * 3, n_sel * 4, G}):
            t_ = book_tier(n_slots)
            for sel in sels:
                B.kv_tier_fetch(t_, sel)
            curve.append({"slots": n_slots, "device_budget_MB": n_slots * slot_mb,
                          "hit_rate": t_.stats.hits / t_.stats.requested})
            t_.close()

        n_slots = 2 * n_sel
        dt = torch.bfloat16
        k_slots = torch.zeros((n_slots,) + blk, dtype=dt, device="cuda:0")
        v_slots = torch.zeros((n_slots,) + blk, dtype=dt, device="cuda:0")
        tier = B.kv_tier_create(k_slots, v_slots, G, cfg.n_q_heads, cfg.rope_base,
                                cfg.n_sel * cfg.capacity + cfg.n_new)
        for g in range(G):
            n = int(w.lens[g])
            kh = torch.from_numpy(I.bf16_bits(np.ascontiguousarray(w.k_pool[g, :, :n])).view(np.int16)).view(dt)
            vh = torch.from_numpy(I.bf16_bits(np.ascontiguousarray(w.v_pool[g, :, :n])).view(np.int16)).view(dt)
            B.kv_tier_put(tier, g, kh, vh)

        def tier_steps(ahead, sels=sels):
            plans = []
            T = len(sels)
            for t, sel in enumerate(sels):
                slots = B.kv_tier_fetch(tier, sel)
                plan = B.segment_select(tier.pool, slots, [0, len(slots)], cfg.n_new)
                assert B.context_bytes(tier.pool, plan) <= st.kc.numel() * st.kc.element_size()
                B.gather_rope(tier.pool, plan, st.k_new, st.v_new, st.kc, st.vt)
                B.kv_tier_fence(tier)
                if ahead and t + 1 < T:
                    B.kv_tier_prefetch(tier, sels[t + 1])
                B.segmented_prefill_attention(tier.pool, plan, st.q, st.kc, st.vt, st.out, st.ws)
                B.segment_attention_mass(tier.pool, plan, st.ws, 1, st.mass_red)
                plans.append(plan)
            torch.cuda.synchronize()
            for p_ in plans:
                p_.close()

        timed_tier = {}
        for name, ahead in (("on_demand", False), ("selection_known_one_step_ahead", True)):
            tier_steps(ahead)                   # warm: slots filled, steady state
            before = tier.stats
            b0 = (before.hits, before.prefetched, before.misses, before.bytes_loaded, before.requested)
            r0 = time.perf_counter()
            tier_steps(ahead)
            r1 = time.perf_counter()
            a = tier.stats
            req = a.requested - b0[4]
            timed_tier[name] = {
                "us_per_planning_step": (r1 - r0) / T * 1e6,
                "hit_rate": (a.hits - b0[0]) / req, "prefetched_rate": (a.prefetched - b0[1]) / req,
                "groups_loaded_late_per_step": (a.misses - b0[2]) / T,
                "MB_loaded_per_step": (a.bytes_loaded - b0[3]) / T / 1e6,
            }
        # nothing resident: three disjoint selections in turn displace one another in 2 * n_sel slots
        cold = [np.arange(i * n_sel, (i + 1) * n_sel, dtype=np.int32) for i in range(3)] * 10
        tier_steps(False, cold)
        b0 = tier.stats
        r0 = time.perf_counter()
        tier_steps(False, cold)
        r1 = time.perf_counter()
        a = tier.stats
        assert a.hits == b0.hits and a.prefetched == b0.prefetched
        timed_tier["nothing_resident"] = {
            "us_per_planning_step": (r1 - r0) / len(cold) * 1e6, "hit_rate": 0.0,
            "MB_loaded_per_step": (a.bytes_loaded - b0.bytes_loaded) / len(cold) / 1e6,
            "host_to_device_GBs_incl_step": (a.bytes_loaded - b0.bytes_loaded) / (r1 - r0) / 1e9,
        }
        res["residency"] = {
            "store_groups": G, "selected_per_step": n_sel, "steps": T, "score_drift_rho": rho,
            "slot_MB": slot_mb, "hit_rate_vs_device_budget": curve,
            "timed_slots": n_slots, "timed": timed_tier,
            "all_resident_us_per_planning_step": sec_per_step * 1e6,
        }
        tier.close()
        del k_slots, v_slots

    if hbm_bound:
        # 8-bit pool (an option beside the paper's method): the same gather from int8 codes and per-row scales,
        # quantised by the library's own append; the context it writes is the same bf16 one.
        G, Hkv, Cap, D = st.k_pool.shape
        kq = torch.zeros((G, Hkv, Cap, D), dtype=torch.int8, device="cuda:0")
        vq = torch.zeros_like(kq)
        ks = torch.zeros((G, Hkv, Cap), dtype=torch.float32, device="cuda:0")
        vs = torch.zeros_like(ks)
        pool_q = B.kv_pool_create(kq, vq, np.zeros(G, np.int32), cfg.n_q_heads, cfg.rope_base,
                                  cfg.n_sel * cfg.capacity + cfg.n_new)
        B.kv_pool_set_scales(pool_q, ks, vs)
        for g in range(G):
            n = int(w.lens[g])
            B.kv_pool_append(pool_q, g, st.k_pool[g, :, :n].permute(1, 0, 2).contiguous(),
                             st.v_pool[g, :, :n].permute(1, 0, 2).contiguous())
        plan_q = B.segment_select(pool_q, w.sel, w.sel_ptr, cfg.n_new)
        torch.cuda.synchronize()

        def time_gather(pool, plan, reps=5):
            B.gather_rope(pool, plan, st.k_new, st.v_new, st.kc, st.vt)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                B.gather_rope(pool, plan, st.k_new, st.v_new, st.kc, st.vt)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / reps
        t_bf16 = time_gather(st.pool, st.plan)
        t_q8 = time_gather(pool_q, plan_q)
        res["q8_pool"] = {"gather_us_bf16_pool": t_bf16, "gather_us_int8_pool": t_q8,
                          "pool_bytes_ratio": (kq.numel() + ks.numel() * 4) / (st.k_pool.numel() * 2)}
        plan_q.close()
        pool_q.close()
        del kq, vq, ks, vs

    if args.workload == "c2" and not args.no_other_workloads:
        # the other workloads in brief, from the same run (each has a full line of its own under --workload)
        del st, w
        other = {}
        for name in ("c1", "c3", "c5", "c4"):
            o_cfg, o_w, o_st, o_info, o_flops, o_hbm, o_sec, o_roof = time_workload(name, 100, 10)
            other[name] = {"workload": WORKLOAD_TEXT[name], "us_per_planning_step": o_sec * 1e6,
                           "value_tflops": o_flops / o_sec / 1e12, "n_splits": int(o_info.n_splits),
                           "roofline": o_roof}
            del o_w, o_st
            torch.cuda.empty_cache()
        res["other_workloads"] = other
        if not args.values_from_pool:
            # Steps that no decode phase follows (the clustering passes of Section 3.3) can leave the values
            # where they are (en_plan_values_from_pool: the attention kernel fetches them from the pool's
            # blocks, bit-identical results): the same steps in that form, same run.
            vp = {}
            for name in ("c2", "c3"):
                o_cfg, o_w, o_st, o_info, o_flops, o_hbm, o_sec, o_roof = time_workload(name, 100, 10, True)
                vp[name] = {"us_per_planning_step": o_sec * 1e6, "value_tflops": o_flops / o_sec / 1e12,
                            "attention_kernel_us": o_roof["kernel_us"]}
                del o_w, o_st
                torch.cuda.empty_cache()
            res["prefill_only_values_from_pool"] = vp
        cfg = I.CONFIGS[args.workload]
        w = I.make_workload(cfg)

    if not args.no_ceilings:
        res["ceilings"] = measure_ceilings(torch, B)
        measured = res["ceilings"]["read_stream_gbs"] if hbm_bound else res["ceilings"]["mfma_only_bf16_tflops"]
        roof["measured_ceiling"] = measured
        roof["frac_of_measured_ceiling"] = roof["achieved"] / measured

    if not args.no_cpu_baseline:
        # The float64 oracle, as it stands, on the host cores: the whole workload
        # when it is small enough, otherwise a bounded sample of output rows.
        from oracle import oracle as O
        O.build()
        rows_total = cfg.n_agents * cfg.n_new * cfg.n_q_heads
        per_row = flops / rows_total
        n = rows_total if flops <= 8e10 and cfg.n_agents == 1 else min(rows_total, 2048)
        rng = np.random.default_rng(9)
        if n == rows_total and cfg.n_agents == 1:
            rows, sample = None, f"all {rows_total} output rows of the workload"
        else:
            agents = rng.integers(0, min(cfg.n_agents, 4), n)
            rows = np.stack([agents, rng.integers(0, cfg.n_new, n),
                             rng.integers(0, cfg.n_q_heads, n)], 1).astype(np.int32)
            sample = (f"{n} of {rows_total} output rows (agent, query, head drawn uniformly from the "
                      f"first {min(cfg.n_agents, 4)} agents, seed 9), each agent's gather+RoPE included")
        c0 = time.perf_counter()
        O.attention(w.k_pool, w.v_pool, w.lens, w.sel, w.sel_ptr, w.q, w.k_new, w.v_new,
                    cfg.rope_base, rows=rows)
        c1 = time.perf_counter()
        res["cpu_baseline"] = {"value": per_row * n / (c1 - c0) / 1e12, "unit": "TFLOP/s",
                               "cores": O.threads(), "kind": "oracle", "sample": sample,
                               "seconds": c1 - c0}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
