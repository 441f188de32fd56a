// Internal declarations shared by the host planner and the HIP kernels of
// libefficientnav.so. Not part of the public ABI (that is include/efficientnav.h).
#pragma once

#include <cstddef>
#include <cstdint>
#include <new>
#include <utility>
#include <vector>

#include <hip/hip_runtime_api.h>

#include "efficientnav.h"

constexpr int EN_KEY_TILE = 64;    // keys per attention tile; context rows are padded to it
constexpr int EN_ROWS_PER_WAVE = 32;
constexpr int EN_WAVES = 8;          // waves per attention workgroup

struct en_pool {
    en_pool_desc d;
    void *k_dev = nullptr;
    void *v_dev = nullptr;
    float *k_scale = nullptr;     // EN_I8 pools: one scale per (group, head, token)
    float *v_scale = nullptr;
    std::vector<int32_t> len;     // current lengths [G]
    int r = 1;                    // Hq / Hkv
    // device side, created on first GPU use
    float *d_cos = nullptr;       // [max_ctx, D/2]
    float *d_sin = nullptr;
    int n_cu = 256;
    // descriptor blocks of destroyed plans, kept for reuse (bytes, pointer)
    mutable std::vector<std::pair<size_t, int32_t *>> desc_cache;
    // plans made on this pool and not yet destroyed: a pool that is destroyed
    // first cuts them loose, so that destroying them later stays safe
    mutable std::vector<struct en_plan *> plans;
    // measurement aid (en_timing_*): event pairs around the attention kernel of the calls on this pool
    std::vector<hipEvent_t> ev_start, ev_stop;
    int ev_used = 0;
};

struct en_plan {
    const en_pool *pool = nullptr;
    int B = 0, Nq = 0, Smax = 0;
    int ctx_stride = 0, max_ctx_len = 0, n_splits = 1;
    int64_t total_pairs = 0, total_cached = 0;
    // host descriptors (uniform stride per agent)
    std::vector<int32_t> nseg;    // [B]
    std::vector<int32_t> sel;     // [B, Smax]   (-1 padded)
    std::vector<int32_t> bnd;     // [B, Smax+2] bucket bounds: offset[0..S], then L_c+N_q
    std::vector<int32_t> hdr;     // [B, 4] S, L_c, L_c+N_q, 0: what a workgroup needs first, in one load
    // device block: nseg | sel | bnd | hdr, created on first GPU use
    int32_t *d_desc = nullptr;
    size_t d_desc_bytes = 0;
    std::vector<int32_t> h_desc;  // staging copy, alive as long as the plan
    bool uploaded = false;
    // behind the tables in the device block: B * (Smax + 1) 64-bit accumulators of the reduced masses
    // that the prefill attention kernel adds up itself (EnAttnArgs::red_direct). Zero when the block is
    // filled; whoever completes a sum sets its word back to zero.
    size_t acc_off = 0;           // in ints from d_desc
    // en_plan_values_from_pool: the gather leaves the values where they are (EnGatherArgs::v_rows)
    bool values_from_pool = false;
    int gathered_values_from_pool = -1;      // mode of the last gather on this plan, -1: none yet
};

// Arguments of the device kernels (plain data, passed by value).
struct EnGatherArgs {
    const void *k_pool, *v_pool, *k_new, *v_new;
    void *kc, *vt;
    const float *cos_tab, *sin_tab;
    const int32_t *nseg, *sel, *bnd;
    int B, Hkv, C, Nq, Smax, T;
    const float *k_scale, *v_scale;    // EN_I8 pools only
    // queries to prepare in the same launch, or null: q [B, Nq, Hq, D] unrotated ->
    // q_prep, rotated at L_c + i, scaled by scale_log2e, bf16
    const void *q;
    void *q_prep;
    int Hq;
    // units (along grid y) that share an agent's query rows with the 64-token tiles along x: a
    // workgroup takes its rows 16 at a time, one dependent round of loads each, so few rows per
    // workgroup keep the query units from outlasting the key and value streams of a small step
    int n_q_units;
    float scale_log2e;
    // 1 (bf16, D = 128): the values stay where they are. vt receives, per (agent, KV head, context
    // row up to the end of the last 64-row tile), the 8-byte address of the row's values in the
    // pool or the new tokens, [B, Hkv, T], and behind that table one row of zeros, which the
    // padding rows of an agent's last tile point at.
    int v_rows;
};

// Bytes of the row-address table of EnGatherArgs::v_rows (the row of zeros follows it).
constexpr size_t en_v_rows_table_bytes(int B, int Hkv, int T)
{
    return ((size_t)B * Hkv * T * 8 + 255) / 256 * 256;
}

// The gather launch can carry a small plan's descriptor block inside its kernel
// arguments: the kernel reads the descriptors from there and one workgroup
// stores them to the plan's device block for the kernels that follow, which
// saves the separate host-to-device copy.
constexpr int EN_INLINE_DESC_MAX = 960;      // ints; keeps the argument block under 4 KB
struct EnGatherLaunch {
    EnGatherArgs a;
    int n_inline;           // ints of `desc` in use, 0: read the device block
    int n_zero;             // ints to set to zero behind them in the device block (the plan's accumulators)
    int off_nseg, off_sel, off_bnd;   // int offsets of the three tables in the block
    int32_t *desc_out;      // device block to fill when n_inline > 0
    int32_t desc[EN_INLINE_DESC_MAX];
};

struct EnAttnArgs {
    const void *q, *kc, *vt;
    void *out;
    const float *cos_tab, *sin_tab;
    const int32_t *nseg, *bnd, *hdr;
    float *ws_ml;      // [n_splits, B*Hq*Nq, 2]  (reference max in log2 units, sum)
    float *ws_seg;     // [n_splits, B*Hq, Smax+1, Nq, 2] (partial sum, its reference max)
    void *ws_opart;    // [n_splits, B*Hq*Nq, D] per-split softmax outputs (pool dtype)
    float *ws_mlfin;   // [B*Hq*Nq, 2] merged (reference, sum), written by the combine kernel
    int B, Hq, Hkv, Nq, Smax, T;
    int q_first;       // the Nq query rows are new tokens q_first .. q_first+Nq-1 of the plan: every key
                       // before L_c + q_first is visible to all of them (0 for a whole prefill)
    int n_splits, n_ptiles, total_wgs;
    int decode;        // 1: all r*Nq query rows of a KV head fit one wave (attn_decode kernel)
    int sub;           // decode kernel: waves per (agent, KV head, split); wave w takes every sub-th 32-key
                       // block of the split's tiles and leaves its own partial results at index
                       // sp * sub + w of n_splits * sub
    float scale_log2e;
    int q_prepared;    // prefill kernel: q holds prepared queries (rotated, scaled, bf16: see EnGatherArgs)
    int v_rows;        // prefill kernel: vt holds no values but the address of every context row's values
                       // (see EnGatherArgs::v_rows)
    // prefill kernel, or null: n_red_zero accumulator words that its first workgroup sets to zero
    // (EnMassArgs::red_acc, which the launches after it add to)
    unsigned long long *red_zero;
    int n_red_zero;
    // prefill kernel with one KV split, or null: the reduced masses [B, Smax+1] without any further
    // launch. Every workgroup adds, per bucket, the masses of its rows to red_direct (fixed point,
    // 2^-red_shift, above a 10-bit count of arrivals, as in EnMassArgs); the one that sees
    // red_target arrivals writes the sum to red_direct_out and sets the word back to zero.
    unsigned long long *red_direct;
    float *red_direct_out;
    int red_shift, red_target;
    // decode kernel only, or null: the rows' own keys / values [B, Nq, Hkv, D], which the kernel
    // writes into the context (kc, vt) at positions L_c + q_first + t before it reads them
    const void *app_k, *app_v;
};

struct EnMassArgs {
    const float *ws_ml, *ws_seg, *ws_mlfin;
    float *ws_red;          // [B, Smax+1, Hq] per-head partial sums of the reduced masses
    // Reduced masses without a launch of their own, or null: every per-head partial sum is also added,
    // as a fixed-point integer (2^-red_shift; integer sums do not depend on the order of the
    // additions), to red_acc [B, Smax+1], whose low 10 bits count the heads that have arrived; the
    // head that arrives last writes the sum to red_out [B, Smax+1].
    float *red_out;
    unsigned long long *red_acc;
    int red_shift;
    const int32_t *nseg, *bnd;
    const int32_t *hdr;     // as in EnAttnArgs
    float *out;
    int B, Hq, Nq, Smax, n_splits;
    int sub;                // as in EnAttnArgs: n_splits * sub partial results per row, the sub of a split side by side
    int q_first;            // as in EnAttnArgs
};

struct EnAppendArgs {
    const void *k_rows, *v_rows;   // [n, Hkv, D]
    void *k_pool, *v_pool;         // [G, Hkv, C, D]
    int n, Hkv, C, group, first;   // rows go to tokens first .. first+n-1 of the group
    int row_chunks;                // 16-byte chunks per (token, head) row
};
struct EnAppendQ8Args {
    const void *k_rows, *v_rows;   // bf16 [n, Hkv, D]
    int8_t *k_pool, *v_pool;       // [G, Hkv, C, D]
    float *k_scale, *v_scale;      // [G, Hkv, C]
    int n, Hkv, C, group, first;
};


constexpr int EN_RED_DIRECT_MAX_BUCKETS = 256;   // EnAttnArgs::red_direct: buckets whose sums a workgroup keeps in LDS
constexpr int EN_MAX_SPLITS = 64;       // KV splits of a plan: the mass kernels hold one split per lane
constexpr int EN_MAX_OBJECTS = 255;    // per segment_cluster_assign call (spans travel in the kernel arguments)
struct EnClusterArgs {
    EnMassArgs m;                  // the scratch of the attention call (m.out unused)
    float *score;                  // [B, n_obj, Smax+1]
    int32_t *assign;               // [B, n_obj] or null
    int n_obj, per_key, accumulate;
    float scale, threshold;
    int32_t spans[EN_MAX_OBJECTS + 1];   // object o = new tokens [spans[o], spans[o+1])
};

// One launch loads up to EN_TIER_LOAD_MAX blocks from the pinned host store into device slots.
constexpr int EN_TIER_LOAD_MAX = 128;
struct EnTierLoadArgs {
    const char *k_store, *v_store;   // device-visible addresses of the store, blocks [G, Hkv, C, D]
    char *k_slots, *v_slots;         // device, blocks [slots, Hkv, C, D]
    unsigned long long block_bytes;  // Hkv * C * D * elem
    int head_bytes;                  // C * D * elem
    int row_bytes;                   // D * elem
    int Hkv, n;
    int32_t desc[EN_TIER_LOAD_MAX * 3];   // per block: group, slot, tokens
};

struct EnCtxAppendArgs {
    const void *k_rows, *v_rows;   // [B, n, Hkv, D], keys unrotated
    void *kc, *vt;                 // the context buffers
    const float *cos_tab, *sin_tab;
    const int32_t *hdr;            // per agent {S, L_c, ...}
    int B, Hkv, n, T, q_first;
};

// Workspace layout helper (bytes, every part 256-byte aligned).
struct EnWsLayout {
    size_t ml_off, seg_off, red_off, redacc_off, mlfin_off, opart_off, total;
};
EnWsLayout en_ws_layout(const en_pool *pool, const en_plan *plan);
EnWsLayout en_ws_layout_for(const en_pool *pool, const en_plan *plan, int n_rows, int n_splits);
int en_attn_sub(const en_pool *pool, const en_plan *plan, int n_rows, int n_splits);

// Kernel launchers (the .hip files). Return hipError_t as int.
int en_launch_gather(const en_pool *pool, EnGatherLaunch &g, int max_ctx_len, void *stream);
int en_launch_attention(const en_pool *pool, const EnAttnArgs &a, void *stream);
int en_launch_attention_prefill(const en_pool *pool, const EnAttnArgs &a, void *stream);   // called by the former
int en_launch_combine(const en_pool *pool, const EnAttnArgs &a, const EnMassArgs &m, void *stream);
int en_launch_append(const en_pool *pool, const EnAppendArgs &a, void *stream);
int en_launch_append_q8(const en_pool *pool, const EnAppendQ8Args &a, void *stream);
int en_launch_cluster(const en_pool *pool, const EnClusterArgs &a, void *stream);
int en_launch_ctx_append(const en_pool *pool, const EnCtxAppendArgs &a, void *stream);
int en_launch_mass(const en_pool *pool, const EnMassArgs &a, int reduce, void *stream);
int en_launch_tier_load(const EnTierLoadArgs &a, int max_tokens, void *stream);

// The static device scratch of segmented_decode_step_static (en_static_scratch.hip,
// EN_STATIC_SCRATCH_BYTES of the public header): the device address of the current device's copy
// (returns 0 or a hipError_t).
int en_static_scratch(void **ptr_out, size_t *bytes_out);

int en_launch_ceiling_mfma(float *sink_dev, int n_workgroups, int iters, int constant, void *stream);
int en_launch_ceiling_read(const void *src_dev, size_t bytes, void *sink_dev, int n_workgroups, void *stream);

void en_set_error(const char *fmt, ...);

// Every extern "C" entry point that returns a status runs its body through this: no C++
// exception (std::bad_alloc from a container sized by caller input, above all) crosses the C ABI.
int en_fail_exception(const char *who, bool out_of_memory);
#define EN_GUARDED(who, call)                      \
    try {                                          \
        return (call);                             \
    } catch (const std::bad_alloc &) {             \
        return en_fail_exception(who, true);       \
    } catch (...) {                                \
        return en_fail_exception(who, false);      \
    }

// Retrieval knapsack of Eq. (1) over `G` candidates with lengths `len` (tokens); ids ascending.
// Returns an en_status: INVALID_ARG for a score or threshold that is not finite, CAPACITY when the
// table of the dynamic programme would exceed EN_KNAPSACK_MAX_BYTES.
constexpr size_t EN_KNAPSACK_MAX_BYTES = size_t(1) << 30;
int en_knapsack(const float *p_host, const int32_t *len, int G, float threshold, int64_t budget_tokens,
                std::vector<int32_t> &chosen);
