// Host side of libefficientnav.so: handles, the planner (validation, prefix
// sums, split choice), the retrieval knapsack of Section 3.4 Eq. (1), and the
// C ABI entry points that marshal arguments into kernel launches.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <memory>
#include <new>
#include <string>

#include "en_internal.h"

// ---------------------------------------------------------------------------
// error text
// ---------------------------------------------------------------------------
static thread_local char g_err[512] = "";

void en_set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

extern "C" const char *en_last_error(void) { return g_err; }

static int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int en_fail_exception(const char *who, bool out_of_memory)
{
    return out_of_memory ? fail(EN_ERR_CAPACITY, "%s: out of host memory", who)
                         : fail(EN_ERR_INVALID_ARG, "%s: unexpected C++ exception", who);
}

static int hip_fail(hipError_t e, const char *what)
{
    return fail(EN_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

static inline int round_up(int x, int m) { return (x + m - 1) / m * m; }
static inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }
// bytes of an element of the contexts, the queries and the outputs (an EN_I8 pool computes in bf16)
static inline size_t elem_size(int dtype) { return dtype == EN_F32 ? 4 : 2; }
// bytes of an element of the pool arrays
static inline size_t pool_elem_size(int dtype) { return dtype == EN_F32 ? 4 : dtype == EN_BF16 ? 2 : 1; }
// the bf16 kernels serve EN_BF16 and EN_I8 pools
static inline bool computes_bf16(int dtype) { return dtype != EN_F32; }

// log2(e) / sqrt(D): scores are taken in the log2 domain
static inline float softmax_scale_log2e(const en_pool *pool)
{
    return float(1.4426950408889634 / std::sqrt(double(pool->d.head_dim)));
}

// ---------------------------------------------------------------------------
// pool
// ---------------------------------------------------------------------------
static int kv_pool_create_impl(const en_pool_desc *desc, void *k_dev, void *v_dev,
                              const int32_t *len_host, en_pool **out)
{
    if (!desc || !k_dev || !v_dev || !len_host || !out)
        return fail(EN_ERR_INVALID_ARG, "kv_pool_create: null argument");
    *out = nullptr;
    if (desc->n_groups <= 0 || desc->capacity <= 0 || desc->n_kv_heads <= 0 ||
        desc->n_q_heads <= 0 || desc->max_ctx <= 0 || desc->reserved != 0 ||
        !(desc->rope_base > 0.0))
        return fail(EN_ERR_INVALID_ARG, "kv_pool_create: non-positive size, reserved != 0 or bad rope_base");
    if (desc->dtype != EN_F32 && desc->dtype != EN_BF16 && desc->dtype != EN_I8)
        return fail(EN_ERR_UNSUPPORTED, "kv_pool_create: dtype %d", desc->dtype);
    if (desc->head_dim != 64 && desc->head_dim != 128)
        return fail(EN_ERR_UNSUPPORTED, "kv_pool_create: head_dim %d (64 or 128)", desc->head_dim);
    if (desc->n_q_heads % desc->n_kv_heads != 0)
        return fail(EN_ERR_UNSUPPORTED, "kv_pool_create: n_q_heads %% n_kv_heads != 0");
    for (int g = 0; g < desc->n_groups; ++g)
        if (len_host[g] < 0 || len_host[g] > desc->capacity)
            return fail(EN_ERR_OUT_OF_RANGE, "kv_pool_create: len[%d] = %d outside [0, %d]", g,
                        len_host[g], desc->capacity);
    en_pool *p = new (std::nothrow) en_pool;
    if (!p)
        return fail(EN_ERR_CAPACITY, "kv_pool_create: out of host memory");
    p->d = *desc;
    p->k_dev = k_dev;
    p->v_dev = v_dev;
    try {
        p->len.assign(len_host, len_host + desc->n_groups);
    } catch (const std::bad_alloc &) {
        delete p;
        return fail(EN_ERR_CAPACITY, "kv_pool_create: out of host memory for %d group lengths", desc->n_groups);
    }
    p->r = desc->n_q_heads / desc->n_kv_heads;
    *out = p;
    return EN_OK;
}
extern "C" int kv_pool_create(const en_pool_desc *desc, void *k_dev, void *v_dev,
                              const int32_t *len_host, en_pool **out)
{
    EN_GUARDED("kv_pool_create", kv_pool_create_impl(desc, k_dev, v_dev, len_host, out));
}

static int kv_pool_set_len_impl(en_pool *pool, int32_t group, int32_t len)
{
    if (!pool)
        return fail(EN_ERR_INVALID_ARG, "kv_pool_set_len: null pool");
    if (group < 0 || group >= pool->d.n_groups || len < 0 || len > pool->d.capacity)
        return fail(EN_ERR_OUT_OF_RANGE, "kv_pool_set_len: group %d len %d", group, len);
    pool->len[group] = len;
    return EN_OK;
}
extern "C" int kv_pool_set_len(en_pool *pool, int32_t group, int32_t len)
{
    EN_GUARDED("kv_pool_set_len", kv_pool_set_len_impl(pool, group, len));
}

static int kv_pool_set_scales_impl(en_pool *pool, float *k_scale_dev, float *v_scale_dev)
{
    if (!pool || !k_scale_dev || !v_scale_dev)
        return fail(EN_ERR_INVALID_ARG, "kv_pool_set_scales: null argument");
    if (pool->d.dtype != EN_I8)
        return fail(EN_ERR_INVALID_ARG, "kv_pool_set_scales: the pool does not hold 8-bit codes");
    pool->k_scale = k_scale_dev;
    pool->v_scale = v_scale_dev;
    return EN_OK;
}
extern "C" int kv_pool_set_scales(en_pool *pool, float *k_scale_dev, float *v_scale_dev)
{
    EN_GUARDED("kv_pool_set_scales", kv_pool_set_scales_impl(pool, k_scale_dev, v_scale_dev));
}

static int kv_pool_append_impl(en_pool *pool, int32_t group, const void *k_rows_dev, const void *v_rows_dev,
                              int32_t n_tokens, void *stream)
{
    if (!pool || n_tokens < 0 || (n_tokens > 0 && (!k_rows_dev || !v_rows_dev)))
        return fail(EN_ERR_INVALID_ARG, "kv_pool_append: null argument or negative count");
    if (group < 0 || group >= pool->d.n_groups)
        return fail(EN_ERR_OUT_OF_RANGE, "kv_pool_append: group %d outside [0, %d)", group, pool->d.n_groups);
    const int len = pool->len[group];
    if (long(len) + n_tokens > pool->d.capacity)
        return fail(EN_ERR_CAPACITY, "kv_pool_append: group %d holds %d tokens, %d more exceed capacity %d",
                    group, len, n_tokens, pool->d.capacity);
    if (n_tokens == 0)
        return EN_OK;
    if (pool->d.dtype == EN_I8) {
        if (!pool->k_scale || !pool->v_scale)
            return fail(EN_ERR_INVALID_ARG, "kv_pool_append: an 8-bit pool needs kv_pool_set_scales first");
        EnAppendQ8Args q;
        q.k_rows = k_rows_dev;
        q.v_rows = v_rows_dev;
        q.k_pool = static_cast<int8_t *>(pool->k_dev);
        q.v_pool = static_cast<int8_t *>(pool->v_dev);
        q.k_scale = pool->k_scale;
        q.v_scale = pool->v_scale;
        q.n = n_tokens;
        q.Hkv = pool->d.n_kv_heads;
        q.C = pool->d.capacity;
        q.group = group;
        q.first = len;
        const int eq = en_launch_append_q8(pool, q, stream);
        if (eq != 0)
            return hip_fail((hipError_t)eq, "kv_pool_append launch");
        pool->len[group] = len + n_tokens;
        return EN_OK;
    }
    EnAppendArgs a;
    a.k_rows = k_rows_dev;
    a.v_rows = v_rows_dev;
    a.k_pool = pool->k_dev;
    a.v_pool = pool->v_dev;
    a.n = n_tokens;
    a.Hkv = pool->d.n_kv_heads;
    a.C = pool->d.capacity;
    a.group = group;
    a.first = len;
    a.row_chunks = pool->d.head_dim * int(pool_elem_size(pool->d.dtype)) / 16;
    const int e = en_launch_append(pool, a, stream);
    if (e != 0)
        return hip_fail((hipError_t)e, "kv_pool_append launch");
    pool->len[group] = len + n_tokens;
    return EN_OK;
}
extern "C" int kv_pool_append(en_pool *pool, int32_t group, const void *k_rows_dev, const void *v_rows_dev,
                              int32_t n_tokens, void *stream)
{
    EN_GUARDED("kv_pool_append", kv_pool_append_impl(pool, group, k_rows_dev, v_rows_dev, n_tokens, stream));
}

static void timing_release(en_pool *pool);

static int kv_pool_destroy_impl(en_pool *pool)
{
    if (!pool)
        return EN_OK;
    timing_release(pool);
    if (pool->d_cos)
        (void)hipFree(pool->d_cos);
    if (pool->d_sin)
        (void)hipFree(pool->d_sin);
    for (auto &c : pool->desc_cache)
        (void)hipFree(c.second);
    for (en_plan *pl : pool->plans)
        pl->pool = nullptr;               // only en_plan_destroy may still be called on these
    delete pool;
    return EN_OK;
}
extern "C" int kv_pool_destroy(en_pool *pool)
{
    EN_GUARDED("kv_pool_destroy", kv_pool_destroy_impl(pool));
}

// Rotary table: cos/sin(pos * base^(-2k/D)) evaluated in double, stored as
// float, [max_ctx, D/2]. Built once per pool on first GPU use.
static int pool_ensure_device(en_pool *p)
{
    if (p->d_cos)
        return EN_OK;
    const int half = p->d.head_dim / 2;
    const size_t n = size_t(p->d.max_ctx) * half;
    std::vector<float> c(n), s(n);
    std::vector<double> theta(half);
    for (int k = 0; k < half; ++k)
        theta[k] = std::pow(p->d.rope_base, -2.0 * double(k) / double(p->d.head_dim));
    for (int pos = 0; pos < p->d.max_ctx; ++pos)
        for (int k = 0; k < half; ++k) {
            const double a = double(pos) * theta[k];
            c[size_t(pos) * half + k] = float(std::cos(a));
            s[size_t(pos) * half + k] = float(std::sin(a));
        }
    hipError_t e;
    if ((e = hipMalloc((void **)&p->d_cos, n * sizeof(float))) != hipSuccess)
        return hip_fail(e, "hipMalloc(rotary table)");
    if ((e = hipMalloc((void **)&p->d_sin, n * sizeof(float))) != hipSuccess)
        return hip_fail(e, "hipMalloc(rotary table)");
    if ((e = hipMemcpy(p->d_cos, c.data(), n * sizeof(float), hipMemcpyHostToDevice)) != hipSuccess)
        return hip_fail(e, "hipMemcpy(rotary table)");
    if ((e = hipMemcpy(p->d_sin, s.data(), n * sizeof(float), hipMemcpyHostToDevice)) != hipSuccess)
        return hip_fail(e, "hipMemcpy(rotary table)");
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
        prop.multiProcessorCount > 0)
        p->n_cu = prop.multiProcessorCount;
    // set-up is also where this device's address of the static scratch is looked up, so that
    // segmented_decode_step_static finds it ready (it asks again by itself if this failed)
    void *sp = nullptr;
    size_t sb = 0;
    (void)en_static_scratch(&sp, &sb);
    return EN_OK;
}

// ---------------------------------------------------------------------------
// planner
// ---------------------------------------------------------------------------
static int choose_splits(const en_pool *pool, const en_plan *pl)
{
    // One workgroup covers 8 (head, 32-query block) pairs of one KV head and
    // fills a compute unit. The key range is split so that the rounds of
    // workgroups the compute units go through, times the length of one
    // workgroup (its key tiles plus a start-up and wind-down worth about six
    // tiles), is shortest; at least four key tiles per split.
    const int r = pool->r;
    if (computes_bf16(pool->d.dtype) && r * pl->Nq <= EN_ROWS_PER_WAVE) {
        // decode path: one wave per (agent, KV head, split); the two LDS stages
        // of a wave let two waves share a compute unit, and a wave takes about
        // 2 us per 64-key tile whatever the load: as many splits as give every
        // compute unit its two waves (measured on 1 and 4 agents x 8 K tokens:
        // more waves than that only add start-up and merge work), down to one
        // tile per split (one agent over 1.7 K tokens: 18.9 us per step with at
        // least four tiles per split, 15.0 with two, 12.8 with one: the waves run
        // side by side and the merge costs the same launch either way).
        // Long contexts of many agents are the exception: two
        // splits measured faster than one (0.73 against 0.78 ms on 64 agents x
        // 16 K tokens).
        const long base = long(pl->B) * pool->d.n_kv_heads;
        const int tiles = std::max(1, (pl->max_ctx_len + EN_KEY_TILE - 1) / EN_KEY_TILE);
        long want = (2L * pool->n_cu + base - 1) / base;
        if (want < 2 && tiles >= 64)
            want = 2;
        want = std::max<long>(1, std::min<long>(std::min<long>(want, tiles), EN_MAX_SPLITS));
        // The fewest splits that keep the longest split as short do with fewer units and merges:
        // 97 tiles are two for some of 64 splits and two for nearly all of 49 (one agent, 6 K
        // tokens: 14.7 -> 13.9 us per step; 137 tiles as 46 x 3 instead of 64 x 2 or 3: 17.5 ->
        // 17.1). Not when only a few splits are three tiles or longer: those then run while the
        // others have finished, and making all of them as long costs more than it saves (65 tiles
        // of two agents as 22 x 3 instead of 32 splits: 16.1 -> 16.6 us).
        const long longest = (tiles + want - 1) / want;
        const long n_longest = tiles - (longest - 1) * want;       // splits of that length
        if (longest <= 2 || 8 * n_longest >= want)
            want = (tiles + longest - 1) / longest;
        return int(want);
    }
    const int nqb = (pl->Nq + EN_ROWS_PER_WAVE - 1) / EN_ROWS_PER_WAVE;
    const int n_ptiles = (r * nqb + EN_WAVES - 1) / EN_WAVES;
    const long base = long(pl->B) * pool->d.n_kv_heads * n_ptiles;
    const int tiles = std::max(1, (pl->max_ctx_len + EN_KEY_TILE - 1) / EN_KEY_TILE);
    const int n_max = std::max(1, std::min(EN_MAX_SPLITS, tiles / 4));
    int best = 1;
    long best_cost = -1;
    for (int n = 1; n <= n_max; ++n) {
        const long rounds = (base * n + pool->n_cu - 1) / pool->n_cu;
        const long cost = rounds * ((tiles + n - 1) / n + 6);
        if (best_cost < 0 || cost < best_cost) {
            best_cost = cost;
            best = n;
        }
    }
    return best;
}

static int build_plan(const en_pool *pool, int32_t B, const int32_t *sel, const int32_t *sel_ptr,
                      int32_t n_new, en_plan **out)
{
    if (!pool || !sel_ptr || !out || (B > 0 && !sel && sel_ptr[B] > 0))
        return fail(EN_ERR_INVALID_ARG, "segment_select: null argument");
    *out = nullptr;
    if (B <= 0 || n_new <= 0)
        return fail(EN_ERR_INVALID_ARG, "segment_select: n_agents and n_new must be positive");
    if (sel_ptr[0] != 0)
        return fail(EN_ERR_INVALID_ARG, "segment_select: sel_ptr[0] != 0");
    int Smax = 0;
    for (int b = 0; b < B; ++b) {
        if (sel_ptr[b + 1] < sel_ptr[b])
            return fail(EN_ERR_INVALID_ARG, "segment_select: sel_ptr not monotone at agent %d", b);
        Smax = std::max(Smax, sel_ptr[b + 1] - sel_ptr[b]);
    }
    const int G = pool->d.n_groups;
    std::unique_ptr<en_plan> holder(new (std::nothrow) en_plan);     // released to the caller at the end
    en_plan *pl = holder.get();
    if (!pl)
        return fail(EN_ERR_CAPACITY, "segment_select: out of host memory");
    pl->pool = pool;
    pl->B = B;
    pl->Nq = n_new;
    pl->Smax = Smax;
    pl->nseg.assign(B, 0);
    pl->sel.assign(size_t(B) * std::max(Smax, 1), -1);
    pl->bnd.assign(size_t(B) * (Smax + 2), 0);
    pl->hdr.assign(size_t(B) * 4, 0);
    std::vector<int32_t> seen(G, -1);
    const int sstr = std::max(Smax, 1);
    for (int b = 0; b < B; ++b) {
        const int S = sel_ptr[b + 1] - sel_ptr[b];
        pl->nseg[b] = S;
        int64_t acc = 0;
        int32_t *bnd = &pl->bnd[size_t(b) * (Smax + 2)];
        for (int s = 0; s < S; ++s) {
            const int g = sel[sel_ptr[b] + s];
            if (g < 0 || g >= G) {
                return fail(EN_ERR_OUT_OF_RANGE, "segment_select: agent %d entry %d: group %d outside [0,%d)",
                            b, s, g, G);
            }
            if (seen[g] == b) {
                return fail(EN_ERR_DUPLICATE, "segment_select: agent %d selects group %d twice", b, g);
            }
            seen[g] = b;
            pl->sel[size_t(b) * sstr + s] = g;
            bnd[s] = int32_t(acc);
            acc += pool->len[g];
            if (acc + n_new > pool->d.max_ctx) {
                return fail(EN_ERR_CAPACITY, "segment_select: agent %d: L_c + N_q exceeds max_ctx %d", b,
                            pool->d.max_ctx);
            }
        }
        if (acc + n_new > pool->d.max_ctx) {
            return fail(EN_ERR_CAPACITY, "segment_select: agent %d: L_c + N_q = %lld exceeds max_ctx %d", b,
                        (long long)(acc + n_new), pool->d.max_ctx);
        }
        bnd[S] = int32_t(acc);
        for (int s = S + 1; s < Smax + 2; ++s)
            bnd[s] = int32_t(acc + n_new);
        pl->hdr[size_t(b) * 4 + 0] = S;
        pl->hdr[size_t(b) * 4 + 1] = int32_t(acc);
        pl->hdr[size_t(b) * 4 + 2] = int32_t(acc + n_new);
        pl->max_ctx_len = std::max<int>(pl->max_ctx_len, int(acc + n_new));
        pl->total_cached += acc;
        pl->total_pairs += int64_t(n_new) * acc + int64_t(n_new) * (n_new + 1) / 2;
    }
    pl->ctx_stride = round_up(pl->max_ctx_len, EN_KEY_TILE);
    pl->n_splits = choose_splits(pool, pl);
    pool->plans.push_back(pl);
    *out = holder.release();
    return EN_OK;
}

static int segment_select_impl(const en_pool *pool, int32_t n_agents, const int32_t *sel_host,
                              const int32_t *sel_ptr_host, int32_t n_new, en_plan **out)
{
    return build_plan(pool, n_agents, sel_host, sel_ptr_host, n_new, out);
}
extern "C" int segment_select(const en_pool *pool, int32_t n_agents, const int32_t *sel_host,
                              const int32_t *sel_ptr_host, int32_t n_new, en_plan **out)
{
    EN_GUARDED("segment_select", segment_select_impl(pool, n_agents, sel_host, sel_ptr_host, n_new, out));
}

// Eq. (1) as an exact 0/1 knapsack over token capacity: the groups with
// p > threshold whose lengths fit the budget and whose summed (p - threshold) is
// largest; among those the fewest tokens, then the lowest ids.
// (the file is compiled without NaN semantics: finiteness is read from the bits)
static inline bool finite_bits(float x)
{
    uint32_t u;
    std::memcpy(&u, &x, sizeof u);
    return (u & 0x7f800000u) != 0x7f800000u;
}

int en_knapsack(const float *p_host, const int32_t *len, int G, float threshold, int64_t budget_tokens,
                std::vector<int32_t> &chosen)
{
    chosen.clear();
    if (!finite_bits(threshold))
        return fail(EN_ERR_INVALID_ARG, "retrieval knapsack: the threshold is not finite");
    struct Item { int id; int64_t v; int w; };
    std::vector<Item> items;
    int64_t wsum = 0;
    for (int g = 0; g < G; ++g) {
        if (len[g] < 0)
            continue;                       // not a candidate (a store group never put)
        if (!finite_bits(p_host[g]))
            return fail(EN_ERR_INVALID_ARG, "retrieval knapsack: score of group %d is not finite", g);
        const double d = double(p_host[g]) - double(threshold);
        const int64_t v = (int64_t)std::nearbyint(d * 4294967296.0);   // ties to even
        if (v > 0) {
            items.push_back({g, v, len[g]});
            wsum += len[g];
        }
    }
    const int m = int(items.size());
    const int64_t W = std::min<int64_t>(budget_tokens, wsum);
    if (wsum <= budget_tokens) {
        for (auto &it : items)
            chosen.push_back(it.id);
        return EN_OK;
    }
    // best[a][w] over items a.. with capacity w: maximal value, then minimal
    // tokens (two rolling rows). take[a][w] records whether taking item a is
    // optimal at that state, ties included, so that the walk from item 0
    // prefers the lowest ids (lexicographically smallest sorted list).
    const size_t cols = size_t(W) + 1;
    {
        // one bit per (item, capacity) plus four rows of the capacity: refused beyond a stated size
        const size_t need = size_t(m) * ((cols + 63) / 64) * 8 + cols * 24;
        if (need > EN_KNAPSACK_MAX_BYTES)
            return fail(EN_ERR_CAPACITY, "retrieval knapsack: %d candidates x %lld tokens of budget need a table of "
                        "%zu bytes (limit %zu)", m, (long long)W, need, EN_KNAPSACK_MAX_BYTES);
    }
    std::vector<int64_t> vcur(cols, 0), vnext(cols, 0);
    std::vector<int32_t> tcur(cols, 0), tnext(cols, 0);
    const size_t words = (cols + 63) / 64;
    std::vector<uint64_t> take(size_t(m) * words, 0);
    for (int a = m - 1; a >= 0; --a) {
        const int64_t vi = items[a].v;
        const int wi = items[a].w;
        uint64_t *tk = &take[size_t(a) * words];
        for (int64_t w = 0; w <= W; ++w) {
            int64_t bv = vnext[w];
            int32_t bt = tnext[w];
            if (wi <= w) {
                const int64_t tv = vnext[w - wi] + vi;
                const int32_t tt = tnext[w - wi] + wi;
                if (tv > bv || (tv == bv && tt <= bt)) {
                    bv = tv;
                    bt = tt;
                    tk[w >> 6] |= uint64_t(1) << (w & 63);
                }
            }
            vcur[w] = bv;
            tcur[w] = bt;
        }
        vcur.swap(vnext);
        tcur.swap(tnext);
    }
    int64_t w = W;
    for (int a = 0; a < m; ++a) {
        if (take[size_t(a) * words + (w >> 6)] >> (w & 63) & 1) {
            chosen.push_back(items[a].id);
            w -= items[a].w;
        }
    }
    return EN_OK;
}

static int segment_select_scored_impl(const en_pool *pool, const float *p_host, float threshold,
                                     int64_t budget_tokens, int32_t n_new, int32_t *sel_out_host,
                                     int32_t *n_sel_out, en_plan **out)
{
    if (!pool || !p_host || !sel_out_host || !n_sel_out)
        return fail(EN_ERR_INVALID_ARG, "segment_select_scored: null argument");
    if (budget_tokens < 0)
        return fail(EN_ERR_INVALID_ARG, "segment_select_scored: negative budget");
    if (out)
        *out = nullptr;
    std::vector<int32_t> chosen;
    const int krc = en_knapsack(p_host, pool->len.data(), pool->d.n_groups, threshold, budget_tokens, chosen);
    if (krc != EN_OK)
        return krc;
    *n_sel_out = int32_t(chosen.size());
    std::copy(chosen.begin(), chosen.end(), sel_out_host);
    if (!out)
        return EN_OK;
    const int32_t ptr[2] = {0, int32_t(chosen.size())};
    return build_plan(pool, 1, chosen.data(), ptr, n_new, out);
}
extern "C" int segment_select_scored(const en_pool *pool, const float *p_host, float threshold,
                                     int64_t budget_tokens, int32_t n_new, int32_t *sel_out_host,
                                     int32_t *n_sel_out, en_plan **out)
{
    EN_GUARDED("segment_select_scored", segment_select_scored_impl(pool, p_host, threshold, budget_tokens, n_new, sel_out_host, n_sel_out, out));
}

static int en_plan_get_info_impl(const en_plan *plan, en_plan_info *info)
{
    if (!plan || !info)
        return fail(EN_ERR_INVALID_ARG, "en_plan_get_info: null argument");
    info->n_agents = plan->B;
    info->n_new = plan->Nq;
    info->max_segments = plan->Smax;
    info->ctx_stride = plan->ctx_stride;
    info->max_ctx_len = plan->max_ctx_len;
    info->n_splits = plan->n_splits;
    info->total_pairs = plan->total_pairs;
    info->total_cached = plan->total_cached;
    return EN_OK;
}
extern "C" int en_plan_get_info(const en_plan *plan, en_plan_info *info)
{
    EN_GUARDED("en_plan_get_info", en_plan_get_info_impl(plan, info));
}

static int en_plan_query_impl(const en_plan *plan, int32_t agent, int32_t *offsets_out_host,
                             int32_t *n_seg_out)
{
    if (!plan)
        return fail(EN_ERR_INVALID_ARG, "en_plan_query: null plan");
    if (agent < 0 || agent >= plan->B)
        return fail(EN_ERR_OUT_OF_RANGE, "en_plan_query: agent %d outside [0,%d)", agent, plan->B);
    const int S = plan->nseg[agent];
    if (n_seg_out)
        *n_seg_out = S;
    if (offsets_out_host)
        std::memcpy(offsets_out_host, &plan->bnd[size_t(agent) * (plan->Smax + 2)],
                    sizeof(int32_t) * size_t(S + 1));
    return EN_OK;
}
extern "C" int en_plan_query(const en_plan *plan, int32_t agent, int32_t *offsets_out_host,
                             int32_t *n_seg_out)
{
    EN_GUARDED("en_plan_query", en_plan_query_impl(plan, agent, offsets_out_host, n_seg_out));
}

static int en_plan_set_splits_impl(en_plan *plan, int32_t n_splits)
{
    if (!plan || n_splits < 1)
        return fail(EN_ERR_INVALID_ARG, "en_plan_set_splits: null plan or n_splits < 1");
    const int tiles = std::max(1, (plan->max_ctx_len + EN_KEY_TILE - 1) / EN_KEY_TILE);
    plan->n_splits = std::min(std::min(n_splits, tiles), EN_MAX_SPLITS);
    return EN_OK;
}
extern "C" int en_plan_set_splits(en_plan *plan, int32_t n_splits)
{
    EN_GUARDED("en_plan_set_splits", en_plan_set_splits_impl(plan, n_splits));
}

static bool decode_kernel_fits(const en_pool *pool, int n_rows);
static int en_plan_values_from_pool_impl(en_plan *plan, int32_t on)
{
    if (!plan || (on != 0 && on != 1))
        return fail(EN_ERR_INVALID_ARG, "en_plan_values_from_pool: null plan or a flag that is neither 0 nor 1");
    const en_pool *pool = plan->pool;
    if (on) {
        if (!pool)
            return fail(EN_ERR_INVALID_ARG, "en_plan_values_from_pool: the plan's pool has been destroyed");
        if (pool->d.dtype != EN_BF16)
            return fail(EN_ERR_UNSUPPORTED, "en_plan_values_from_pool: bf16 pools only (rows that the attention "
                        "kernel fetches as they are)");
        if (decode_kernel_fits(pool, plan->Nq))
            return fail(EN_ERR_UNSUPPORTED, "en_plan_values_from_pool: a step of so few query rows (%d per KV head) "
                        "runs in the decode kernel, which reads gathered values", pool->r * plan->Nq);
        if (reinterpret_cast<uintptr_t>(pool->v_dev) & uintptr_t(2 * pool->d.head_dim - 1))
            return fail(EN_ERR_INVALID_ARG, "en_plan_values_from_pool: the pool's values must be aligned to a row "
                        "(%d bytes)", 2 * pool->d.head_dim);
    }
    plan->values_from_pool = on != 0;
    return EN_OK;
}
extern "C" int en_plan_values_from_pool(en_plan *plan, int32_t on)
{
    EN_GUARDED("en_plan_values_from_pool", en_plan_values_from_pool_impl(plan, on));
}

static int en_plan_destroy_impl(en_plan *plan)
{
    if (!plan)
        return EN_OK;
    // The descriptor block goes back to the pool for the next plan: no device
    // synchronisation here. Work still queued on a stream keeps reading it
    // safely as long as later plans of this pool are used on that same stream.
    if (plan->pool) {
        auto &live = plan->pool->plans;
        live.erase(std::remove(live.begin(), live.end(), plan), live.end());
        if (plan->d_desc)
            plan->pool->desc_cache.emplace_back(plan->d_desc_bytes, plan->d_desc);
    } else if (plan->d_desc) {
        (void)hipFree(plan->d_desc);      // the pool went first: nothing to give the block back to
    }
    delete plan;
    return EN_OK;
}
extern "C" int en_plan_destroy(en_plan *plan)
{
    EN_GUARDED("en_plan_destroy", en_plan_destroy_impl(plan));
}

// Device block of a plan (taken from the pool's cache of released blocks when
// one fits) and its host image. With inline_ok the upload is left to the
// gather kernel, which receives the image in its arguments, provided it is
// small enough; *inlined says which way it went.
static int plan_ensure_device(en_plan *pl, hipStream_t stream, bool inline_ok = false,
                              bool *inlined = nullptr)
{
    if (inlined)
        *inlined = false;
    if (pl->uploaded)
        return EN_OK;
    const size_t n = pl->nseg.size() + pl->sel.size() + pl->bnd.size() + pl->hdr.size();
    pl->acc_off = (n + 1) & ~size_t(1);                                   // 8-byte aligned
    const size_t n_all = pl->acc_off + 2 * size_t(pl->B) * (pl->Smax + 1);    // tables, then the accumulators
    const size_t bytes = n_all * sizeof(int32_t);
    pl->h_desc.clear();
    pl->h_desc.reserve(n_all);
    pl->h_desc.insert(pl->h_desc.end(), pl->nseg.begin(), pl->nseg.end());
    pl->h_desc.insert(pl->h_desc.end(), pl->sel.begin(), pl->sel.end());
    pl->h_desc.insert(pl->h_desc.end(), pl->bnd.begin(), pl->bnd.end());
    pl->h_desc.insert(pl->h_desc.end(), pl->hdr.begin(), pl->hdr.end());
    hipError_t e;
    auto &cache = pl->pool->desc_cache;
    for (size_t i = 0; i < cache.size(); ++i)
        if (cache[i].first >= bytes) {
            pl->d_desc = cache[i].second;
            pl->d_desc_bytes = cache[i].first;
            cache.erase(cache.begin() + i);
            break;
        }
    if (!pl->d_desc) {
        const size_t cap = std::max<size_t>(align256(bytes), 4096);
        if ((e = hipMalloc((void **)&pl->d_desc, cap)) != hipSuccess)
            return hip_fail(e, "hipMalloc(plan descriptors)");
        pl->d_desc_bytes = cap;
    }
    if (inline_ok && n <= size_t(EN_INLINE_DESC_MAX)) {
        *inlined = true;              // (the launch also sets the accumulators to zero)
    } else {
        pl->h_desc.resize(n_all, 0);
        // Stream-ordered copy; the staging vector lives as long as the plan.
        if ((e = hipMemcpyAsync(pl->d_desc, pl->h_desc.data(), bytes, hipMemcpyHostToDevice, stream)) !=
            hipSuccess)
            return hip_fail(e, "hipMemcpyAsync(plan descriptors)");
    }
    pl->uploaded = true;
    return EN_OK;
}

static inline const int32_t *d_nseg(const en_plan *pl) { return pl->d_desc; }
static inline const int32_t *d_sel(const en_plan *pl) { return d_nseg(pl) + pl->nseg.size(); }
static inline const int32_t *d_bnd(const en_plan *pl) { return d_sel(pl) + pl->sel.size(); }
static inline const int32_t *d_hdr(const en_plan *pl) { return d_bnd(pl) + pl->bnd.size(); }

// ---------------------------------------------------------------------------
// sizes
// ---------------------------------------------------------------------------
extern "C" size_t en_context_bytes(const en_pool *pool, const en_plan *plan)
{
    if (!pool || !plan)
        return 0;
    return size_t(plan->B) * pool->d.n_kv_heads * plan->ctx_stride * pool->d.head_dim *
           elem_size(pool->d.dtype);
}

// All r * n_rows query rows of a KV head fit one wave: the decode attention kernel takes the step.
static bool decode_kernel_fits(const en_pool *pool, int n_rows)
{
    return computes_bf16(pool->d.dtype) && pool->r * n_rows <= EN_ROWS_PER_WAVE;
}

// Waves per (agent, KV head, split) in the decode attention kernel. One wave alone on its SIMD
// takes about 2 us per 64-key tile whatever the load, and the kernel's LDS stages leave room for
// two workgroups per compute unit: when a step has no more units than that, two waves share each
// unit's tiles, each takes every other 32-key block and leaves partial results of its own (the
// scratch then holds n_splits * 2 of them per row; the units' key ranges stay whole tiles).
// Measured per decoded token with 8 KV heads, two waves against one: 10.9 / 12.4 us (1 agent,
// 25 splits), 11.3 / 12.5 (2 agents, 17 splits), 12.6 / 13.9 (2 agents, 32 splits), 13.1 / 14.0
// (4 agents, 16 splits), 12.9 / 13.0 (1 agent, 4K tokens, 64 splits), 17.5 / 18.0 (1 agent, 8.7K
// tokens, 64 splits); the attention launch itself 9.6 / 10.0 us in the last but one case. (The
// merge of twice as many partial results must not eat the gain: see its lane groups.)
int en_attn_sub(const en_pool *pool, const en_plan *pl, int n_rows, int n_splits)
{
    if (!decode_kernel_fits(pool, n_rows))
        return 1;
    return long(pl->B) * pool->d.n_kv_heads * n_splits <= 2L * pool->n_cu ? 2 : 1;
}

// Scratch layout for n_rows query rows per agent and n_splits KV splits.
EnWsLayout en_ws_layout_for(const en_pool *pool, const en_plan *pl, int n_rows, int n_splits_plan)
{
    const int n_splits = n_splits_plan * en_attn_sub(pool, pl, n_rows, n_splits_plan);     // partial results per row
    EnWsLayout L;
    const size_t rows = size_t(pl->B) * pool->d.n_q_heads * n_rows;
    L.ml_off = 0;
    L.seg_off = align256(L.ml_off + size_t(n_splits) * rows * 2 * sizeof(float));
    L.red_off = align256(L.seg_off + size_t(n_splits) * rows * (pl->Smax + 1) * 2 * sizeof(float));
    L.redacc_off = align256(L.red_off + size_t(pl->B) * (pl->Smax + 1) * pool->d.n_q_heads * sizeof(float));
    L.mlfin_off = align256(L.redacc_off + size_t(pl->B) * (pl->Smax + 1) * sizeof(unsigned long long));
    L.opart_off = align256(L.mlfin_off + (n_splits > 1 ? rows * 2 * sizeof(float) : 0));
    L.total = L.opart_off;
    if (n_splits > 1)
        L.total = align256(L.opart_off + size_t(n_splits) * rows * pool->d.head_dim * elem_size(pool->d.dtype));
    return L;
}

EnWsLayout en_ws_layout(const en_pool *pool, const en_plan *pl)
{
    return en_ws_layout_for(pool, pl, pl->Nq, pl->n_splits);
}

extern "C" size_t en_workspace_bytes(const en_pool *pool, const en_plan *plan)
{
    if (!pool || !plan)
        return 0;
    return en_ws_layout(pool, plan).total;
}

// ---------------------------------------------------------------------------
// kernel timing with HIP events (measurement aid); the events live in the pool
// ---------------------------------------------------------------------------
static void timing_release(en_pool *pool)
{
    for (auto e : pool->ev_start)
        (void)hipEventDestroy(e);
    for (auto e : pool->ev_stop)
        (void)hipEventDestroy(e);
    pool->ev_start.clear();
    pool->ev_stop.clear();
    pool->ev_used = 0;
}

static int en_timing_enable_impl(en_pool *pool, int32_t max_records)
{
    if (!pool || max_records < 0)
        return fail(EN_ERR_INVALID_ARG, "en_timing_enable: null pool or negative count");
    timing_release(pool);
    try {
        pool->ev_start.reserve(size_t(max_records));
        pool->ev_stop.reserve(size_t(max_records));
    } catch (const std::bad_alloc &) {
        return fail(EN_ERR_CAPACITY, "en_timing_enable: out of host memory for %d records", max_records);
    }
    for (int i = 0; i < max_records; ++i) {
        hipEvent_t a, b;
        hipError_t e;
        if ((e = hipEventCreate(&a)) != hipSuccess)
            return hip_fail(e, "hipEventCreate");
        if ((e = hipEventCreate(&b)) != hipSuccess) {
            (void)hipEventDestroy(a);
            return hip_fail(e, "hipEventCreate");
        }
        pool->ev_start.push_back(a);
        pool->ev_stop.push_back(b);
    }
    return EN_OK;
}
extern "C" int en_timing_enable(en_pool *pool, int32_t max_records)
{
    EN_GUARDED("en_timing_enable", en_timing_enable_impl(pool, max_records));
}

static int en_timing_collect_impl(en_pool *pool, float *ms_out_host, int32_t cap, int32_t *n_out)
{
    if (!pool || !ms_out_host || !n_out || cap < 0)
        return fail(EN_ERR_INVALID_ARG, "en_timing_collect: null argument");
    const int n = std::min<int>(pool->ev_used, cap);
    for (int i = 0; i < n; ++i) {
        hipError_t e;
        if ((e = hipEventSynchronize(pool->ev_stop[i])) != hipSuccess)
            return hip_fail(e, "hipEventSynchronize");
        if ((e = hipEventElapsedTime(&ms_out_host[i], pool->ev_start[i], pool->ev_stop[i])) != hipSuccess)
            return hip_fail(e, "hipEventElapsedTime");
    }
    *n_out = n;
    pool->ev_used = 0;
    return EN_OK;
}
extern "C" int en_timing_collect(en_pool *pool, float *ms_out_host, int32_t cap, int32_t *n_out)
{
    EN_GUARDED("en_timing_collect", en_timing_collect_impl(pool, ms_out_host, cap, n_out));
}

// ---------------------------------------------------------------------------
// measured ceilings (measurement aid): a loop of matrix instructions only, a read-only stream
// ---------------------------------------------------------------------------
static int en_ceiling_mfma_bf16_impl(void *sink_dev, size_t sink_bytes, int32_t n_workgroups, int32_t iters,
                                     int32_t constant_operands, double *flops_out, void *stream)
{
    if (!sink_dev || !flops_out || n_workgroups <= 0 || iters <= 0 || (constant_operands != 0 && constant_operands != 1))
        return fail(EN_ERR_INVALID_ARG, "en_ceiling_mfma_bf16: null argument, non-positive size or bad flag");
    if (sink_bytes < size_t(n_workgroups) * 512 * sizeof(float))
        return fail(EN_ERR_CAPACITY, "en_ceiling_mfma_bf16: sink of %zu bytes, %zu needed", sink_bytes,
                    size_t(n_workgroups) * 512 * sizeof(float));
    const int e = en_launch_ceiling_mfma(static_cast<float *>(sink_dev), n_workgroups, iters, constant_operands, stream);
    if (e != 0)
        return hip_fail((hipError_t)e, "en_ceiling_mfma_bf16 launch");
    // 8 waves per workgroup, 8 instructions per round, 2 * 32 * 32 * 16 operations each
    *flops_out = double(n_workgroups) * 8.0 * double(iters) * 8.0 * 32768.0;
    return EN_OK;
}
extern "C" int en_ceiling_mfma_bf16(void *sink_dev, size_t sink_bytes, int32_t n_workgroups, int32_t iters,
                                    int32_t constant_operands, double *flops_out, void *stream)
{
    EN_GUARDED("en_ceiling_mfma_bf16",
               en_ceiling_mfma_bf16_impl(sink_dev, sink_bytes, n_workgroups, iters, constant_operands, flops_out, stream));
}

static int en_ceiling_read_stream_impl(const void *src_dev, size_t bytes, void *sink_dev, size_t sink_bytes,
                                       int32_t n_workgroups, void *stream)
{
    if (!src_dev || !sink_dev || n_workgroups <= 0 || bytes < 16 || (bytes & 15) ||
        (reinterpret_cast<uintptr_t>(src_dev) & 15))
        return fail(EN_ERR_INVALID_ARG, "en_ceiling_read_stream: null argument, or size / address not a multiple of 16");
    if (sink_bytes < 256 * sizeof(uint32_t))
        return fail(EN_ERR_CAPACITY, "en_ceiling_read_stream: the sink needs 1024 bytes");
    const int e = en_launch_ceiling_read(src_dev, bytes, sink_dev, n_workgroups, stream);
    if (e != 0)
        return hip_fail((hipError_t)e, "en_ceiling_read_stream launch");
    return EN_OK;
}
extern "C" int en_ceiling_read_stream(const void *src_dev, size_t bytes, void *sink_dev, size_t sink_bytes,
                                      int32_t n_workgroups, void *stream)
{
    EN_GUARDED("en_ceiling_read_stream", en_ceiling_read_stream_impl(src_dev, bytes, sink_dev, sink_bytes, n_workgroups, stream));
}

// ---------------------------------------------------------------------------
// GPU entry points
// ---------------------------------------------------------------------------
static int gather_common(en_pool *pool, en_plan *plan, const void *k_new_dev, const void *v_new_dev,
                         const void *q_dev, void *kc_dev, void *vt_dev, void *q_prep_dev, void *stream)
{
    if (!pool || !plan || !k_new_dev || !v_new_dev || !kc_dev || !vt_dev)
        return fail(EN_ERR_INVALID_ARG, "gather_rope: null argument");
    if (plan->pool != pool)
        return fail(EN_ERR_INVALID_ARG, "gather_rope: plan belongs to another pool");
    if (pool->d.dtype == EN_I8 && (!pool->k_scale || !pool->v_scale))
        return fail(EN_ERR_INVALID_ARG, "gather_rope: an 8-bit pool needs kv_pool_set_scales first");
    int rc;
    bool inlined = false;
    if ((rc = pool_ensure_device(pool)) != EN_OK ||
        (rc = plan_ensure_device(plan, (hipStream_t)stream, true, &inlined)) != EN_OK)
        return rc;
    EnGatherLaunch g;
    EnGatherArgs &a = g.a;
    a.k_pool = pool->k_dev;
    a.v_pool = pool->v_dev;
    a.k_new = k_new_dev;
    a.v_new = v_new_dev;
    a.kc = kc_dev;
    a.vt = vt_dev;
    a.cos_tab = pool->d_cos;
    a.sin_tab = pool->d_sin;
    a.k_scale = pool->k_scale;
    a.v_scale = pool->v_scale;
    a.nseg = d_nseg(plan);
    a.sel = d_sel(plan);
    a.bnd = d_bnd(plan);
    a.B = plan->B;
    a.Hkv = pool->d.n_kv_heads;
    a.C = pool->d.capacity;
    a.Nq = plan->Nq;
    a.Smax = plan->Smax;
    a.T = plan->ctx_stride;
    a.q = q_dev;
    a.q_prep = q_prep_dev;
    a.Hq = pool->d.n_q_heads;
    {
        // at most about 64 query rows (four rounds of loads) per workgroup, at most 16 units
        const long rows = long(plan->Nq) * pool->d.n_q_heads;
        const long tiles = std::max(1, (plan->max_ctx_len + EN_KEY_TILE - 1) / EN_KEY_TILE);
        a.n_q_units = int(std::min<long>(16, std::max<long>(1, (rows + 64 * tiles - 1) / (64 * tiles))));
    }
    a.scale_log2e = softmax_scale_log2e(pool);
    a.v_rows = plan->values_from_pool ? 1 : 0;
    if (a.v_rows && (reinterpret_cast<uintptr_t>(v_new_dev) & uintptr_t(2 * pool->d.head_dim - 1)))
        return fail(EN_ERR_INVALID_ARG, "gather_rope: with the values taken from where they are "
                    "(en_plan_values_from_pool) the new tokens' values must be aligned to a row (%d bytes)",
                    2 * pool->d.head_dim);
    g.n_inline = 0;
    g.off_nseg = 0;
    g.off_sel = g.off_nseg + int(plan->nseg.size());
    g.off_bnd = g.off_sel + int(plan->sel.size());
    g.desc_out = plan->d_desc;
    g.n_zero = 0;
    if (inlined) {
        g.n_inline = int(plan->h_desc.size());
        g.n_zero = int(plan->acc_off + 2 * size_t(plan->B) * (plan->Smax + 1)) - g.n_inline;
        std::memcpy(g.desc, plan->h_desc.data(), plan->h_desc.size() * sizeof(int32_t));
    }
    const int e = en_launch_gather(pool, g, plan->max_ctx_len, stream);
    if (e != 0) {
        if (inlined)
            plan->uploaded = false;       // the block was to be filled by this launch
        return hip_fail((hipError_t)e, "gather_rope launch");
    }
    plan->gathered_values_from_pool = a.v_rows;
    return EN_OK;
}
extern "C" int gather_rope(en_pool *pool, en_plan *plan, const void *k_new_dev, const void *v_new_dev,
                           void *kc_dev, void *vt_dev, void *stream)
{
    EN_GUARDED("gather_rope", gather_common(pool, plan, k_new_dev, v_new_dev, nullptr, kc_dev, vt_dev, nullptr, stream));
}

static int gather_rope_queries_impl(en_pool *pool, en_plan *plan, const void *k_new_dev, const void *v_new_dev,
                                    const void *q_dev, void *kc_dev, void *vt_dev, void *q_prep_dev, void *stream)
{
    if (!q_dev || !q_prep_dev)
        return fail(EN_ERR_INVALID_ARG, "gather_rope_queries: null argument");
    if (pool && !computes_bf16(pool->d.dtype))
        return fail(EN_ERR_UNSUPPORTED, "gather_rope_queries: prepared queries are bf16; a float32 pool keeps its "
                    "queries as they are (gather_rope, segmented_prefill_attention)");
    return gather_common(pool, plan, k_new_dev, v_new_dev, q_dev, kc_dev, vt_dev, q_prep_dev, stream);
}
extern "C" int gather_rope_queries(en_pool *pool, en_plan *plan, const void *k_new_dev, const void *v_new_dev,
                                   const void *q_dev, void *kc_dev, void *vt_dev, void *q_prep_dev, void *stream)
{
    EN_GUARDED("gather_rope_queries",
               gather_rope_queries_impl(pool, plan, k_new_dev, v_new_dev, q_dev, kc_dev, vt_dev, q_prep_dev, stream));
}

// For the rows q_first .. q_first + n_rows - 1 of the plan's new tokens, attended with n_splits KV splits.
static EnMassArgs mass_args(const en_pool *pool, const en_plan *plan, char *ws, const EnWsLayout &L, int n_rows,
                            int n_splits, int q_first)
{
    EnMassArgs a;
    a.ws_ml = reinterpret_cast<const float *>(ws + L.ml_off);
    a.ws_seg = reinterpret_cast<const float *>(ws + L.seg_off);
    a.ws_mlfin = reinterpret_cast<const float *>(ws + L.mlfin_off);
    a.ws_red = reinterpret_cast<float *>(ws + L.red_off);
    a.red_out = nullptr;
    a.red_acc = reinterpret_cast<unsigned long long *>(ws + L.redacc_off);
    {
        // fixed point of the reduced masses: a sum is at most Hq * n_rows, and sum << (shift + 10) must fit 63 bits
        int bits = 0;
        while ((uint64_t(1) << bits) < uint64_t(pool->d.n_q_heads) * uint64_t(n_rows))
            ++bits;
        a.red_shift = std::max(0, std::min(30, 52 - bits));
    }
    a.nseg = d_nseg(plan);
    a.bnd = d_bnd(plan);
    a.hdr = d_hdr(plan);
    a.out = nullptr;
    a.B = plan->B;
    a.Hq = pool->d.n_q_heads;
    a.Nq = n_rows;
    a.Smax = plan->Smax;
    a.n_splits = n_splits;
    a.sub = en_attn_sub(pool, plan, n_rows, n_splits);
    a.q_first = q_first;
    return a;
}

// Attention of n_rows query rows per agent (new tokens q_first .. q_first+n_rows-1 of the plan)
// with n_splits KV splits; the scratch is laid out for exactly these.
static int run_attention(en_pool *pool, en_plan *plan, const void *q_dev, const void *kc_dev,
                         const void *vt_dev, void *out_dev, void *ws_dev, size_t ws_bytes, void *stream,
                         int q_first, int n_rows, int n_splits, const char *who,
                         const void *app_k_dev = nullptr, const void *app_v_dev = nullptr,
                         bool q_prepared = false, float *mass_red_out_dev = nullptr)
{
    const EnWsLayout L = en_ws_layout_for(pool, plan, n_rows, n_splits);
    // the merge kernel splits a row number into (agent, head, token) in 32-bit arithmetic
    if (size_t(plan->B) * pool->d.n_q_heads * size_t(n_rows) > 0x7fffffffu)
        return fail(EN_ERR_UNSUPPORTED, "%s: more than 2^31 - 1 (agent, head, token) rows", who);
    // (without scratch there is nowhere to leave partial results: one wave per unit then)
    const int sub = ws_dev ? en_attn_sub(pool, plan, n_rows, n_splits) : 1;
    const int n_partials = n_splits * sub;
    if (!ws_dev && n_partials > 1)
        return fail(EN_ERR_INVALID_ARG, "%s: workspace required with %d partial results per row", who, n_partials);
    if (ws_dev && ws_bytes < L.total)
        return fail(EN_ERR_CAPACITY, "%s: workspace %zu < %zu bytes", who, ws_bytes, L.total);
    if (ws_dev && (reinterpret_cast<uintptr_t>(ws_dev) & 15))
        return fail(EN_ERR_INVALID_ARG, "%s: workspace must be 16-byte aligned", who);
    int rc;
    if ((rc = pool_ensure_device(pool)) != EN_OK || (rc = plan_ensure_device(plan, (hipStream_t)stream)) != EN_OK)
        return rc;
    EnAttnArgs a;
    a.q = q_dev;
    a.kc = kc_dev;
    a.vt = vt_dev;
    a.out = out_dev;
    a.cos_tab = pool->d_cos;
    a.sin_tab = pool->d_sin;
    a.nseg = d_nseg(plan);
    a.bnd = d_bnd(plan);
    a.hdr = d_hdr(plan);
    char *ws = static_cast<char *>(ws_dev);
    a.ws_ml = ws ? reinterpret_cast<float *>(ws + L.ml_off) : nullptr;
    a.ws_seg = ws ? reinterpret_cast<float *>(ws + L.seg_off) : nullptr;
    a.ws_opart = (ws && n_partials > 1) ? static_cast<void *>(ws + L.opart_off) : nullptr;
    a.ws_mlfin = (ws && n_partials > 1) ? reinterpret_cast<float *>(ws + L.mlfin_off) : nullptr;
    a.B = plan->B;
    a.Hq = pool->d.n_q_heads;
    a.Hkv = pool->d.n_kv_heads;
    a.Nq = n_rows;
    a.Smax = plan->Smax;
    a.T = plan->ctx_stride;
    a.q_first = q_first;
    a.n_splits = n_splits;
    a.sub = sub;
    const int nqb = (n_rows + EN_ROWS_PER_WAVE - 1) / EN_ROWS_PER_WAVE;
    a.n_ptiles = (pool->r * nqb + EN_WAVES - 1) / EN_WAVES;
    a.decode = decode_kernel_fits(pool, n_rows) ? 1 : 0;
    if (a.decode)
        a.n_ptiles = 1;
    a.total_wgs = plan->B * pool->d.n_kv_heads * n_splits * a.n_ptiles;
    a.scale_log2e = softmax_scale_log2e(pool);
    a.app_k = a.decode ? app_k_dev : nullptr;
    a.app_v = a.decode ? app_v_dev : nullptr;
    a.q_prepared = q_prepared ? 1 : 0;
    a.v_rows = plan->values_from_pool ? 1 : 0;
    if (a.v_rows && (a.decode || q_first != 0 || n_rows != plan->Nq))
        return fail(EN_ERR_UNSUPPORTED, "%s: a plan whose values stay in the pool (en_plan_values_from_pool) has no "
                    "gathered values for a step of its own rows; gather them (flag 0) first", who);
    if (plan->gathered_values_from_pool >= 0 && plan->gathered_values_from_pool != a.v_rows)
        return fail(EN_ERR_INVALID_ARG, "%s: en_plan_values_from_pool was changed after the plan's last gather; "
                    "gather again", who);
    a.red_zero = (mass_red_out_dev && ws) ? reinterpret_cast<unsigned long long *>(ws + L.redacc_off) : nullptr;
    a.n_red_zero = a.red_zero ? plan->B * (plan->Smax + 1) : 0;
    // One partial result per row in the matrix-core kernel: its workgroups add the reduced masses up
    // themselves, in the plan's own accumulators (every workgroup arrives once per bucket; the
    // kernel keeps its eight waves' sums of the buckets in LDS).
    a.red_direct = nullptr;
    a.red_direct_out = nullptr;
    a.red_shift = a.red_target = 0;
    const int arrivals = pool->d.n_kv_heads * a.n_ptiles;        // workgroups per agent
    const bool red_direct = mass_red_out_dev && ws && n_partials == 1 && !a.decode && computes_bf16(pool->d.dtype) &&
                            q_first == 0 && n_rows == plan->Nq && arrivals <= 1023 && plan->Smax + 1 <= EN_RED_DIRECT_MAX_BUCKETS;
    if (red_direct) {
        a.red_direct = reinterpret_cast<unsigned long long *>(plan->d_desc + plan->acc_off);
        a.red_direct_out = mass_red_out_dev;
        a.red_shift = mass_args(pool, plan, ws, L, n_rows, n_splits, q_first).red_shift;
        a.red_target = arrivals;
        a.red_zero = nullptr;
        a.n_red_zero = 0;
    }
    const bool timed = pool->ev_used < (int)pool->ev_start.size();
    if (timed)
        (void)hipEventRecord(pool->ev_start[pool->ev_used], (hipStream_t)stream);
    int e = en_launch_attention(pool, a, stream);
    if (timed)
        (void)hipEventRecord(pool->ev_stop[pool->ev_used++], (hipStream_t)stream);
    if (e != 0)
        return hip_fail((hipError_t)e, who);
    if (n_partials > 1) {
        // the same launch also leaves the per-head partial sums of the segment masses
        EnMassArgs m = mass_args(pool, plan, ws, L, n_rows, n_splits, q_first);
        m.red_out = mass_red_out_dev;
        EnAttnArgs c = a;
        c.n_splits = n_partials;              // the merge only counts partial results
        e = en_launch_combine(pool, c, m, stream);
        if (e != 0)
            return hip_fail((hipError_t)e, "split combine launch");
    }
    if (mass_red_out_dev && !red_direct) {
        // stage 1 of the reduced masses as a launch of its own where no merge launch carried it (one
        // partial result per row, or few rows per head): en_launch_mass launches nothing otherwise
        EnMassArgs m = mass_args(pool, plan, ws, L, n_rows, n_splits, q_first);
        m.red_out = mass_red_out_dev;
        e = en_launch_mass(pool, m, 2, stream);
        if (e != 0)
            return hip_fail((hipError_t)e, "reduced masses launch");
    }
    return EN_OK;
}

static int segmented_prefill_attention_impl(en_pool *pool, en_plan *plan, const void *q_dev,
                                           const void *kc_dev, const void *vt_dev, void *out_dev,
                                           void *ws_dev, size_t ws_bytes, void *stream)
{
    if (!pool || !plan || !q_dev || !kc_dev || !vt_dev || !out_dev)
        return fail(EN_ERR_INVALID_ARG, "segmented_prefill_attention: null argument");
    if (plan->pool != pool)
        return fail(EN_ERR_INVALID_ARG, "segmented_prefill_attention: plan belongs to another pool");
    return run_attention(pool, plan, q_dev, kc_dev, vt_dev, out_dev, ws_dev, ws_bytes, stream, 0, plan->Nq,
                         plan->n_splits, "segmented_prefill_attention");
}
extern "C" int segmented_prefill_attention(en_pool *pool, en_plan *plan, const void *q_dev,
                                           const void *kc_dev, const void *vt_dev, void *out_dev,
                                           void *ws_dev, size_t ws_bytes, void *stream)
{
    EN_GUARDED("segmented_prefill_attention", segmented_prefill_attention_impl(pool, plan, q_dev, kc_dev, vt_dev, out_dev, ws_dev, ws_bytes, stream));
}

static int segmented_prefill_attention_prepared_impl(en_pool *pool, en_plan *plan, const void *q_prep_dev,
                                                     const void *kc_dev, const void *vt_dev, void *out_dev,
                                                     float *mass_red_out_dev, void *ws_dev, size_t ws_bytes,
                                                     void *stream)
{
    if (!pool || !plan || !q_prep_dev || !kc_dev || !vt_dev || !out_dev)
        return fail(EN_ERR_INVALID_ARG, "segmented_prefill_attention_prepared: null argument");
    if (plan->pool != pool)
        return fail(EN_ERR_INVALID_ARG, "segmented_prefill_attention_prepared: plan belongs to another pool");
    if (!computes_bf16(pool->d.dtype))
        return fail(EN_ERR_UNSUPPORTED, "segmented_prefill_attention_prepared: prepared queries are bf16");
    if (decode_kernel_fits(pool, plan->Nq))
        return fail(EN_ERR_UNSUPPORTED, "segmented_prefill_attention_prepared: a step of so few query rows "
                    "(%d per KV head) goes through segmented_prefill_attention or segmented_decode_step",
                    pool->r * plan->Nq);
    if (mass_red_out_dev && !ws_dev)
        return fail(EN_ERR_INVALID_ARG, "segmented_prefill_attention_prepared: masses need the workspace");
    if (mass_red_out_dev && pool->d.n_q_heads > 1023)
        return fail(EN_ERR_UNSUPPORTED, "segmented_prefill_attention_prepared: reduced masses in the attention call "
                    "count at most 1023 query heads; use segment_attention_mass");
    return run_attention(pool, plan, q_prep_dev, kc_dev, vt_dev, out_dev, ws_dev, ws_bytes, stream, 0, plan->Nq,
                         plan->n_splits, "segmented_prefill_attention_prepared", nullptr, nullptr, true,
                         mass_red_out_dev);
}
extern "C" int segmented_prefill_attention_prepared(en_pool *pool, en_plan *plan, const void *q_prep_dev,
                                                    const void *kc_dev, const void *vt_dev, void *out_dev,
                                                    float *mass_red_out_dev, void *ws_dev, size_t ws_bytes,
                                                    void *stream)
{
    EN_GUARDED("segmented_prefill_attention_prepared",
               segmented_prefill_attention_prepared_impl(pool, plan, q_prep_dev, kc_dev, vt_dev, out_dev,
                                                         mass_red_out_dev, ws_dev, ws_bytes, stream));
}

// KV splits for a step of n_rows query rows (same rule as for a whole plan).
static int cluster_assign(en_pool *pool, en_plan *plan, int q_first, int n_rows, int n_splits, void *ws_dev,
                          int32_t n_obj, const int32_t *span_ptr_host, int32_t per_key, int32_t accumulate,
                          float scale, float threshold, float *score_dev, int32_t *assign_dev, void *stream,
                          const char *who);

static int step_splits(const en_pool *pool, const en_plan *plan, int n_rows)
{
    en_plan tmp;
    tmp.pool = pool;
    tmp.B = plan->B;
    tmp.Nq = n_rows;
    tmp.max_ctx_len = plan->max_ctx_len;
    return choose_splits(pool, &tmp);
}

extern "C" size_t en_decode_workspace_bytes(const en_pool *pool, const en_plan *plan, int32_t n_rows)
{
    if (!pool || !plan || n_rows <= 0)
        return 0;
    return en_ws_layout_for(pool, plan, n_rows, step_splits(pool, plan, n_rows)).total;
}

static int segmented_decode_step_impl(en_pool *pool, en_plan *plan, int32_t q_first, int32_t n_rows,
                                     const void *q_dev, const void *k_rows_dev, const void *v_rows_dev,
                                     void *kc_dev, void *vt_dev, void *out_dev, float *mass_out_dev,
                                     void *ws_dev, size_t ws_bytes, void *stream)
{
    if (!pool || !plan || !q_dev || !k_rows_dev || !v_rows_dev || !kc_dev || !vt_dev || !out_dev)
        return fail(EN_ERR_INVALID_ARG, "segmented_decode_step: null argument");
    if (plan->pool != pool)
        return fail(EN_ERR_INVALID_ARG, "segmented_decode_step: plan belongs to another pool");
    if (q_first < 0 || n_rows <= 0 || q_first + n_rows > plan->Nq)
        return fail(EN_ERR_OUT_OF_RANGE, "segmented_decode_step: new tokens [%d, %d) outside the plan's %d",
                    q_first, q_first + n_rows, plan->Nq);
    if (mass_out_dev && !ws_dev)
        return fail(EN_ERR_INVALID_ARG, "segmented_decode_step: masses need the workspace");
    if (plan->values_from_pool)
        return fail(EN_ERR_UNSUPPORTED, "segmented_decode_step: the plan's values stay in the pool "
                    "(en_plan_values_from_pool); the decode steps read a gathered context");
    int rc;
    if ((rc = pool_ensure_device(pool)) != EN_OK || (rc = plan_ensure_device(plan, (hipStream_t)stream)) != EN_OK)
        return rc;
    // 1. the step's keys (rotated at their positions) and values join the gathered context. When
    // the step's rows fit the decode attention kernel, that kernel does it itself (the wave whose
    // key range holds a new token writes it before it loads that range): a launch of its own for
    // a few rows costs as much as a quarter of such a step.
    const bool fused = decode_kernel_fits(pool, n_rows);
    EnCtxAppendArgs c;
    c.k_rows = k_rows_dev;
    c.v_rows = v_rows_dev;
    c.kc = kc_dev;
    c.vt = vt_dev;
    c.cos_tab = pool->d_cos;
    c.sin_tab = pool->d_sin;
    c.hdr = d_hdr(plan);
    c.B = plan->B;
    c.Hkv = pool->d.n_kv_heads;
    c.n = n_rows;
    c.T = plan->ctx_stride;
    c.q_first = q_first;
    int e = fused ? 0 : en_launch_ctx_append(pool, c, stream);
    if (e != 0)
        return hip_fail((hipError_t)e, "segmented_decode_step context append");
    // 2. attention of the step's rows over everything before and including them
    const int n_splits = step_splits(pool, plan, n_rows);
    if ((rc = run_attention(pool, plan, q_dev, kc_dev, vt_dev, out_dev, ws_dev, ws_bytes, stream, q_first, n_rows,
                            n_splits, "segmented_decode_step", fused ? k_rows_dev : nullptr,
                            fused ? v_rows_dev : nullptr)) != EN_OK)
        return rc;
    // 3. per-row masses, if wanted
    if (mass_out_dev) {
        const EnWsLayout L = en_ws_layout_for(pool, plan, n_rows, n_splits);
        EnMassArgs m = mass_args(pool, plan, static_cast<char *>(ws_dev), L, n_rows, n_splits, q_first);
        m.out = mass_out_dev;
        e = en_launch_mass(pool, m, 0, stream);
        if (e != 0)
            return hip_fail((hipError_t)e, "segmented_decode_step mass");
    }
    return EN_OK;
}
extern "C" int segmented_decode_step(en_pool *pool, en_plan *plan, int32_t q_first, int32_t n_rows,
                                     const void *q_dev, const void *k_rows_dev, const void *v_rows_dev,
                                     void *kc_dev, void *vt_dev, void *out_dev, float *mass_out_dev,
                                     void *ws_dev, size_t ws_bytes, void *stream)
{
    EN_GUARDED("segmented_decode_step", segmented_decode_step_impl(pool, plan, q_first, n_rows, q_dev, k_rows_dev, v_rows_dev, kc_dev, vt_dev, out_dev, mass_out_dev, ws_dev, ws_bytes, stream));
}

// The decode step for callers that cannot allocate: the scratch is the library's static device
// array, and neither the rotary table nor the plan's descriptor block is created here.
static int segmented_decode_step_static_impl(en_pool *pool, en_plan *plan, int32_t q_first, int32_t n_rows,
                                             const void *q_dev, const void *k_rows_dev, const void *v_rows_dev,
                                             void *kc_dev, void *vt_dev, void *out_dev, float *mass_out_dev,
                                             void *stream)
{
    if (!pool || !plan)
        return fail(EN_ERR_INVALID_ARG, "segmented_decode_step_static: null argument");
    if (plan->pool != pool)
        return fail(EN_ERR_INVALID_ARG, "segmented_decode_step_static: plan belongs to another pool");
    if (n_rows <= 0)
        return fail(EN_ERR_OUT_OF_RANGE, "segmented_decode_step_static: n_rows = %d", n_rows);
    const size_t need = en_ws_layout_for(pool, plan, n_rows, step_splits(pool, plan, n_rows)).total;
    if (need > EN_STATIC_SCRATCH_BYTES)
        return fail(EN_ERR_CAPACITY, "segmented_decode_step_static: the step needs %zu bytes of scratch, the static "
                    "scratch holds %zu; use segmented_decode_step with a workspace of the caller's", need,
                    size_t(EN_STATIC_SCRATCH_BYTES));
    if (!pool->d_cos || !plan->uploaded)
        return fail(EN_ERR_INVALID_ARG, "segmented_decode_step_static: the plan has not been through gather_rope "
                    "(which creates the pool's rotary table and the plan's descriptor block); this call creates nothing");
    void *ws = nullptr;
    size_t ws_bytes = 0;
    const int e = en_static_scratch(&ws, &ws_bytes);
    if (e != 0)
        return hip_fail((hipError_t)e, "segmented_decode_step_static: address of the static scratch");
    return segmented_decode_step_impl(pool, plan, q_first, n_rows, q_dev, k_rows_dev, v_rows_dev, kc_dev, vt_dev,
                                      out_dev, mass_out_dev, ws, ws_bytes, stream);
}
extern "C" int segmented_decode_step_static(en_pool *pool, en_plan *plan, int32_t q_first, int32_t n_rows,
                                            const void *q_dev, const void *k_rows_dev, const void *v_rows_dev,
                                            void *kc_dev, void *vt_dev, void *out_dev, float *mass_out_dev,
                                            void *stream)
{
    EN_GUARDED("segmented_decode_step_static",
               segmented_decode_step_static_impl(pool, plan, q_first, n_rows, q_dev, k_rows_dev, v_rows_dev, kc_dev,
                                                 vt_dev, out_dev, mass_out_dev, stream));
}

static int segment_cluster_assign_rows_impl(en_pool *pool, en_plan *plan, int32_t q_first, int32_t n_rows,
                                           void *ws_dev, int32_t n_obj, const int32_t *span_ptr_host,
                                           int32_t per_key, int32_t accumulate, float scale, float threshold,
                                           float *score_dev, int32_t *assign_dev, void *stream)
{
    if (!pool || !plan)
        return fail(EN_ERR_INVALID_ARG, "segment_cluster_assign_rows: null argument");
    if (q_first < 0 || n_rows <= 0 || long(q_first) + n_rows > plan->Nq)
        return fail(EN_ERR_OUT_OF_RANGE, "segment_cluster_assign_rows: rows %d .. %d of %d new tokens", q_first,
                    q_first + n_rows - 1, plan->Nq);
    return cluster_assign(pool, plan, q_first, n_rows, step_splits(pool, plan, n_rows), ws_dev, n_obj, span_ptr_host,
                          per_key, accumulate, scale, threshold, score_dev, assign_dev, stream,
                          "segment_cluster_assign_rows");
}
extern "C" int segment_cluster_assign_rows(en_pool *pool, en_plan *plan, int32_t q_first, int32_t n_rows,
                                           void *ws_dev, int32_t n_obj, const int32_t *span_ptr_host,
                                           int32_t per_key, int32_t accumulate, float scale, float threshold,
                                           float *score_dev, int32_t *assign_dev, void *stream)
{
    EN_GUARDED("segment_cluster_assign_rows", segment_cluster_assign_rows_impl(pool, plan, q_first, n_rows, ws_dev, n_obj, span_ptr_host, per_key, accumulate, scale, threshold, score_dev, assign_dev, stream));
}

static int segment_attention_mass_impl(en_pool *pool, en_plan *plan, void *ws_dev, int32_t reduce,
                                      float *mass_out_dev, void *stream)
{
    if (!pool || !plan || !ws_dev || !mass_out_dev || (reduce != 0 && reduce != 1))
        return fail(EN_ERR_INVALID_ARG, "segment_attention_mass: null argument or bad reduce mode");
    if (plan->pool != pool)
        return fail(EN_ERR_INVALID_ARG, "segment_attention_mass: plan belongs to another pool");
    int rc;
    if ((rc = pool_ensure_device(pool)) != EN_OK || (rc = plan_ensure_device(plan, (hipStream_t)stream)) != EN_OK)
        return rc;
    const EnWsLayout L = en_ws_layout(pool, plan);
    char *ws = static_cast<char *>(ws_dev);
    EnMassArgs a = mass_args(pool, plan, ws, L, plan->Nq, plan->n_splits, 0);
    a.out = mass_out_dev;
    const int e = en_launch_mass(pool, a, reduce, stream);
    if (e != 0)
        return hip_fail((hipError_t)e, "segment_attention_mass launch");
    return EN_OK;
}
extern "C" int segment_attention_mass(en_pool *pool, en_plan *plan, void *ws_dev, int32_t reduce,
                                      float *mass_out_dev, void *stream)
{
    EN_GUARDED("segment_attention_mass", segment_attention_mass_impl(pool, plan, ws_dev, reduce, mass_out_dev, stream));
}

// Shared by the two entry points below: the scratch is the one an attention call over rows
// q_first .. q_first + n_rows - 1 with n_splits splits left behind.
static int cluster_assign(en_pool *pool, en_plan *plan, int q_first, int n_rows, int n_splits, void *ws_dev,
                          int32_t n_obj, const int32_t *span_ptr_host, int32_t per_key, int32_t accumulate,
                          float scale, float threshold, float *score_dev, int32_t *assign_dev, void *stream,
                          const char *who)
{
    if (!pool || !plan || !ws_dev || !span_ptr_host || !score_dev || n_obj <= 0 ||
        (per_key != 0 && per_key != 1) || (accumulate != 0 && accumulate != 1))
        return fail(EN_ERR_INVALID_ARG, "%s: null argument, no objects or bad flag", who);
    if (plan->pool != pool)
        return fail(EN_ERR_INVALID_ARG, "%s: plan belongs to another pool", who);
    if (n_obj > EN_MAX_OBJECTS)
        return fail(EN_ERR_UNSUPPORTED, "%s: %d objects, at most %d per call", who, n_obj, EN_MAX_OBJECTS);
    for (int o = 0; o < n_obj; ++o)
        if (span_ptr_host[o] < 0 || span_ptr_host[o] >= span_ptr_host[o + 1] || span_ptr_host[o + 1] > n_rows)
            return fail(EN_ERR_INVALID_ARG, "%s: object %d spans [%d, %d) of %d new tokens", who, o, span_ptr_host[o],
                        span_ptr_host[o + 1], n_rows);
    int rc;
    if ((rc = pool_ensure_device(pool)) != EN_OK || (rc = plan_ensure_device(plan, (hipStream_t)stream)) != EN_OK)
        return rc;
    const EnWsLayout L = en_ws_layout_for(pool, plan, n_rows, n_splits);
    EnClusterArgs a;
    a.m = mass_args(pool, plan, static_cast<char *>(ws_dev), L, n_rows, n_splits, q_first);
    a.score = score_dev;
    a.assign = assign_dev;
    a.n_obj = n_obj;
    a.per_key = per_key;
    a.accumulate = accumulate;
    a.scale = scale;
    a.threshold = threshold;
    std::memcpy(a.spans, span_ptr_host, size_t(n_obj + 1) * sizeof(int32_t));
    const int e = en_launch_cluster(pool, a, stream);
    if (e != 0)
        return hip_fail((hipError_t)e, who);
    return EN_OK;
}

static int segment_cluster_assign_impl(en_pool *pool, en_plan *plan, void *ws_dev, int32_t n_obj,
                                      const int32_t *span_ptr_host, int32_t per_key, int32_t accumulate,
                                      float scale, float threshold, float *score_dev, int32_t *assign_dev,
                                      void *stream)
{
    if (!plan)
        return fail(EN_ERR_INVALID_ARG, "segment_cluster_assign: null plan");
    return cluster_assign(pool, plan, 0, plan->Nq, plan->n_splits, ws_dev, n_obj, span_ptr_host, per_key, accumulate,
                          scale, threshold, score_dev, assign_dev, stream, "segment_cluster_assign");
}
extern "C" int segment_cluster_assign(en_pool *pool, en_plan *plan, void *ws_dev, int32_t n_obj,
                                      const int32_t *span_ptr_host, int32_t per_key, int32_t accumulate,
                                      float scale, float threshold, float *score_dev, int32_t *assign_dev,
                                      void *stream)
{
    EN_GUARDED("segment_cluster_assign", segment_cluster_assign_impl(pool, plan, ws_dev, n_obj, span_ptr_host, per_key, accumulate, scale, threshold, score_dev, assign_dev, stream));
}
