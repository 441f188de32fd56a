// libefficientnav.so — residency tier: which groups' K/V blocks are in device
// memory, and the loads of those that are not (Section 3.2: the KV cache lives
// in a large, slow store and only the selected groups are loaded, once per
// planning step; groups selected in consecutive steps are already in device
// memory. Section 4, cache hit rate: the share of the selected groups found
// there).
//
// The device side is an ordinary en_pool whose "groups" are the tier's slots;
// the store is pinned host memory in the same [Hkv, C, D] block layout, which a
// kernel reads directly: one launch loads every missing block of a step. Loads
// run on a stream of the tier's own; two events order them against the caller's
// stream (see kv_tier_fetch).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "en_internal.h"

struct en_tier {
    en_pool_desc d;                // n_groups = number of slots
    int G = 0;                     // groups in the store
    bool dry = false;              // accounting only: no memory, no HIP calls
    en_pool *pool = nullptr;       // over the caller's slot arrays
    char *k_host = nullptr;        // pinned, [G, Hkv, C, D]
    char *v_host = nullptr;
    size_t block_bytes = 0;        // Hkv * C * D * elem
    size_t row_bytes = 0;          // D * elem
    std::vector<int32_t> len;      // [G], -1: never put
    std::vector<int32_t> slot_of;  // [G], -1: not resident
    std::vector<int32_t> group_in; // [slots], -1: free
    std::vector<int64_t> last_use; // [slots], tick of the last fetch / prefetch that asked for it, -1: never
    std::vector<char> ahead;       // [slots], loaded or kept by a prefetch and not yet asked for by a fetch
    int64_t tick = 0;              // fetches so far
    int64_t fence_tick = -1;       // readers of every slot handed out by fetches <= this tick are covered by ev_fence
    bool have_fence = false;
    bool unjoined = false;         // copies issued that no fetch has made the caller's stream wait for
    const char *k_store_dev = nullptr;   // the store as the device sees it
    const char *v_store_dev = nullptr;
    std::vector<int32_t> pending;  // blocks to load with the next launch: group, slot, tokens
    hipStream_t copy = nullptr;
    hipEvent_t ev_fence = nullptr, ev_copy = nullptr, ev_append = nullptr;
    bool append_pending = false;   // an append is writing the store on the caller's stream
    en_tier_stats st{};
};

static int tfail(int code, const char *msg)
{
    en_set_error("%s", msg);
    return code;
}

static int thip(hipError_t e, const char *what)
{
    en_set_error("%s: %s", what, hipGetErrorString(e));
    return EN_ERR_DEVICE;
}

static size_t tier_elem(int dtype) { return dtype == EN_BF16 ? 2 : 4; }

extern "C" int64_t kv_tier_slot_bytes(const en_pool_desc *desc)
{
    if (!desc || desc->capacity <= 0 || desc->n_kv_heads <= 0 || desc->head_dim <= 0)
        return 0;
    return int64_t(2) * desc->n_kv_heads * desc->capacity * desc->head_dim * int64_t(tier_elem(desc->dtype));
}

static int kv_tier_destroy_impl(en_tier *t)
{
    if (!t)
        return EN_OK;
    if (!t->dry) {
        if (t->copy)
            (void)hipStreamSynchronize(t->copy);
        if (t->ev_fence)
            (void)hipEventDestroy(t->ev_fence);
        if (t->ev_copy)
            (void)hipEventDestroy(t->ev_copy);
        if (t->ev_append) {
            (void)hipEventSynchronize(t->ev_append);
            (void)hipEventDestroy(t->ev_append);
        }
        if (t->copy)
            (void)hipStreamDestroy(t->copy);
        if (t->k_host)
            (void)hipHostFree(t->k_host);
        if (t->v_host)
            (void)hipHostFree(t->v_host);
        if (t->pool)
            (void)kv_pool_destroy(t->pool);
    }
    delete t;
    return EN_OK;
}
extern "C" int kv_tier_destroy(en_tier *t)
{
    EN_GUARDED("kv_tier_destroy", kv_tier_destroy_impl(t));
}

static int kv_tier_create_impl(const en_pool_desc *desc, int32_t n_groups_total, void *k_dev, void *v_dev,
                              en_tier **out)
{
    if (!desc || !out)
        return tfail(EN_ERR_INVALID_ARG, "kv_tier_create: null argument");
    *out = nullptr;
    if ((k_dev == nullptr) != (v_dev == nullptr))
        return tfail(EN_ERR_INVALID_ARG, "kv_tier_create: k_dev and v_dev must both be given or both be null");
    if (n_groups_total <= 0 || desc->n_groups <= 0)
        return tfail(EN_ERR_INVALID_ARG, "kv_tier_create: non-positive group or slot count");
    if (desc->dtype == EN_I8)
        return tfail(EN_ERR_UNSUPPORTED, "kv_tier_create: 8-bit pools are not served by a tier");
    en_tier *t = new (std::nothrow) en_tier;
    if (!t)
        return tfail(EN_ERR_CAPACITY, "kv_tier_create: out of host memory");
    t->d = *desc;
    t->G = n_groups_total;
    t->dry = (k_dev == nullptr);
    const int n_slots = desc->n_groups;
    std::vector<int32_t> zeros;
    try {
        t->len.assign(size_t(n_groups_total), -1);
        t->slot_of.assign(size_t(n_groups_total), -1);
        t->group_in.assign(size_t(n_slots), -1);
        t->last_use.assign(size_t(n_slots), -1);
        t->ahead.assign(size_t(n_slots), 0);
        zeros.assign(size_t(n_slots), 0);
    } catch (const std::bad_alloc &) {
        delete t;
        return tfail(EN_ERR_CAPACITY, "kv_tier_create: out of host memory for the books of the groups");
    }
    if (t->dry) {
        if (desc->capacity <= 0) {
            delete t;
            return tfail(EN_ERR_INVALID_ARG, "kv_tier_create: non-positive capacity");
        }
        *out = t;
        return EN_OK;
    }
    int rc = kv_pool_create(desc, k_dev, v_dev, zeros.data(), &t->pool);   // validates the description
    if (rc != EN_OK) {
        delete t;
        return rc;
    }
    t->row_bytes = size_t(desc->head_dim) * tier_elem(desc->dtype);
    t->block_bytes = size_t(desc->n_kv_heads) * size_t(desc->capacity) * t->row_bytes;
    hipError_t e;
    const size_t store = t->block_bytes * size_t(n_groups_total);
    if ((e = hipHostMalloc((void **)&t->k_host, store, hipHostMallocDefault)) != hipSuccess ||
        (e = hipHostMalloc((void **)&t->v_host, store, hipHostMallocDefault)) != hipSuccess) {
        rc = thip(e, "kv_tier_create: hipHostMalloc(store)");
        kv_tier_destroy(t);
        return rc;
    }
    void *kd = nullptr, *vd = nullptr;
    if ((e = hipHostGetDevicePointer(&kd, t->k_host, 0)) != hipSuccess ||
        (e = hipHostGetDevicePointer(&vd, t->v_host, 0)) != hipSuccess) {
        rc = thip(e, "kv_tier_create: hipHostGetDevicePointer");
        kv_tier_destroy(t);
        return rc;
    }
    t->k_store_dev = (const char *)kd;
    t->v_store_dev = (const char *)vd;
    if ((e = hipStreamCreateWithFlags(&t->copy, hipStreamNonBlocking)) != hipSuccess ||
        (e = hipEventCreateWithFlags(&t->ev_fence, hipEventDisableTiming)) != hipSuccess ||
        (e = hipEventCreateWithFlags(&t->ev_copy, hipEventDisableTiming)) != hipSuccess ||
        (e = hipEventCreateWithFlags(&t->ev_append, hipEventDisableTiming)) != hipSuccess) {
        rc = thip(e, "kv_tier_create: stream / event");
        kv_tier_destroy(t);
        return rc;
    }
    *out = t;
    return EN_OK;
}
extern "C" int kv_tier_create(const en_pool_desc *desc, int32_t n_groups_total, void *k_dev, void *v_dev,
                              en_tier **out)
{
    EN_GUARDED("kv_tier_create", kv_tier_create_impl(desc, n_groups_total, k_dev, v_dev, out));
}

extern "C" en_pool *kv_tier_pool(en_tier *t) { return t ? t->pool : nullptr; }

// Forget the device copy of a group. The slot keeps its age: kernels of the
// caller may still be reading it, so it is reused under the same ordering rules
// as a slot that holds a group.
static void drop_resident(en_tier *t, int group)
{
    const int s = t->slot_of[group];
    if (s < 0)
        return;
    t->slot_of[group] = -1;
    t->group_in[s] = -1;
    t->ahead[s] = 0;
    if (t->pool)
        t->pool->len[s] = 0;
}

static int kv_tier_put_impl(en_tier *t, int32_t group, const void *k_host, const void *v_host, int32_t len)
{
    if (!t || len < 0)
        return tfail(EN_ERR_INVALID_ARG, "kv_tier_put: null tier or negative length");
    if (group < 0 || group >= t->G)
        return tfail(EN_ERR_OUT_OF_RANGE, "kv_tier_put: group outside the store");
    if (len > t->d.capacity)
        return tfail(EN_ERR_OUT_OF_RANGE, "kv_tier_put: length exceeds the capacity of a block");
    if (!t->dry) {
        if (len > 0 && (!k_host || !v_host))
            return tfail(EN_ERR_INVALID_ARG, "kv_tier_put: null rows");
        // a load of this block may still be reading the store, an append writing it
        hipError_t e = hipStreamSynchronize(t->copy);
        if (e == hipSuccess && t->append_pending) {
            e = hipEventSynchronize(t->ev_append);
            t->append_pending = false;
        }
        if (e != hipSuccess)
            return thip(e, "kv_tier_put: wait for the store");
        const size_t head_src = size_t(len) * t->row_bytes;
        const size_t head_dst = size_t(t->d.capacity) * t->row_bytes;
        for (int h = 0; h < t->d.n_kv_heads && len > 0; ++h) {
            std::memcpy(t->k_host + size_t(group) * t->block_bytes + h * head_dst,
                        (const char *)k_host + h * head_src, head_src);
            std::memcpy(t->v_host + size_t(group) * t->block_bytes + h * head_dst,
                        (const char *)v_host + h * head_src, head_src);
        }
    }
    t->len[group] = len;
    drop_resident(t, group);      // the device copy, if any, is stale
    return EN_OK;
}
extern "C" int kv_tier_put(en_tier *t, int32_t group, const void *k_host, const void *v_host, int32_t len)
{
    EN_GUARDED("kv_tier_put", kv_tier_put_impl(t, group, k_host, v_host, len));
}

static int kv_tier_append_impl(en_tier *t, int32_t group, const void *k_rows_dev, const void *v_rows_dev,
                              int32_t n_tokens, void *stream)
{
    if (!t || n_tokens < 0)
        return tfail(EN_ERR_INVALID_ARG, "kv_tier_append: null tier or negative count");
    if (group < 0 || group >= t->G || t->len[group] < 0)
        return tfail(EN_ERR_OUT_OF_RANGE, "kv_tier_append: group outside the store or never put");
    const int len = t->len[group];
    if (long(len) + n_tokens > t->d.capacity)
        return tfail(EN_ERR_CAPACITY, "kv_tier_append: the block is full");
    if (n_tokens == 0)
        return EN_OK;
    if (!t->dry) {
        if (!k_rows_dev || !v_rows_dev)
            return tfail(EN_ERR_INVALID_ARG, "kv_tier_append: null rows");
        hipStream_t st = (hipStream_t)stream;
        hipError_t e;
        // loads still in flight may be reading this block of the store, or filling the slot
        if (t->unjoined) {
            if ((e = hipEventRecord(t->ev_copy, t->copy)) != hipSuccess ||
                (e = hipStreamWaitEvent(st, t->ev_copy, 0)) != hipSuccess)
                return thip(e, "kv_tier_append: join of the loads");
            t->unjoined = false;
        }
        EnAppendArgs a;
        a.k_rows = k_rows_dev;
        a.v_rows = v_rows_dev;
        a.n = n_tokens;
        a.Hkv = t->d.n_kv_heads;
        a.C = t->d.capacity;
        a.first = len;
        a.row_chunks = int(t->row_bytes / 16);
        // the store: the same copy kernel, writing host memory
        a.k_pool = const_cast<char *>(t->k_store_dev);
        a.v_pool = const_cast<char *>(t->v_store_dev);
        a.group = group;
        int rc = en_launch_append(t->pool, a, stream);
        const int slot = t->slot_of[group];
        if (rc == 0 && slot >= 0) {        // and the device copy, if there is one
            a.k_pool = t->pool->k_dev;
            a.v_pool = t->pool->v_dev;
            a.group = slot;
            rc = en_launch_append(t->pool, a, stream);
        }
        if (rc != 0)
            return thip((hipError_t)rc, "kv_tier_append: launch");
        // later loads of the block must see the new rows
        if ((e = hipEventRecord(t->ev_append, st)) != hipSuccess ||
            (e = hipStreamWaitEvent(t->copy, t->ev_append, 0)) != hipSuccess)
            return thip(e, "kv_tier_append: ordering of later loads");
        t->append_pending = true;
    }
    t->len[group] = len + n_tokens;
    const int slot = t->slot_of[group];
    if (slot >= 0 && t->pool)
        t->pool->len[slot] = len + n_tokens;
    return EN_OK;
}
extern "C" int kv_tier_append(en_tier *t, int32_t group, const void *k_rows_dev, const void *v_rows_dev,
                              int32_t n_tokens, void *stream)
{
    EN_GUARDED("kv_tier_append", kv_tier_append_impl(t, group, k_rows_dev, v_rows_dev, n_tokens, stream));
}

static int kv_tier_select_scored_impl(const en_tier *t, const float *p_host, float threshold,
                                     int64_t budget_tokens, int32_t *groups_out_host, int32_t *n_out)
{
    if (!t || !p_host || !groups_out_host || !n_out)
        return tfail(EN_ERR_INVALID_ARG, "kv_tier_select_scored: null argument");
    if (budget_tokens < 0)
        return tfail(EN_ERR_INVALID_ARG, "kv_tier_select_scored: negative budget");
    // groups never put are not candidates: give them a length no budget admits
    std::vector<int32_t> len(t->len);
    std::vector<float> p(p_host, p_host + t->G);
    for (int g = 0; g < t->G; ++g)
        if (len[g] < 0) {
            len[g] = 0;
            p[g] = threshold;     // value 0: never taken
        }
    std::vector<int32_t> chosen;
    const int krc = en_knapsack(p.data(), len.data(), t->G, threshold, budget_tokens, chosen);
    if (krc != EN_OK)
        return krc;
    *n_out = int32_t(chosen.size());
    std::copy(chosen.begin(), chosen.end(), groups_out_host);
    return EN_OK;
}
extern "C" int kv_tier_select_scored(const en_tier *t, const float *p_host, float threshold,
                                     int64_t budget_tokens, int32_t *groups_out_host, int32_t *n_out)
{
    EN_GUARDED("kv_tier_select_scored", kv_tier_select_scored_impl(t, p_host, threshold, budget_tokens, groups_out_host, n_out));
}

static int check_groups(const en_tier *t, const int32_t *groups, int n, const char *who)
{
    if (!t || n < 0 || (n > 0 && !groups)) {
        en_set_error("%s: null argument or negative count", who);
        return EN_ERR_INVALID_ARG;
    }
    if (n > t->d.n_groups) {
        en_set_error("%s: %d groups asked for, the tier has %d slots", who, n, t->d.n_groups);
        return EN_ERR_CAPACITY;
    }
    std::vector<char> seen(size_t(t->G), 0);
    for (int i = 0; i < n; ++i) {
        const int g = groups[i];
        if (g < 0 || g >= t->G || t->len[g] < 0) {
            en_set_error("%s: group %d is outside the store or was never put", who, g);
            return EN_ERR_OUT_OF_RANGE;
        }
        if (seen[g]) {
            en_set_error("%s: group %d twice", who, g);
            return EN_ERR_DUPLICATE;
        }
        seen[g] = 1;
    }
    return EN_OK;
}

// Least recently used slot among those with keep[s] == 0 and last_use <= limit;
// free slots (last_use -1) come first, ties go to the lowest index. -1: none.
static int pick_victim(const en_tier *t, const std::vector<char> &keep, int64_t limit)
{
    int best = -1;
    for (int s = 0; s < t->d.n_groups; ++s) {
        if (keep[s] || t->last_use[s] > limit)
            continue;
        if (best < 0 || t->last_use[s] < t->last_use[best])
            best = s;
    }
    return best;
}

// Count the load of `group` into `slot` and queue it for the next launch.
static void load_block(en_tier *t, int group, int slot)
{
    const int len = t->len[group];
    t->st.loads += 1;
    t->st.bytes_loaded += int64_t(2) * t->d.n_kv_heads * int64_t(len) * t->d.head_dim * int64_t(tier_elem(t->d.dtype));
    if (t->dry || len == 0)
        return;
    t->pending.push_back(group);
    t->pending.push_back(slot);
    t->pending.push_back(len);
}

// Launch the queued loads on the tier's stream, EN_TIER_LOAD_MAX blocks per launch.
static int flush_loads(en_tier *t)
{
    const size_t n_blocks = t->pending.size() / 3;
    for (size_t first = 0; first < n_blocks; first += EN_TIER_LOAD_MAX) {
        EnTierLoadArgs a;
        a.k_store = t->k_store_dev;
        a.v_store = t->v_store_dev;
        a.k_slots = (char *)t->pool->k_dev;
        a.v_slots = (char *)t->pool->v_dev;
        a.block_bytes = t->block_bytes;
        a.head_bytes = int(size_t(t->d.capacity) * t->row_bytes);
        a.row_bytes = int(t->row_bytes);
        a.Hkv = t->d.n_kv_heads;
        a.n = int(std::min<size_t>(EN_TIER_LOAD_MAX, n_blocks - first));
        int max_tokens = 0;
        for (int i = 0; i < a.n; ++i) {
            for (int j = 0; j < 3; ++j)
                a.desc[3 * i + j] = t->pending[3 * (first + i) + j];
            max_tokens = std::max(max_tokens, a.desc[3 * i + 2]);
        }
        const int e = en_launch_tier_load(a, max_tokens, t->copy);
        if (e != 0) {
            t->pending.clear();
            return thip((hipError_t)e, "kv_tier: load launch");
        }
        t->unjoined = true;
    }
    t->pending.clear();
    return EN_OK;
}

static void place(en_tier *t, int group, int slot)
{
    const int old = t->group_in[slot];
    if (old >= 0) {
        t->slot_of[old] = -1;
        t->st.evictions += 1;
    }
    t->group_in[slot] = group;
    t->slot_of[group] = slot;
    if (t->pool)
        t->pool->len[slot] = t->len[group];
}

static int kv_tier_fetch_impl(en_tier *t, const int32_t *groups_host, int32_t n, int32_t *slots_out_host,
                             void *stream)
{
    int rc = check_groups(t, groups_host, n, "kv_tier_fetch");
    if (rc != EN_OK)
        return rc;
    if (n > 0 && !slots_out_host)
        return tfail(EN_ERR_INVALID_ARG, "kv_tier_fetch: null slots_out");
    hipStream_t st = (hipStream_t)stream;
    t->pending.clear();
    t->tick += 1;
    t->st.fetches += 1;
    t->st.requested += n;
    const int n_slots = t->d.n_groups;
    std::vector<char> keep(size_t(n_slots), 0);
    // first every group that is already there, so that none of them is a victim
    for (int i = 0; i < n; ++i) {
        const int s = t->slot_of[groups_host[i]];
        if (s < 0)
            continue;
        keep[s] = 1;
        t->last_use[s] = t->tick;
        if (t->ahead[s]) {
            t->ahead[s] = 0;
            t->st.prefetched += 1;
        } else {
            t->st.hits += 1;
        }
        slots_out_host[i] = s;
    }
    bool waited = false;
    for (int i = 0; i < n; ++i) {
        const int g = groups_host[i];
        if (t->slot_of[g] >= 0)
            continue;
        const int s = pick_victim(t, keep, t->tick - 1);
        if (s < 0)
            return tfail(EN_ERR_CAPACITY, "kv_tier_fetch: no slot left");      // cannot happen: n <= slots
        if (!waited) {
            // Kernels of the caller that read the slots handed out earlier must
            // be done before a slot is overwritten. A fence the caller set after
            // enqueuing them covers fetches up to fence_tick; otherwise the fetch
            // fences for itself: everything queued on the caller's stream so far
            // is waited for, which covers every earlier fetch. (The books are kept
            // the same way by a tier without device memory.)
            hipError_t e;
            if (t->tick > 1 && t->fence_tick < t->tick - 1) {
                if (!t->dry && (e = hipEventRecord(t->ev_fence, st)) != hipSuccess)
                    return thip(e, "kv_tier_fetch: hipEventRecord");
                t->fence_tick = t->tick - 1;
                t->have_fence = true;
            }
            if (!t->dry && t->have_fence && (e = hipStreamWaitEvent(t->copy, t->ev_fence, 0)) != hipSuccess)
                return thip(e, "kv_tier_fetch: hipStreamWaitEvent");
            waited = true;
        }
        t->st.misses += 1;
        place(t, g, s);
        keep[s] = 1;
        t->last_use[s] = t->tick;
        t->ahead[s] = 0;
        slots_out_host[i] = s;
        load_block(t, g, s);
    }
    if (!t->dry && (rc = flush_loads(t)) != EN_OK)
        return rc;
    if (!t->dry && t->unjoined) {
        hipError_t e;
        if ((e = hipEventRecord(t->ev_copy, t->copy)) != hipSuccess ||
            (e = hipStreamWaitEvent(st, t->ev_copy, 0)) != hipSuccess)
            return thip(e, "kv_tier_fetch: join of the loads");
        t->unjoined = false;
    }
    return EN_OK;
}
extern "C" int kv_tier_fetch(en_tier *t, const int32_t *groups_host, int32_t n, int32_t *slots_out_host,
                             void *stream)
{
    EN_GUARDED("kv_tier_fetch", kv_tier_fetch_impl(t, groups_host, n, slots_out_host, stream));
}

static int kv_tier_fence_impl(en_tier *t, void *stream)
{
    if (!t)
        return tfail(EN_ERR_INVALID_ARG, "kv_tier_fence: null tier");
    if (!t->dry) {
        const hipError_t e = hipEventRecord(t->ev_fence, (hipStream_t)stream);
        if (e != hipSuccess)
            return thip(e, "kv_tier_fence: hipEventRecord");
    }
    t->have_fence = true;
    t->fence_tick = t->tick;
    return EN_OK;
}
extern "C" int kv_tier_fence(en_tier *t, void *stream)
{
    EN_GUARDED("kv_tier_fence", kv_tier_fence_impl(t, stream));
}

static int kv_tier_prefetch_impl(en_tier *t, const int32_t *groups_host, int32_t n, int32_t *n_loaded_out)
{
    int rc = check_groups(t, groups_host, n, "kv_tier_prefetch");
    if (rc != EN_OK)
        return rc;
    const int n_slots = t->d.n_groups;
    std::vector<char> keep(size_t(n_slots), 0);
    for (int i = 0; i < n; ++i) {
        const int s = t->slot_of[groups_host[i]];
        if (s >= 0)
            keep[s] = 1;              // stays; its age is left as it is
    }
    int loaded = 0;
    bool waited = false;
    t->pending.clear();
    for (int i = 0; i < n; ++i) {
        const int g = groups_host[i];
        if (t->slot_of[g] >= 0)
            continue;
        // only slots whose readers the fence covers: the copy may then run
        // beside whatever the caller has queued since
        const int s = pick_victim(t, keep, t->fence_tick);
        if (s < 0)
            break;
        if (!t->dry && !waited) {
            hipError_t e;
            if (t->have_fence && (e = hipStreamWaitEvent(t->copy, t->ev_fence, 0)) != hipSuccess)
                return thip(e, "kv_tier_prefetch: hipStreamWaitEvent");
            waited = true;
        }
        place(t, g, s);
        keep[s] = 1;
        // as old as the fence allows: a fetch that does not ask for it may
        // take the slot back without waiting for anything new
        t->last_use[s] = t->fence_tick;
        t->ahead[s] = 1;
        load_block(t, g, s);
        loaded += 1;
    }
    if (!t->dry && (rc = flush_loads(t)) != EN_OK)
        return rc;
    if (n_loaded_out)
        *n_loaded_out = loaded;
    return EN_OK;
}
extern "C" int kv_tier_prefetch(en_tier *t, const int32_t *groups_host, int32_t n, int32_t *n_loaded_out)
{
    EN_GUARDED("kv_tier_prefetch", kv_tier_prefetch_impl(t, groups_host, n, n_loaded_out));
}

static int kv_tier_get_stats_impl(const en_tier *t, en_tier_stats *out)
{
    if (!t || !out)
        return tfail(EN_ERR_INVALID_ARG, "kv_tier_get_stats: null argument");
    *out = t->st;
    return EN_OK;
}
extern "C" int kv_tier_get_stats(const en_tier *t, en_tier_stats *out)
{
    EN_GUARDED("kv_tier_get_stats", kv_tier_get_stats_impl(t, out));
}

static int kv_tier_residency_impl(const en_tier *t, int32_t *slot_of_group_out_host)
{
    if (!t || !slot_of_group_out_host)
        return tfail(EN_ERR_INVALID_ARG, "kv_tier_residency: null argument");
    std::copy(t->slot_of.begin(), t->slot_of.end(), slot_of_group_out_host);
    return EN_OK;
}
extern "C" int kv_tier_residency(const en_tier *t, int32_t *slot_of_group_out_host)
{
    EN_GUARDED("kv_tier_residency", kv_tier_residency_impl(t, slot_of_group_out_host));
}
