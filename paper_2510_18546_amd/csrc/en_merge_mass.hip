// Merge of the KV splits (log-sum-exp), per-segment attention mass and the
// clustering scores and decision of Section 3.3 of arXiv 2510.18546.
#include "en_device.h"

// ---------------------------------------------------------------------------
// combine: out = sum_sp w_sp y_sp / sum_sp w_sp with y_sp the split's own
// softmax output and w_sp = l_sp 2^(m_sp - m). One thread per 16 bytes of an
// output row. grid: ceil(rows * D / V / 256), V = elements in 16 bytes.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void mass_partial_block(const EnMassArgs &a, int blk, float *red);

// The reduced masses without a launch of their own: a head's sum for (agent, bucket) `idx` joins the
// others in ONE atomic addition on a 64-bit word that holds the sum in fixed point (so that it does
// not depend on the order in which the heads arrive) above a 10-bit count of arrivals; whoever
// arrives last (sees Hq in the count) has the complete sum in hand, from the atomic's own return
// value, and writes it out. The word was set to zero by the attention launch before.
__device__ __forceinline__ void add_reduced_mass(const EnMassArgs &a, size_t idx, float head_sum)
{
    if (!a.red_out)
        return;
    const long long q = __float2ll_rn(ldexpf(head_sum, a.red_shift));
    const unsigned long long add = ((unsigned long long)q << 10) + 1ull;
    const unsigned long long now = atomicAdd(a.red_acc + idx, add) + add;
    if ((int)(now & 1023ull) == a.Hq)
        a.red_out[idx] = ldexpf((float)((long long)(now - (unsigned long long)a.Hq) >> 10), -a.red_shift);
}

constexpr int EN_MASS_FEW_ROWS = 64;      // below this many query rows per head the partial sums go thread-wise
// Stage 1 of the reduced masses: a workgroup takes EN_MASS_BG consecutive buckets of one
// (agent, head) over all query rows (see mass_partial_block).
constexpr int EN_MASS_BG = 8;
__host__ __device__ inline int mass_bucket_groups(const EnMassArgs &m)
{
    return (m.Smax + 1 + EN_MASS_BG - 1) / EN_MASS_BG;
}
__host__ inline int mass_partial_blocks(const EnMassArgs &m)
{
    return mass_bucket_groups(m) * m.Hq * m.B;
}

// With many splits (decode over a long context by few agents) G = 4, 16 or 32 neighbouring lanes
// share a (row, 16-byte chunk): lane g takes the splits g, g + G, ... and the G partial results
// are merged with lane shuffles, so that the chain of dependent loads is 1/G as long (with 16
// lanes, up to 64 splits are one batch of loads) and the few rows of such a step make G times
// as many workgroups.
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void combine_kernel(EnAttnArgs a, EnMassArgs m, int n_comb)
{
    // head of the grid (these workgroups take longest: they start first): per-head partial sums
    // of the segment masses
    const int n_part = (int)gridDim.x - n_comb;
    if ((int)blockIdx.x < n_part) {
        __shared__ float red[4 * EN_MASS_BG];
        mass_partial_block(m, blockIdx.x, red);
        return;
    }
    constexpr int V = 16 / sizeof(T);
    typedef T tvec __attribute__((ext_vector_type(V)));
    typedef float fvec __attribute__((ext_vector_type(V)));
    const size_t rows = (size_t)a.B * a.Hq * a.Nq;
    size_t idx = (size_t)(blockIdx.x - n_part) * 256 + threadIdx.x;
    const int g = (int)(idx % G);
    idx /= G;
    if (idx >= rows * (D / V))
        return;
    const size_t row = idx / (D / V);
    const int d0 = (int)(idx % (D / V)) * V;
    // The splits are read in batches of independent loads, (reference, sum) pairs and outputs
    // together, and merged batch by batch with a running reference: read one after the other,
    // the latencies of 2 * n_splits dependent loads are what this kernel would take.
    constexpr int NB = G == 4 ? 8 : 4;
    float M = EN_NEG_INF, l = 0.f;
    fvec acc = 0.f;
    for (int sp0 = g; sp0 < a.n_splits; sp0 += NB * G) {
        f32x2 ml[NB];
        tvec v[NB];
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const bool on = sp0 + j * G < a.n_splits;
            const size_t r = (size_t)(on ? sp0 + j * G : 0) * rows + row;
            ml[j] = *reinterpret_cast<const f32x2 *>(a.ws_ml + r * 2);
            v[j] = *reinterpret_cast<const tvec *>((const T *)a.ws_opart + r * D + d0);
            if (!on)
                ml[j][0] = EN_NEG_INF;
        }
        float Mb = M;
#pragma unroll
        for (int j = 0; j < NB; ++j)
            Mb = fmaxf(Mb, ml[j][0]);
        if (Mb == EN_NEG_INF)
            continue;
        const float keep = M == EN_NEG_INF ? 0.f : fast_exp2(M - Mb);
        l *= keep;
        acc *= keep;
        M = Mb;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            // a split that saw no key of this row left (-inf, 0) and an output that is not to be used
            const float w = ml[j][0] == EN_NEG_INF ? 0.f : ml[j][1] * fast_exp2(ml[j][0] - M);
            l += w;
            acc += w == 0.f ? (fvec)0.f : __builtin_convertvector(v[j], fvec) * w;
        }
    }
    if constexpr (G > 1) {
        float Mall = M;
#pragma unroll
        for (int o = 1; o < G; o <<= 1)
            Mall = fmaxf(Mall, __shfl_xor(Mall, o, 64));
        const float keep = M == EN_NEG_INF ? 0.f : fast_exp2(M - Mall);
        l *= keep;
        acc *= keep;
        M = Mall;
#pragma unroll
        for (int o = 1; o < G; o <<= 1) {
            l += __shfl_xor(l, o, 64);
#pragma unroll
            for (int e = 0; e < V; ++e)
                acc[e] += __shfl_xor(acc[e], o, 64);
        }
        if (g != 0)
            return;
    }
    const float inv = 1.f / l;
    if (d0 == 0 && a.ws_mlfin) {
        f32x2 ml = {M, l};
        *reinterpret_cast<f32x2 *>(a.ws_mlfin + row * 2) = ml;
    }
    // 32-bit divisions (the host refuses more rows than that): a 64-bit division by a run-time
    // value is some hundred instructions, a third of this kernel
    const unsigned bh = (unsigned)row / (unsigned)a.Nq;
    const unsigned i = (unsigned)row - bh * (unsigned)a.Nq;
    const unsigned b = bh / (unsigned)a.Hq;
    const unsigned hq = bh - b * (unsigned)a.Hq;
    T *op = (T *)a.out + (((size_t)b * a.Nq + i) * a.Hq + hq) * D + d0;
    *reinterpret_cast<tvec *>(op) = __builtin_convertvector(acc * inv, tvec);
}

// ---------------------------------------------------------------------------
// ---------------------------------------------------------------------------
// mass: probability mass per (row, bucket) from the raw partial sums.
//   mass = sum over splits touching the bucket of seg * 2^(m_seg - M) / L
// with (M, L) the row's final reference maximum and sum.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void row_final_ml(const EnMassArgs &a, size_t rows, size_t row, float &M,
                                             float &L)
{
    // one split: its own (reference, sum); several: the pair the combine kernel merged
    const float *p = (a.n_splits * a.sub > 1 ? a.ws_mlfin : a.ws_ml) + row * 2;
    (void)rows;
    M = p[0];
    L = p[1];
}

// The row's reference maximum and sum merged from the splits' pairs (what the combine kernel
// writes to ws_mlfin, for code that runs beside it). Independent loads in batches of four.
__device__ __forceinline__ void merged_ml(const EnMassArgs &a, size_t rows, size_t row, float &M, float &L)
{
    constexpr int NB = 4;
    M = EN_NEG_INF;
    L = 0.f;
    const int n_part = a.n_splits * a.sub;      // partial results per row
    for (int sp0 = 0; sp0 < n_part; sp0 += NB) {
        f32x2 ml[NB];
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            ml[j] = *reinterpret_cast<const f32x2 *>(a.ws_ml + ((size_t)(sp0 + j < n_part ? sp0 + j : 0) * rows + row) * 2);
            if (sp0 + j >= n_part)
                ml[j][0] = EN_NEG_INF;
        }
        float Mb = M;
#pragma unroll
        for (int j = 0; j < NB; ++j)
            Mb = fmaxf(Mb, ml[j][0]);
        if (Mb == EN_NEG_INF)
            continue;
        L *= M == EN_NEG_INF ? 0.f : fast_exp2(M - Mb);
        M = Mb;
#pragma unroll
        for (int j = 0; j < NB; ++j)
            L += ml[j][0] == EN_NEG_INF ? 0.f : ml[j][1] * fast_exp2(ml[j][0] - M);
    }
}

// Tiles of the KV splits, one split per lane (a plan has at most 64 splits): the attention
// kernels give split sp the tiles [split_first_tile(sp), split_first_tile(sp + 1)). Code that
// has to know which splits cover a bucket asks this map with two wave votes instead of doing
// integer divisions per bucket (a division by a run-time value is some thirty instructions, and
// these kernels are bound by their instruction count).
struct EnSplitMap {
    int end_tile;                  // first tile after this lane's split; lanes >= n_splits: INT_MAX
    unsigned long long keys;       // bit sp: split sp holds at least one tile
};
// whole wave, uniform arguments
__device__ __forceinline__ EnSplitMap split_map(int n_splits, int ntiles)
{
    const unsigned q = threadIdx.x % 64;
    const unsigned bgn = split_first_tile(q, ntiles, n_splits);
    const unsigned end = split_first_tile(q + 1, ntiles, n_splits);
    EnSplitMap m;
    m.end_tile = (int)q < n_splits ? (int)end : 0x7fffffff;
    m.keys = __ballot((int)q < n_splits && end != bgn);
    return m;
}
// Splits whose key range meets bucket [blo, bhi): a contiguous range [lo, hi]. Whole wave, uniform
// arguments: the split that holds tile t is the number of splits that end at or before t.
__device__ __forceinline__ void bucket_splits(const EnSplitMap &m, int n_splits, int Ltot, int blo, int bhi,
                                              int &lo, int &hi)
{
    bhi = min(bhi, Ltot);          // a decode step's rows see less than the plan's whole new block
    const int t_lo = blo / EN_KEY_TILE, t_hi = (bhi - 1) / EN_KEY_TILE;
    const int l = (int)__popcll(__ballot(m.end_tile <= t_lo));
    const int h = (int)__popcll(__ballot(m.end_tile <= t_hi));
    lo = bhi <= blo ? n_splits : l;
    hi = bhi <= blo ? -1 : h;
}
// The same for one thread on its own (32-bit arithmetic: t * n_splits <= Ltot): the split
// that holds tile t is the largest sp whose first tile is <= t, t * n_splits / ntiles.
// Also returns the mask of the splits in [lo, hi] that hold keys.
__device__ __forceinline__ void bucket_splits_thread(int n_splits, int ntiles, int Ltot, int blo, int bhi,
                                                     int &lo, int &hi, unsigned long long &keys)
{
    bhi = min(bhi, Ltot);
    keys = 0;
    if (bhi <= blo) {
        lo = n_splits;
        hi = -1;
        return;
    }
    const unsigned t_lo = blo / EN_KEY_TILE, t_hi = (bhi - 1) / EN_KEY_TILE;
    lo = (int)(t_lo * (unsigned)n_splits / (unsigned)ntiles);
    hi = (int)(t_hi * (unsigned)n_splits / (unsigned)ntiles);
    for (int sp = lo; sp <= hi; ++sp)
        if (split_first_tile(sp, ntiles, n_splits) != split_first_tile(sp + 1, ntiles, n_splits))
            keys |= 1ull << sp;
}

__device__ __forceinline__ float row_bucket_mass(const EnMassArgs &a, int b, int hq, int i, int bucket,
                                                 int sp_lo, int sp_hi, float M, float L,
                                                 unsigned long long keys)
{
    float acc = 0.f;
    for (int sp = sp_lo; sp <= sp_hi; ++sp) {
        // an agent with fewer key tiles than the plan has splits leaves some splits without
        // keys: nothing was written for them
        if (!((keys >> sp) & 1))
            continue;
        // the waves that shared the split's tiles each left a pair of their own
        for (int w = 0; w < a.sub; ++w) {
            const f32x2 v = *reinterpret_cast<const f32x2 *>(
                a.ws_seg +
                (((((size_t)(sp * a.sub + w) * a.B + b) * a.Hq + hq) * (a.Smax + 1) + bucket) * a.Nq + i) * 2);
            if (v[1] != EN_NEG_INF)
                acc += v[0] * fast_exp2(v[1] - M);
        }
    }
    return acc / L;
}

// reduce = 0. grid: (ceil(Nq/64), Hq, B), 256 threads: the block takes 64 queries of one head.
// The scratch is laid out query-fastest, the result bucket-fastest: each wave computes the
// masses of its share of the buckets for the 64 queries (coalesced reads), the block transposes
// them through LDS, 64 buckets at a time, and writes whole runs of buckets per query.
__global__ __launch_bounds__(256) void mass_rows_kernel(EnMassArgs a)
{
    constexpr int SB = 64;                       // buckets per pass
    __shared__ float tile[64][SB + 1];
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int i = blockIdx.x * 64 + lane;
    const int hq = blockIdx.y, b = blockIdx.z;
    const bool valid = i < a.Nq;
    const size_t rows = (size_t)a.B * a.Hq * a.Nq;
    const size_t row = ((size_t)b * a.Hq + hq) * a.Nq + (valid ? i : 0);
    const int S = a.nseg[b];
    const int32_t *bnd = a.bnd + (size_t)b * (a.Smax + 2);
    const int Ltot = bnd[S] + a.q_first + a.Nq;     // end of what the rows could see
    const int ntiles = (Ltot + EN_KEY_TILE - 1) / EN_KEY_TILE;
    const EnSplitMap map = split_map(a.n_splits, ntiles);
    float M, L;
    row_final_ml(a, rows, row, M, L);
    for (int s0 = 0; s0 <= a.Smax; s0 += SB) {
        const int n = min(SB, a.Smax + 1 - s0);
        for (int c = wave; c < n; c += 4) {
            const int s = s0 + c;                 // the same for the whole wave
            float v = 0.f;
            if (s <= S && bnd[s + 1] > bnd[s]) {
                int lo, hi;
                bucket_splits(map, a.n_splits, Ltot, bnd[s], bnd[s + 1], lo, hi);
                if (valid)
                    v = row_bucket_mass(a, b, hq, i, s, lo, hi, M, L, map.keys);
            }
            tile[lane][c] = v;
        }
        __syncthreads();
        for (int r = wave; r < 64; r += 4) {
            const int ir = blockIdx.x * 64 + r;
            if (ir < a.Nq && lane < n)
                a.out[(((size_t)b * a.Nq + ir) * a.Hq + hq) * (a.Smax + 1) + s0 + lane] = tile[r][lane];
        }
        __syncthreads();
    }
}

// reduce = 1, stage 1: workgroup blk = (b * Hq + hq) * n_groups + group sums EN_MASS_BG buckets
// of one head over the queries into partial[b][s][hq]. With several KV splits this runs in the
// first workgroups of the combine launch (the partial sums are a by-product of the attention call, whatever
// the caller asks of the mass call later) and merges the splits' (reference, sum) pairs itself;
// with one split it is a launch of its own.
//
// What this costs is instructions per (row, bucket) and dependent trips to memory (about a
// microsecond each), not bytes. So lanes are rows: a row's merged (reference, sum) pair is made
// once for the group's buckets; everything that is the same for all rows (which splits cover a
// bucket, whether they hold keys) is decided from the agent's header and bounds in scalar
// registers before the rows start; and a row's loads for all buckets go out together: a bucket
// is covered by one split or by two neighbours unless it is longer than a split, so two entries
// per bucket are fetched whether or not the second one counts (it lies inside the scratch either
// way). A group with a bucket over more than two splits takes them one after the other.
// (Other forms, measured on 16 agents x 25 buckets x 32 heads x 128 rows and on the tail of the
// 8K-context merge: one workgroup per (bucket, head), all of the above per row: 23 us / 6 us;
// the same buckets in one workgroup with loads as they are needed: 27 us / 13 us; one launch that
// lets the last workgroup finish (a device-scope release per workgroup, which writes the L2
// back): 25 us; one workgroup per bucket: 14 us.)
__device__ __forceinline__ void mass_partial_block(const EnMassArgs &a, int blk, float *red)
{
    constexpr int BG = EN_MASS_BG;
    const int ng = mass_bucket_groups(a);
    const int s0 = (blk % ng) * BG;
    const int hq = (blk / ng) % a.Hq;
    const int b = blk / (ng * a.Hq);
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    float acc[BG];
#pragma unroll
    for (int j = 0; j < BG; ++j)
        acc[j] = 0.f;
    if (wave * 64 < a.Nq) {                        // a wave without rows has nothing to set up
        const size_t rows = (size_t)a.B * a.Hq * a.Nq;
        const en_table_ptr hdr = as_table(a.hdr + 4 * (size_t)b);
        const int S = hdr[0];
        const int Ltot = hdr[1] + a.q_first + a.Nq;     // end of what the rows could see
        const unsigned ntiles = (Ltot + EN_KEY_TILE - 1) / EN_KEY_TILE;
        const unsigned n = a.n_splits;
        // Bucket s0 + j is worked out by the lanes j, j + BG, ... (all of them alike), every bucket
        // of the group at once: the first split that covers it and whether that split and the one
        // after it count. Done bucket by bucket in scalar registers, this set-up was most of the
        // kernel's time: the scalar unit is shared by all waves of a compute unit.
        int lo_v, hi_v;
        bool live_v, use0_v, use1_v, next_v;
        size_t off0_v, off1_v;                          // byte offsets of the bucket's two entries of row 0
        const size_t per_split = (size_t)a.B * a.Hq * (a.Smax + 1) * a.Nq * 8;      // bytes
        {
            const int jl = lane % BG;
            const int s = min(s0 + jl, a.Smax);
            const int32_t *bnd = a.bnd + (size_t)b * (a.Smax + 2);
            const int blo = bnd[s];
            const int bhi = min(bnd[s + 1], Ltot);      // a decode step's rows see less than the whole new block
            live_v = s0 + jl <= S && bhi > blo;
            const unsigned t_lo = live_v ? blo / EN_KEY_TILE : 0, t_hi = live_v ? (bhi - 1) / EN_KEY_TILE : 0;
            // the split that holds tile t is the largest sp whose first tile is <= t
            const unsigned l = t_lo * n / ntiles, h = t_hi * n / ntiles;
            const unsigned e0 = split_first_tile(l, ntiles, n), e1 = split_first_tile(l + 1, ntiles, n),
                           e2 = split_first_tile(l + 2, ntiles, n);
            next_v = l + 1 < n;
            use0_v = live_v && e0 != e1;                // an agent with fewer tiles than splits leaves some empty
            use1_v = live_v && h > l && next_v && e1 != e2;
            lo_v = (int)l;
            hi_v = (int)h;
            off0_v = l * per_split + (((size_t)b * a.Hq + hq) * (a.Smax + 1) + s) * a.Nq * 8;
            off1_v = off0_v + (next_v ? per_split : 0);
        }
        const unsigned use0 = (unsigned)__ballot(use0_v), use1 = (unsigned)__ballot(use1_v);
        const unsigned live = (unsigned)__ballot(live_v);
        const bool simple = a.sub == 1 && __ballot(live_v && hi_v - lo_v > 1) == 0;
        int lo[BG];
#pragma unroll
        for (int j = 0; j < BG; ++j)
            lo[j] = __builtin_amdgcn_readlane(lo_v, j);
        if (simple) {
            const char *p0[BG], *p1[BG];
#pragma unroll
            for (int j = 0; j < BG; ++j) {
                p0[j] = (const char *)a.ws_seg + readlane64(off0_v, j);
                p1[j] = (const char *)a.ws_seg + readlane64(off1_v, j);
            }
            for (int i = threadIdx.x; i < a.Nq; i += 256) {
                const size_t row = ((size_t)b * a.Hq + hq) * a.Nq + i;
                f32x2 v0[BG], v1[BG];
#pragma unroll
                for (int j = 0; j < BG; ++j) {
                    v0[j] = *reinterpret_cast<const f32x2 *>(p0[j] + (unsigned)i * 8u);
                    v1[j] = *reinterpret_cast<const f32x2 *>(p1[j] + (unsigned)i * 8u);
                }
                float M, L;
                merged_ml(a, rows, row, M, L);
                const float inv = 1.f / L;
#pragma unroll
                for (int j = 0; j < BG; ++j) {
                    float part = 0.f;
                    if (((use0 >> j) & 1) && v0[j][1] != EN_NEG_INF)
                        part += v0[j][0] * fast_exp2(v0[j][1] - M);
                    if (((use1 >> j) & 1) && v1[j][1] != EN_NEG_INF)
                        part += v1[j][0] * fast_exp2(v1[j][1] - M);
                    acc[j] += part * inv;
                }
            }
        } else {
            const EnSplitMap map = split_map(a.n_splits, (int)ntiles);
            int hi[BG];
#pragma unroll
            for (int j = 0; j < BG; ++j)
                hi[j] = __builtin_amdgcn_readlane(hi_v, j);
            for (int i = threadIdx.x; i < a.Nq; i += 256) {
                const size_t row = ((size_t)b * a.Hq + hq) * a.Nq + i;
                float M, L;
                merged_ml(a, rows, row, M, L);
#pragma unroll
                for (int j = 0; j < BG; ++j)
                    if ((live >> j) & 1)
                        acc[j] += row_bucket_mass(a, b, hq, i, s0 + j, lo[j], hi[j], M, L, map.keys);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < BG; ++j) {
        const float t = wave_sum(acc[j]);
        if (lane == 0)
            red[wave * BG + j] = t;
    }
    __syncthreads();
    if (threadIdx.x < BG && s0 + (int)threadIdx.x <= a.Smax) {
        const int j = threadIdx.x;
        const float tot = red[j] + red[BG + j] + red[2 * BG + j] + red[3 * BG + j];
        a.ws_red[((size_t)b * (a.Smax + 1) + s0 + j) * a.Hq + hq] = tot;
        add_reduced_mass(a, (size_t)b * (a.Smax + 1) + s0 + j, tot);
    }
}

// The same for few query rows per head (decode steps): one THREAD per (agent, bucket, head) walks
// the rows, so that a step of one token does not launch a workgroup per (bucket, head). This form
// is a launch of its own in the mass call, whatever the number of splits: a decode step that asks
// for no masses then does no work for them.
__device__ __forceinline__ void mass_partial_few_rows(const EnMassArgs &a, size_t pair)
{
    if (pair >= (size_t)a.B * (a.Smax + 1) * a.Hq)
        return;
    const int hq = (int)(pair % a.Hq);
    const int s = (int)((pair / a.Hq) % (a.Smax + 1));
    const int b = (int)(pair / ((size_t)a.Hq * (a.Smax + 1)));
    const size_t rows = (size_t)a.B * a.Hq * a.Nq;
    const int S = a.nseg[b];
    const int32_t *bnd = a.bnd + (size_t)b * (a.Smax + 2);
    const int Ltot = bnd[S] + a.q_first + a.Nq;
    const int ntiles = (Ltot + EN_KEY_TILE - 1) / EN_KEY_TILE;
    float acc = 0.f;
    if (s <= S && bnd[s + 1] > bnd[s]) {
        int lo, hi;
        unsigned long long keys;
        bucket_splits_thread(a.n_splits, ntiles, Ltot, bnd[s], bnd[s + 1], lo, hi, keys);
        for (int i = 0; i < a.Nq; ++i) {
            const size_t row = ((size_t)b * a.Hq + hq) * a.Nq + i;
            float M, L;
            row_final_ml(a, rows, row, M, L);      // runs after the combine launch: the merged pair is there
            acc += row_bucket_mass(a, b, hq, i, s, lo, hi, M, L, keys);
        }
    }
    a.ws_red[pair] = acc;              // [b][s][hq]
    add_reduced_mass(a, (size_t)b * (a.Smax + 1) + s, acc);
}

// grid: mass_partial_blocks(a), or ceil(B (Smax+1) Hq / 256) blocks when Nq < EN_MASS_FEW_ROWS
__global__ __launch_bounds__(256) void mass_partial_kernel(EnMassArgs a)
{
    __shared__ float red[4 * EN_MASS_BG];
    if (a.Nq < EN_MASS_FEW_ROWS)
        mass_partial_few_rows(a, (size_t)blockIdx.x * 256 + threadIdx.x);
    else
        mass_partial_block(a, blockIdx.x, red);
}

// reduce = 1, stage 2. One wave per (agent, bucket) adds up the heads.
__global__ __launch_bounds__(256) void mass_final_kernel(EnMassArgs a)
{
    const int pair = blockIdx.x * 4 + threadIdx.x / 64;
    if (pair >= a.B * (a.Smax + 1))
        return;
    const float *p = a.ws_red + (size_t)pair * a.Hq;
    float acc = 0.f;
    for (int h = threadIdx.x % 64; h < a.Hq; h += 64)
        acc += p[h];
    acc = wave_sum(acc);
    if (threadIdx.x % 64 == 0)
        a.out[pair] = acc;
}

// ---------------------------------------------------------------------------
// cluster: score of every (object, segment) pair and the join / new-group
// decision of Section 3.3. Scores: grid (Smax+1, n_obj, B), 256 threads, the
// block sums the masses that the object's (token, head) pairs put on one bucket.
// Decision: one thread per (agent, object) walks that object's scores.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void cluster_score_kernel(EnClusterArgs a)
{
    __shared__ float red[4];
    const EnMassArgs &m = a.m;
    const int s = blockIdx.x, o = blockIdx.y, b = blockIdx.z;
    // the spans are read from the argument segment itself (a run-time index into a
    // by-value argument would make a private copy of the whole array)
    const int32_t *spans = reinterpret_cast<const int32_t *>(
        reinterpret_cast<uintptr_t>(__builtin_amdgcn_kernarg_segment_ptr()) + offsetof(EnClusterArgs, spans));
    const int lo = spans[o], hi = spans[o + 1];
    const int n_pairs = (hi - lo) * m.Hq;
    const size_t rows = (size_t)m.B * m.Hq * m.Nq;
    const int S = m.nseg[b];
    const int32_t *bnd = m.bnd + (size_t)b * (m.Smax + 2);
    const int Ltot = bnd[S] + m.q_first + m.Nq;     // end of what the rows could see
    const int ntiles = (Ltot + EN_KEY_TILE - 1) / EN_KEY_TILE;
    const int len = s <= S ? bnd[s + 1] - bnd[s] : 0;
    float acc = 0.f;
    const EnSplitMap map = split_map(m.n_splits, ntiles);
    if (len > 0) {
        int slo, shi;
        bucket_splits(map, m.n_splits, Ltot, bnd[s], bnd[s + 1], slo, shi);
        for (int idx = threadIdx.x; idx < n_pairs; idx += 256) {
            // token fastest: neighbouring lanes read neighbouring scratch entries
            const int hq = idx / (hi - lo), i = lo + idx % (hi - lo);
            const size_t row = ((size_t)b * m.Hq + hq) * m.Nq + i;
            float M, L;
            row_final_ml(m, rows, row, M, L);
            acc += row_bucket_mass(m, b, hq, i, s, slo, shi, M, L, map.keys);
        }
    }
    acc = wave_sum(acc);
    if (threadIdx.x % 64 == 0)
        red[threadIdx.x / 64] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float *score = a.score + ((size_t)b * a.n_obj + o) * (m.Smax + 1) + s;
        float v = (red[0] + red[1] + red[2] + red[3]) / (float)n_pairs;
        if (a.per_key && s < S && len > 0)       // the new tokens' own bucket stays a mass
            v /= (float)len;
        if (a.accumulate)
            v += *score;
        *score = v;
    }
}

__global__ __launch_bounds__(256) void cluster_decide_kernel(EnClusterArgs a)
{
    const EnMassArgs &m = a.m;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= m.B * a.n_obj)
        return;
    const int b = idx / a.n_obj;
    const int S = m.nseg[b];
    const int32_t *bnd = m.bnd + (size_t)b * (m.Smax + 2);
    const float *score = a.score + (size_t)idx * (m.Smax + 1);
    float best = EN_NEG_INF;
    int best_s = -1;
    for (int s = 0; s < S; ++s) {
        const float v = score[s] * a.scale;
        if (bnd[s + 1] > bnd[s] && v > best) {   // empty segments never win; the lowest s among equals
            best = v;
            best_s = s;
        }
    }
    a.assign[idx] = (best_s >= 0 && best >= a.threshold) ? best_s : -1;
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
int en_launch_combine(const en_pool *pool, const EnAttnArgs &a, const EnMassArgs &m, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const int D = pool->d.head_dim;
    const int vec = pool->d.dtype == EN_F32 ? 4 : 8;      // elements in 16 bytes
    // Lanes that share a (row, chunk). What the merge of a step of few rows costs is the partial
    // results per lane (each a dependent step of the running merge), not the number of workgroups:
    // about four per lane is best. Per decoded token, same box: 128 partial results by 16 / 32 / 64
    // lanes 18.0 / 17.5 / 17.9 us; 74 by 16 / 32 / 64 lanes 12.1 / 11.5 / 11.6; 32 (four agents) by
    // 4 / 16 lanes 14.0 / 13.1. A prefill's many rows fill the chip without that.
    int G = a.n_splits > 32 ? 16 : (a.n_splits > 8 ? 4 : 1);
    if ((size_t)a.B * a.Hq * a.Nq * (D / vec) <= 16384)
        G = a.n_splits > 64 ? 32 : (a.n_splits > 16 ? 16 : (a.n_splits > 4 ? 4 : 1));
    const size_t n = (size_t)a.B * a.Hq * a.Nq * (D / vec) * G;
    const int n_comb = (int)((n + 255) / 256);
    const int n_part = m.Nq < EN_MASS_FEW_ROWS ? 0 : mass_partial_blocks(m);
    const dim3 grid((unsigned)(n_comb + n_part)), blk(256);
#define EN_COMBINE(T, DD)                                                                             \
    do {                                                                                              \
        if (G == 1)                                                                                   \
            hipLaunchKernelGGL((combine_kernel<T, DD, 1>), grid, blk, 0, st, a, m, n_comb);           \
        else if (G == 4)                                                                              \
            hipLaunchKernelGGL((combine_kernel<T, DD, 4>), grid, blk, 0, st, a, m, n_comb);           \
        else if (G == 16)                                                                             \
            hipLaunchKernelGGL((combine_kernel<T, DD, 16>), grid, blk, 0, st, a, m, n_comb);          \
        else                                                                                          \
            hipLaunchKernelGGL((combine_kernel<T, DD, 32>), grid, blk, 0, st, a, m, n_comb);          \
    } while (0)
    if (pool->d.dtype == EN_F32) {
        if (D == 64)
            EN_COMBINE(float, 64);
        else
            EN_COMBINE(float, 128);
    } else {
        if (D == 64)
            EN_COMBINE(bf16_t, 64);
        else
            EN_COMBINE(bf16_t, 128);
    }
#undef EN_COMBINE
    return (int)hipGetLastError();
}

int en_launch_cluster(const en_pool *pool, const EnClusterArgs &a, void *stream)
{
    (void)pool;
    const dim3 grid(a.m.Smax + 1, a.n_obj, a.m.B), blk(256);
    hipLaunchKernelGGL(cluster_score_kernel, grid, blk, 0, (hipStream_t)stream, a);
    if (a.assign) {
        const dim3 grid2((a.m.B * a.n_obj + 255) / 256);
        hipLaunchKernelGGL(cluster_decide_kernel, grid2, blk, 0, (hipStream_t)stream, a);
    }
    return (int)hipGetLastError();
}

int en_launch_mass(const en_pool *pool, const EnMassArgs &a, int reduce, void *stream)
{
    (void)pool;
    hipStream_t st = (hipStream_t)stream;
    if (reduce == 0) {
        const dim3 grid((a.Nq + 63) / 64, a.Hq, a.B), blk(256);
        hipLaunchKernelGGL(mass_rows_kernel, grid, blk, 0, st, a);
    } else {
        // with several splits and many rows stage 1 has already run in the combine launch
        const dim3 blk(256);
        const dim3 grid = a.Nq < EN_MASS_FEW_ROWS ? dim3(((a.Smax + 1) * a.Hq * a.B + 255) / 256)
                                                  : dim3(mass_partial_blocks(a));
        if (a.n_splits * a.sub == 1 || a.Nq < EN_MASS_FEW_ROWS)
            hipLaunchKernelGGL(mass_partial_kernel, grid, blk, 0, st, a);
        if (reduce == 1) {           // reduce == 2: stage 1 only, which adds into a.red_out
            const dim3 grid2((a.B * (a.Smax + 1) + 3) / 4);
            hipLaunchKernelGGL(mass_final_kernel, grid2, blk, 0, st, a);
        }
    }
    return (int)hipGetLastError();
}
