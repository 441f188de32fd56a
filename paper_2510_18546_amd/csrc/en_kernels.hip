// HIP kernels of libefficientnav.so for gfx950 (MI355X, CDNA4, wave64).
//
//   gather_k / gather_vt   index-driven gather of the selected K/V blocks into
//                          one contiguous context per agent; keys receive the
//                          rotary encoding of their concatenated position
//                          (Section 3.2 of arXiv 2510.18546: select, then load
//                          each group's KV once per planning step)
//   attn_bf16              softmax(QK^T/sqrt(D))V of the new tokens over the
//                          context (Appendix A) on the bf16 matrix cores, with
//                          an online softmax and per-segment partial sums
//   attn_f32               the same in fp32 vector arithmetic (small configs)
//   combine                merge of KV splits by log-sum-exp
//   mass                   per-segment attention mass (Section 3.3)
//
// Softmax runs in the log2 domain: scores are scaled by log2(e)/sqrt(D) and
// exponentials are exp2.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "en_internal.h"

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

#define EN_NEG_INF (-__builtin_inff())

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Exchange a value with the lane 32 positions away.
__device__ __forceinline__ float xor32(float v)
{
    // v_permlane32_swap exchanges the two halves of the wave in the vector ALU (no LDS crossbar,
    // hence no wait on the LDS counter that the operand prefetches also use)
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    // lanes 0..31 hold (own, partner) in (r[0], r[1]); lanes 32..63 in (r[1], r[0]): pick the partner
    const unsigned lane = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    return __uint_as_float(lane < 32 ? r[1] : r[0]);
}

// ---------------------------------------------------------------------------
// Segment lookup: largest s with bnd[s] <= tok among buckets 0..S (bucket S is
// the new block). Empty buckets are skipped because of the "largest".
// ---------------------------------------------------------------------------
// The plan's tables are read-only for every kernel that takes them from device
// memory. Addressed through the constant address space, their wave-uniform
// reads become scalar loads; as plain global reads they would be vector loads
// whose wait (vmcnt) also waits for every tile load in flight.
typedef const int32_t __attribute__((address_space(4))) *en_table_ptr;
__device__ __forceinline__ en_table_ptr as_table(const int32_t *p)
{
    return (en_table_ptr)(uintptr_t)p;
}

template <typename P>
__device__ __forceinline__ int find_bucket(P bnd, int S, int tok)
{
    int lo = 0, hi = S;             // invariant: bnd[lo] <= tok
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (bnd[mid] <= tok)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

// The bucket bounds and the selected groups of an agent, staged in LDS for the searches of a
// gather block: a binary search over the table in global memory is six dependent trips to memory
// per row, the group number a seventh (about 3 us before a block that moves 16 KB can issue its
// first load); over LDS it is a few hundred cycles. All threads of the block call stage_tables;
// staged = false: the tables do not fit and are read where they are.
constexpr int EN_GATHER_TAB_LDS = 256;          // entries of either table
struct EnGatherTables {
    const int32_t *bnd, *sel;                   // the agent's bounds [Smax + 2] and groups [Smax]
    bool staged;
};
__device__ __forceinline__ EnGatherTables stage_tables(const EnGatherArgs &a, int b, int32_t *lds)
{
    const int nb = a.Smax + 2;
    const int sstr = a.Smax > 0 ? a.Smax : 1;
    EnGatherTables t;
    t.bnd = a.bnd + (size_t)b * nb;
    t.sel = a.sel + (size_t)b * sstr;
    t.staged = nb <= EN_GATHER_TAB_LDS;
    if (t.staged) {
        for (int i = threadIdx.x; i < nb; i += 256)
            lds[i] = t.bnd[i];
        for (int i = threadIdx.x; i < a.Smax; i += 256)
            lds[EN_GATHER_TAB_LDS + i] = t.sel[i];
        __syncthreads();
    }
    return t;
}

// Source row of context token `tok` for (agent b, KV head kvh); nullptr for
// padding rows at or beyond L_c + N_q. `bnd` and `sel` are the agent's tables
// (global or staged), S its number of segments.
template <typename T, int D, typename P>
__device__ __forceinline__ const T *context_src(const EnGatherArgs &a, P bnd, P sel, int S, const T *pool,
                                               const T *fresh, int b, int kvh, int tok)
{
    const int Lc = bnd[S];
    const int Ltot = bnd[S + 1];
    if (tok >= Ltot)
        return nullptr;
    if (tok >= Lc)
        return fresh + (((size_t)b * a.Nq + (tok - Lc)) * a.Hkv + kvh) * D;
    const int s = find_bucket(bnd, S, tok);
    const int g = sel[s];
    return pool + (((size_t)g * a.Hkv + kvh) * a.C + (tok - bnd[s])) * D;
}

// ---------------------------------------------------------------------------
// gather_k: 8 lanes per token row. Lane c owns elements [c*E, c*E+E) of the
// first half and their rotary partners in the second half (E = D/16).
// With COPY_V (fp32 path) the value row is copied alongside.
// grid: (ceil(Lpad/32), Hkv, B), 256 threads.
// ---------------------------------------------------------------------------
template <typename T, int D, bool COPY_V, typename P>
__device__ __forceinline__ void gather_k_rows(const EnGatherArgs &a, int bx, P bnd, P sel, int S)
{
    constexpr int E = D / 16;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int tok = bx * 32 + threadIdx.x / 8;
    const int c = threadIdx.x % 8;
    const int Ltot = bnd[S + 1];
    const int Lpad = (Ltot + EN_KEY_TILE - 1) / EN_KEY_TILE * EN_KEY_TILE;
    if (tok >= Lpad)
        return;
    T *dst = (T *)a.kc + (((size_t)b * a.Hkv + kvh) * a.T + tok) * D;
    const T *src = context_src<T, D>(a, bnd, sel, S, (const T *)a.k_pool, (const T *)a.k_new, b, kvh, tok);
    typedef T tvec __attribute__((ext_vector_type(E)));
    typedef float fvec __attribute__((ext_vector_type(E)));
    fvec y1 = 0.f, y2 = 0.f;
    if (src) {
        const fvec x1 = __builtin_convertvector(*reinterpret_cast<const tvec *>(src + c * E), fvec);
        const fvec x2 = __builtin_convertvector(*reinterpret_cast<const tvec *>(src + D / 2 + c * E), fvec);
        const fvec cs = *reinterpret_cast<const fvec *>(a.cos_tab + (size_t)tok * (D / 2) + c * E);
        const fvec sn = *reinterpret_cast<const fvec *>(a.sin_tab + (size_t)tok * (D / 2) + c * E);
        y1 = x1 * cs - x2 * sn;
        y2 = x2 * cs + x1 * sn;
    }
    *reinterpret_cast<tvec *>(dst + c * E) = __builtin_convertvector(y1, tvec);
    *reinterpret_cast<tvec *>(dst + D / 2 + c * E) = __builtin_convertvector(y2, tvec);
    if constexpr (COPY_V) {
        T *vdst = (T *)a.vt + (((size_t)b * a.Hkv + kvh) * a.T + tok) * D;
        const T *vsrc = context_src<T, D>(a, bnd, sel, S, (const T *)a.v_pool, (const T *)a.v_new, b, kvh, tok);
        tvec v1 = (T)0.f, v2 = (T)0.f;
        if (vsrc) {
            v1 = *reinterpret_cast<const tvec *>(vsrc + c * E);
            v2 = *reinterpret_cast<const tvec *>(vsrc + D / 2 + c * E);
        }
        *reinterpret_cast<tvec *>(vdst + c * E) = v1;
        *reinterpret_cast<tvec *>(vdst + D / 2 + c * E) = v2;
    }
}

template <typename T, int D, bool COPY_V>
__device__ __forceinline__ void gather_k_block(const EnGatherArgs &a, int bx, int32_t *lbnd)
{
    const int b = blockIdx.z;
    const int S = a.nseg[b];
    const EnGatherTables t = stage_tables(a, b, lbnd);
    if (t.staged)
        gather_k_rows<T, D, COPY_V>(a, bx, (const int32_t *)lbnd, (const int32_t *)lbnd + EN_GATHER_TAB_LDS, S);
    else
        gather_k_rows<T, D, COPY_V>(a, bx, t.bnd, t.sel, S);
}

// ---------------------------------------------------------------------------
// gather_vt (bf16): values of a 64-token tile are staged in LDS and written
// transposed, vt[d][column], where token j sits at column j with bits 2 and 3
// exchanged. grid: (Lpad/64, Hkv, B), 256 threads.
// ---------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ void gather_vt_block(const EnGatherArgs &a, int bx, int32_t *lbnd)
{
    constexpr int STR = D + 2;                 // LDS row stride in elements
    __shared__ uint16_t tile[EN_KEY_TILE * STR];
    __shared__ const uint16_t *srcs[EN_KEY_TILE];
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int t0 = bx * EN_KEY_TILE;
    const int S = a.nseg[b];
    const EnGatherTables t = stage_tables(a, b, lbnd);
    const int32_t *lsel = lbnd + EN_GATHER_TAB_LDS;
    const int Ltot = t.staged ? lbnd[S + 1] : t.bnd[S + 1];
    if (t0 >= Ltot)                            // the same for the whole block
        return;
    if (threadIdx.x < EN_KEY_TILE) {
        const uint16_t *vp = (const uint16_t *)a.v_pool, *vn = (const uint16_t *)a.v_new;
        srcs[threadIdx.x] =
            t.staged ? context_src<uint16_t, D>(a, (const int32_t *)lbnd, lsel, S, vp, vn, b, kvh, t0 + threadIdx.x)
                     : context_src<uint16_t, D>(a, t.bnd, t.sel, S, vp, vn, b, kvh, t0 + threadIdx.x);
    }
    __syncthreads();
    // load: D/8 chunks of 16 bytes per token
    constexpr int CH = D / 8;
    for (int idx = threadIdx.x; idx < EN_KEY_TILE * CH; idx += 256) {
        const int tk = idx / CH, ch = idx % CH;
        const uint16_t *s = srcs[tk];
        uint4 v = make_uint4(0, 0, 0, 0);
        if (s)
            v = *reinterpret_cast<const uint4 *>(s + ch * 8);
        uint16_t *d = &tile[tk * STR + ch * 8];
        // STR is even but not a multiple of 8: store as 4 dwords
        reinterpret_cast<uint32_t *>(d)[0] = v.x;
        reinterpret_cast<uint32_t *>(d)[1] = v.y;
        reinterpret_cast<uint32_t *>(d)[2] = v.z;
        reinterpret_cast<uint32_t *>(d)[3] = v.w;
    }
    __syncthreads();
    // store: for every d, 8 chunks of 8 columns
    uint16_t *vt = (uint16_t *)a.vt + ((size_t)b * a.Hkv + kvh) * D * (size_t)a.T + t0;
    for (int idx = threadIdx.x; idx < D * 8; idx += 256) {
        const int d = idx / 8, ch = idx % 8;      // columns ch*8 .. ch*8+7
        const int g16 = ch / 2, hf = ch % 2;
        uint16_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int tk = 16 * g16 + 8 * (e >> 2) + 4 * hf + (e & 3);
            v[e] = tile[tk * STR + d];
        }
        uint4 o;
        o.x = v[0] | ((uint32_t)v[1] << 16);
        o.y = v[2] | ((uint32_t)v[3] << 16);
        o.z = v[4] | ((uint32_t)v[5] << 16);
        o.w = v[6] | ((uint32_t)v[7] << 16);
        *reinterpret_cast<uint4 *>(vt + (size_t)d * a.T + ch * 8) = o;
    }
}

// One launch for the whole gather: the first nk blocks of the grid's x
// dimension rotate keys (and copy fp32 values), the rest transpose bf16 values.
// When the launch carries the plan's descriptor block in its arguments, the
// tables are read from the argument segment and the first workgroup stores the
// block to device memory for the kernels that follow on the stream.
template <typename T, int D>
__global__ __launch_bounds__(256) void gather_kernel(EnGatherLaunch g)
{
    EnGatherArgs a = g.a;
    if (g.n_inline > 0) {
        const int32_t *img = reinterpret_cast<const int32_t *>(
            reinterpret_cast<uintptr_t>(__builtin_amdgcn_kernarg_segment_ptr()) + offsetof(EnGatherLaunch, desc));
        a.nseg = img + g.off_nseg;
        a.sel = img + g.off_sel;
        a.bnd = img + g.off_bnd;
        if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
            for (int i = threadIdx.x; i < g.n_inline; i += 256)
                g.desc_out[i] = img[i];
    }
    __shared__ int32_t lbnd[2 * EN_GATHER_TAB_LDS];       // bucket bounds, then selected groups
    if constexpr (sizeof(T) == 4) {
        gather_k_block<T, D, true>(a, blockIdx.x, lbnd);
    } else {
        if ((int)blockIdx.x < g.nk)
            gather_k_block<T, D, false>(a, blockIdx.x, lbnd);
        else
            gather_vt_block<D>(a, blockIdx.x - g.nk, lbnd);
    }
}

// ---------------------------------------------------------------------------
// gather from an 8-bit pool: the same bf16 contexts as above from rows of int8
// codes with one float scale per (group, head, token): value = code * scale in
// float32, keys rotated, everything rounded to bf16 once. New tokens arrive in
// bf16 as ever. grid as for the bf16 gather.
// ---------------------------------------------------------------------------
struct EnCtxLoc {
    int kind;        // 0 padding, 1 row of the pool, 2 row of the new tokens
    size_t row;      // index of the row, in rows of D elements
};
// the tables staged in LDS (at lds and lds + EN_GATHER_TAB_LDS) or where they are, see stage_tables
__device__ __forceinline__ EnCtxLoc context_loc(const EnGatherArgs &a, const EnGatherTables &t, const int32_t *lds,
                                               int b, int kvh, int tok)
{
    const int32_t *bnd = t.staged ? lds : t.bnd;
    const int32_t *sel = t.staged ? lds + EN_GATHER_TAB_LDS : t.sel;
    const int S = a.nseg[b];
    const int Lc = bnd[S];
    const int Ltot = bnd[S + 1];
    if (tok >= Ltot)
        return {0, 0};
    if (tok >= Lc)
        return {2, ((size_t)b * a.Nq + (tok - Lc)) * a.Hkv + kvh};
    const int s = find_bucket(bnd, S, tok);
    const int g = sel[s];
    return {1, ((size_t)g * a.Hkv + kvh) * a.C + (tok - bnd[s])};
}

template <int D>
__device__ __forceinline__ void gather_q8_k_block(const EnGatherArgs &a, int bx, int32_t *lds)
{
    constexpr int E = D / 16;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int tok = bx * 32 + threadIdx.x / 8;
    const int c = threadIdx.x % 8;
    const int S = a.nseg[b];
    const EnGatherTables tabs = stage_tables(a, b, lds);
    const int Ltot = tabs.staged ? lds[S + 1] : tabs.bnd[S + 1];
    const int Lpad = (Ltot + EN_KEY_TILE - 1) / EN_KEY_TILE * EN_KEY_TILE;
    if (tok >= Lpad)
        return;
    bf16_t *dst = (bf16_t *)a.kc + (((size_t)b * a.Hkv + kvh) * a.T + tok) * D;
    typedef bf16_t tvec __attribute__((ext_vector_type(E)));
    typedef float fvec __attribute__((ext_vector_type(E)));
    const EnCtxLoc loc = context_loc(a, tabs, lds, b, kvh, tok);
    fvec x1 = 0.f, x2 = 0.f;
    if (loc.kind == 1) {
        const int8_t *src = (const int8_t *)a.k_pool + loc.row * D;
        const float sc = a.k_scale[loc.row];
        int8_t c1[E], c2[E];
        __builtin_memcpy(c1, src + c * E, E);
        __builtin_memcpy(c2, src + D / 2 + c * E, E);
#pragma unroll
        for (int e = 0; e < E; ++e) {
            x1[e] = (float)c1[e] * sc;
            x2[e] = (float)c2[e] * sc;
        }
    } else if (loc.kind == 2) {
        const bf16_t *src = (const bf16_t *)a.k_new + loc.row * D;
        x1 = __builtin_convertvector(*reinterpret_cast<const tvec *>(src + c * E), fvec);
        x2 = __builtin_convertvector(*reinterpret_cast<const tvec *>(src + D / 2 + c * E), fvec);
    }
    fvec y1 = 0.f, y2 = 0.f;
    if (loc.kind != 0) {
        const fvec cs = *reinterpret_cast<const fvec *>(a.cos_tab + (size_t)tok * (D / 2) + c * E);
        const fvec sn = *reinterpret_cast<const fvec *>(a.sin_tab + (size_t)tok * (D / 2) + c * E);
        y1 = x1 * cs - x2 * sn;
        y2 = x2 * cs + x1 * sn;
    }
    *reinterpret_cast<tvec *>(dst + c * E) = __builtin_convertvector(y1, tvec);
    *reinterpret_cast<tvec *>(dst + D / 2 + c * E) = __builtin_convertvector(y2, tvec);
}

template <int D>
__device__ __forceinline__ void gather_q8_vt_block(const EnGatherArgs &a, int bx, int32_t *lds)
{
    constexpr int STR = D + 2;                 // LDS row stride in elements
    __shared__ uint16_t tile[EN_KEY_TILE * STR];
    __shared__ size_t rows[EN_KEY_TILE];
    __shared__ int kinds[EN_KEY_TILE];
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int t0 = bx * EN_KEY_TILE;
    const int S = a.nseg[b];
    const EnGatherTables tabs = stage_tables(a, b, lds);
    const int Ltot = tabs.staged ? lds[S + 1] : tabs.bnd[S + 1];
    if (t0 >= Ltot)                            // the same for the whole block
        return;
    if (threadIdx.x < EN_KEY_TILE) {
        const EnCtxLoc loc = context_loc(a, tabs, lds, b, kvh, t0 + threadIdx.x);
        rows[threadIdx.x] = loc.row;
        kinds[threadIdx.x] = loc.kind;
    }
    __syncthreads();
    typedef bf16_t bvec __attribute__((ext_vector_type(8)));
    typedef float fvec8 __attribute__((ext_vector_type(8)));
    constexpr int CH = D / 8;                  // chunks of 8 elements per token
    for (int idx = threadIdx.x; idx < EN_KEY_TILE * CH; idx += 256) {
        const int tk = idx / CH, ch = idx % CH;
        bvec v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (kinds[tk] == 1) {
            const int8_t *src = (const int8_t *)a.v_pool + rows[tk] * D + ch * 8;
            const float sc = a.v_scale[rows[tk]];
            int8_t cd[8];
            __builtin_memcpy(cd, src, 8);
            fvec8 f;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                f[e] = (float)cd[e] * sc;
            v = __builtin_convertvector(f, bvec);
        } else if (kinds[tk] == 2) {
            v = *reinterpret_cast<const bvec *>((const bf16_t *)a.v_new + rows[tk] * D + ch * 8);
        }
        uint4 raw;
        __builtin_memcpy(&raw, &v, 16);
        uint16_t *d = &tile[tk * STR + ch * 8];
        // STR is even but not a multiple of 8: store as 4 dwords
        reinterpret_cast<uint32_t *>(d)[0] = raw.x;
        reinterpret_cast<uint32_t *>(d)[1] = raw.y;
        reinterpret_cast<uint32_t *>(d)[2] = raw.z;
        reinterpret_cast<uint32_t *>(d)[3] = raw.w;
    }
    __syncthreads();
    // store: for every d, 8 chunks of 8 columns (the same order as the bf16 gather)
    uint16_t *vt = (uint16_t *)a.vt + ((size_t)b * a.Hkv + kvh) * D * (size_t)a.T + t0;
    for (int idx = threadIdx.x; idx < D * 8; idx += 256) {
        const int d = idx / 8, ch = idx % 8;      // columns ch*8 .. ch*8+7
        const int g16 = ch / 2, hf = ch % 2;
        uint16_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int tk = 16 * g16 + 8 * (e >> 2) + 4 * hf + (e & 3);
            v[e] = tile[tk * STR + d];
        }
        uint4 o;
        o.x = v[0] | ((uint32_t)v[1] << 16);
        o.y = v[2] | ((uint32_t)v[3] << 16);
        o.z = v[4] | ((uint32_t)v[5] << 16);
        o.w = v[6] | ((uint32_t)v[7] << 16);
        *reinterpret_cast<uint4 *>(vt + (size_t)d * a.T + ch * 8) = o;
    }
}

template <int D>
__global__ __launch_bounds__(256) void gather_q8_kernel(EnGatherLaunch g)
{
    EnGatherArgs a = g.a;
    if (g.n_inline > 0) {
        const int32_t *img = reinterpret_cast<const int32_t *>(
            reinterpret_cast<uintptr_t>(__builtin_amdgcn_kernarg_segment_ptr()) + offsetof(EnGatherLaunch, desc));
        a.nseg = img + g.off_nseg;
        a.sel = img + g.off_sel;
        a.bnd = img + g.off_bnd;
        if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
            for (int i = threadIdx.x; i < g.n_inline; i += 256)
                g.desc_out[i] = img[i];
    }
    __shared__ int32_t ltab[2 * EN_GATHER_TAB_LDS];       // bucket bounds, then selected groups
    if ((int)blockIdx.x < g.nk)
        gather_q8_k_block<D>(a, blockIdx.x, ltab);
    else
        gather_q8_vt_block<D>(a, blockIdx.x - g.nk, ltab);
}

// ---------------------------------------------------------------------------
// attn_bf16: matrix-core attention.
//
// Work unit: one workgroup of 8 waves = 8 (query head, 32-query block) pairs of
// one KV head and one KV split, one workgroup per compute unit, two waves per
// SIMD.
//
// Each wave keeps its 32 rotated, pre-scaled queries in registers and computes
// S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so that every lane owns ONE query
// (column l%32) and 16 scores of a 32-key block; row reductions then need a
// single exchange with lane l^32. P^T goes straight back into the matrix core
// as the B operand of O^T += V^T P^T: no LDS round trip for P.
//
// The key loop is software-pipelined over 32-key blocks. Phase j issues, step
// by step, the matrix instructions of S(j+1) = K(j+1) Q^T and of
// O += V(j-1) P(j-1), and between them the vector work that turns S(j) into
// P(j). Everything a phase reads was finished one phase earlier, so neither
// unit waits for the other.
//
// What limits a wave here is the number of instructions it issues per matrix
// instruction (a wave issues in order; scalar instructions cost it about seven
// cycles each), so the loop is kept free of scalar address arithmetic: it is
// unrolled over the three LDS stages, which turns every LDS address into a
// per-lane base plus an immediate, the loader issues unconditionally (tiles
// past the end are clamped to the last one and land in a dead stage), and the
// common case of a block is decided by one scalar and one vector comparison.
//
// K tiles [64][D] and V^T tiles [D][64] go from global memory straight into
// LDS (global_load_lds_dwordx4: 64 lanes x 16 bytes land contiguously), three
// stages each, one workgroup barrier per 64-key tile; the loads of a tile are
// spread over the steps of the two phases before it is needed. Inside a tile
// the 16-byte chunks of a row are rotated by the number of the row's 256-byte
// line (the loader does this through its per-lane source offsets), which
// keeps the operand reads of 16 consecutive lanes on distinct banks without
// padding.
//
// Element e of a 32x32 accumulator in lane l is row 8*(e/4) + 4*(l/32) + e%4,
// column l%32.
// ---------------------------------------------------------------------------

// One LDS-DMA load: lane i fetches 16 bytes from sbase + voff and the wave's
// 1024 bytes land at LDS byte address lds_base + IMM + 16*i. Completion is
// tracked by vmcnt; the compiler does not see the LDS write, so every wait is
// explicit.
template <int IMM>
__device__ __forceinline__ void dma16_imm(const void *sbase, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(voff), "s"(sbase), "n"(IMM)
                 : "memory", "scc");
}

// The same with a run-time LDS address.
__device__ __forceinline__ void dma16(const void *sbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory");
}

__device__ __forceinline__ void wait_all_memory()
{
    __builtin_amdgcn_s_waitcnt(0x0070);      // vmcnt(0) lgkmcnt(0)
}

// The loader writes LDS behind the compiler's back: after a wait or barrier
// that publishes loaded data, no LDS read may be moved up across this point.
__device__ __forceinline__ void lds_data_ready()
{
    asm volatile("" ::: "memory");
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), in order
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>{});
    }
}

__device__ __forceinline__ size_t readlane64(size_t v, int l)
{
    const unsigned lo = __builtin_amdgcn_readlane((int)(unsigned)v, l);
    const unsigned hi = __builtin_amdgcn_readlane((int)(unsigned)(v >> 32), l);
    return ((size_t)hi << 32) | lo;
}

__device__ __forceinline__ float pair_max(float v)
{
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

constexpr int ATT_WAVES = EN_WAVES;

template <int D>
__global__ __launch_bounds__(64 * ATT_WAVES) void attn_bf16_kernel(EnAttnArgs a)
{
    constexpr int KT = EN_KEY_TILE;              // keys per LDS tile
    constexpr int KB = 32;                       // keys per pipeline block
    constexpr int NKS = D / 16;                  // k-steps of one block's QK^T product
    constexpr int NDB = D / 32;                  // 32-row blocks of O^T
    constexpr int NSTEP = 2 * NKS;               // matrix instructions per phase
    constexpr int EPS = 16 / NKS;                // scores turned into P per pair of steps
    constexpr int ROWB = 2 * D;                  // bytes per K row
    constexpr int KCPR = ROWB / 16;              // 16-byte chunks per K row
    constexpr int KRPL = 256 / ROWB;             // K rows per 256-byte line
    constexpr int KBYTES = KT * ROWB;
    constexpr int VROWB = KT * 2;                // bytes per V^T row of a tile
    constexpr int VBYTES = D * VROWB;
    constexpr int NST = 3;                       // LDS stages of K and of V^T
    constexpr int VBASE = NST * KBYTES;
    constexpr int NBK = KBYTES / 1024, NBV = VBYTES / 1024;   // 1 KB loader blocks per tile
    constexpr int KJ = NBK / ATT_WAVES, VJ = NBV / ATT_WAVES; // blocks per wave
    static_assert(NBK % ATT_WAVES == 0 && NBV % ATT_WAVES == 0 && KJ <= 2 && VJ <= 2, "loader blocks");
    static_assert(KRPL == 1 || KRPL == 2, "row rotation");
    __shared__ __attribute__((aligned(1024))) char smem[NST * (KBYTES + VBYTES)];

    // ---- work decode: consecutive logical ids share K/V and map to one XCD ----
    const int per_xcd = gridDim.x / 8;
    const int logical = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (logical >= a.total_wgs)
        return;
    int t = logical;
    const int ptile = t % a.n_ptiles;
    t /= a.n_ptiles;
    const int sp = t % a.n_splits;
    t /= a.n_splits;
    const int kvh = t % a.Hkv;
    const int b = t / a.Hkv;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int lane = tid % 64;
    const int col = lane % 32, half = lane / 32;
    const int r = a.Hq / a.Hkv;
    const int nqb = (a.Nq + 31) / 32;
    const int pair = ptile * ATT_WAVES + wave;
    // A wave without a valid (head, query block) pair computes on zero queries
    // and writes nothing.
    const bool wave_valid = pair < r * nqb;
    const int hl = wave_valid ? pair % r : 0;
    const int qb = wave_valid ? pair / r : 0;
    const int hq = kvh * r + hl;
    const int i_row = qb * 32 + col;
    const bool row_valid = wave_valid && i_row < a.Nq;

    // What the workgroup needs before it can start loading: the agent's header
    // {S, L_c, L_c + N_q} in one scalar load and, when they fit one wave, all
    // bucket bounds at once, one per lane (a binary search over the table would
    // be six dependent trips to memory, about half of the start-up time).
    const int32_t *bnd_g = a.bnd + (size_t)b * (a.Smax + 2);
    const bool bnd_in_lanes = a.Smax + 2 <= 64;
    int my_bnd = 0x7fffffff;
    if (bnd_in_lanes && lane <= a.Smax + 1)
        my_bnd = bnd_g[lane];
    const en_table_ptr hdr = as_table(a.hdr + 4 * (size_t)b);
    const int S = hdr[0];
    // the rows are new tokens q_first .. q_first+Nq-1: everything before them counts as context
    const int Lc = hdr[1] + a.q_first;
    const int Ltot = Lc + a.Nq;
    const en_table_ptr bnd = as_table(bnd_g);
    auto bound_at = [&](int s) {          // s is wave-uniform
        return bnd_in_lanes ? __builtin_amdgcn_readlane(my_bnd, s) : bnd[s];
    };
    const int ntiles = (Ltot + KT - 1) / KT;
    const int t_begin = (int)((long)sp * ntiles / a.n_splits);
    int t_end = (int)((long)(sp + 1) * ntiles / a.n_splits);
    const int split_key_begin = t_begin * KT;
    const int split_key_end = min(t_end * KT, Ltot);
    {
        // causal frontier of the workgroup: last key any of its rows may see.
        // Every wave walks all tiles up to it; a wave whose own frontier is
        // earlier sees only masked scores in the last ones.
        const int qb_hi = min((ptile * ATT_WAVES + ATT_WAVES - 1) / r, nqb - 1);
        const int last_key = Lc + min(a.Nq - 1, qb_hi * 32 + 31);
        t_end = min(t_end, last_key / KT + 1);
    }
    const int nt = max(t_end - t_begin, 0);      // tiles of the workgroup
    const int i_lo = qb * 32;

    // ---- loader set-up. Block blk of a tile is LDS bytes [1024 blk, 1024 blk + 1024);
    // lane L of it is chunk q = 64 blk + L of the tile: row q / CPR, position
    // q % CPR in that row, which holds the row's chunk (position - line) mod CPR. ----
    const char *kg = (const char *)a.kc + ((size_t)b * a.Hkv + kvh) * (size_t)a.T * ROWB;
    const char *vg = (const char *)a.vt + ((size_t)b * a.Hkv + kvh) * (size_t)D * a.T * 2;
    const uint32_t lds_w = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem + wave * 1024;
    uint32_t koff[KJ], voff[VJ];
#pragma unroll
    for (int j = 0; j < KJ; ++j) {
        const int q = (wave + ATT_WAVES * j) * 64 + lane;
        const int row = q / KCPR, pos = q % KCPR;
        koff[j] = (uint32_t)(row * ROWB + ((pos - row / KRPL) & (KCPR - 1)) * 16);
    }
#pragma unroll
    for (int j = 0; j < VJ; ++j) {
        const int q = (wave + ATT_WAVES * j) * 64 + lane;
        const int d = q / 8, pos = q % 8;
        voff[j] = (uint32_t)((size_t)d * a.T * 2 + ((pos - d / 2) & 7) * 16);
    }
    // Loader job of the current phase: one tile of K or of V^T, issued block by
    // block between the matrix instructions. A tile index past the end is
    // clamped: the last tile is fetched once more, into a stage nobody reads.
    uint32_t job_goff = 0;
    auto job_k = [&](int tile) { job_goff = (uint32_t)min(tile, t_end - 1) * KBYTES; };
    auto job_v = [&](int tile) { job_goff = (uint32_t)min(tile, t_end - 1) * (KT * 2); };
    auto dma_k = [&](auto j_tag, auto stage_tag) {
        constexpr int j = decltype(j_tag)::value, stage = decltype(stage_tag)::value;
        if constexpr (j < KJ)
            dma16_imm<stage * KBYTES + j * ATT_WAVES * 1024>(kg, koff[j] + job_goff, lds_w);
    };
    auto dma_v = [&](auto j_tag, auto stage_tag) {
        constexpr int j = decltype(j_tag)::value, stage = decltype(stage_tag)::value;
        if constexpr (j < VJ)
            dma16_imm<VBASE + stage * VBYTES + j * ATT_WAVES * 1024>(vg, voff[j] + job_goff, lds_w);
    };

    // ---- first loads, issued before the queries are prepared so that both are in
    // flight together. The loop is unrolled over the three stages; the nt % 3
    // tiles that do not fill a round come first, so the first tile's stage s0
    // is chosen such that the last tile always sits in stage 2. ----
    const int rem = nt % NST;
    const int s0 = (NST - rem) % NST;
    const int s1 = (s0 + 1) % NST, s2 = (s0 + 2) % NST;
    if (nt > 0) {
        char *vz = smem + VBASE + s2 * VBYTES;     // the first product reads a zero V^T stage
        for (int i = tid * 16; i < VBYTES; i += 64 * ATT_WAVES * 16)
            *reinterpret_cast<uint4 *>(vz + i) = make_uint4(0, 0, 0, 0);
        job_k(t_begin);
#pragma unroll
        for (int j = 0; j < KJ; ++j)
            dma16(kg, koff[j] + job_goff, lds_w + s0 * KBYTES + j * ATT_WAVES * 1024);
        job_k(t_begin + 1);
#pragma unroll
        for (int j = 0; j < KJ; ++j)
            dma16(kg, koff[j] + job_goff, lds_w + s1 * KBYTES + j * ATT_WAVES * 1024);
        job_v(t_begin);
#pragma unroll
        for (int j = 0; j < VJ; ++j)
            dma16(vg, voff[j] + job_goff, lds_w + VBASE + s0 * VBYTES + j * ATT_WAVES * 1024);
    }

    // ---- operand read addresses inside a stage (plus immediates per step) ----
    uint32_t kaddr[NKS];          // K row `col` of a 32-key block, chunk 2 ks + half
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
        kaddr[ks] = (uint32_t)(col * ROWB + ((2 * ks + half + col / KRPL) & (KCPR - 1)) * 16);
    uint32_t vaddr[2][2];         // V^T row `col` of a 32-row block, keys 32 h + 16 kk + 8 half ..
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
            vaddr[h][kk] = (uint32_t)(VBASE + col * VROWB + ((4 * h + 2 * kk + half + col / 2) & 7) * 16);

    // ---- Q: load, rotate at L_c + i, scale, round to bf16 ----
    bf16x8 qf[NKS];
    {
        float qx[NKS][8];
        const bf16_t *qp = (const bf16_t *)a.q + (((size_t)b * a.Nq + i_row) * a.Hq + hq) * D + 8 * half;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (row_valid)
                v = *reinterpret_cast<const bf16x8 *>(qp + 16 * ks);
#pragma unroll
            for (int j = 0; j < 8; ++j)
                qx[ks][j] = (float)v[j];
        }
        const int pos = row_valid ? Lc + i_row : 0;
        const float *ct = a.cos_tab + (size_t)pos * (D / 2) + 8 * half;
        const float *st = a.sin_tab + (size_t)pos * (D / 2) + 8 * half;
#pragma unroll
        for (int ks = 0; ks < NKS / 2; ++ks) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float cs = ct[16 * ks + j], sn = st[16 * ks + j];
                const float x1 = qx[ks][j], x2 = qx[ks + NKS / 2][j];
                qx[ks][j] = (x1 * cs - x2 * sn) * a.scale_log2e;
                qx[ks + NKS / 2][j] = (x2 * cs + x1 * sn) * a.scale_log2e;
            }
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                qf[ks][j] = (bf16_t)qx[ks][j];
    }

    // ---- state ----
    f32x16 o[NDB];
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            o[d][e] = 0.f;
    f32x16 sbuf[2];               // scores: block j in sbuf[j%2]
    bf16x8 pbuf[2][2];            // P^T: block j in pbuf[j%2][0..1] (16 keys each)
#pragma unroll
    for (int p = 0; p < 2; ++p) {
#pragma unroll
        for (int e = 0; e < 16; ++e)
            sbuf[p][e] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                pbuf[p][kk][j] = (bf16_t)0.f;
    }
    // Softmax reference of this row (log2 units). It is chosen at the first
    // block in which the row sees a key and afterwards only moved when the
    // exponentials of a block would overflow (see phase). Scores leave the
    // matrix core already reduced by it: the accumulators start at -m_ref.
    float m_ref = 0.f;
    bool has_ref = false;
    bool pending = row_valid && Lc + i_row >= split_key_begin;   // the row will see a key in this split
    // the same as a wave mask, kept beside it: the test at the end of every phase is then one
    // vector compare, one scalar OR and one branch
    unsigned long long pend_mask = __builtin_amdgcn_ballot_w64(pending);
    f32x16 negm;
#pragma unroll
    for (int e = 0; e < 16; ++e)
        negm[e] = 0.f;
    float l_part = 0.f;           // this lane's share of the row sum
    float seg_part = 0.f;         // this lane's share of the current bucket's sum

    // bucket tracking (wave-uniform): bucket `cur` covers [cur_begin, cur_end);
    // the bound after that is fetched ahead of its use
    const int tok0 = min(split_key_begin, Ltot - 1);
    int cur = bnd_in_lanes ? (int)__popcll(__ballot(lane <= S && my_bnd <= tok0)) - 1 : find_bucket(bnd, S, tok0);
    int cur_begin = bound_at(cur);
    int cur_end = bound_at(cur + 1);
    int nxt_end = (cur + 1 <= S) ? bound_at(cur + 2) : 0x7fffffff;
    // Blocks whose first key is at most `calm` need neither the causal mask on
    // the block after them nor any bucket bookkeeping.
    auto calm_limit = [&]() {
        if (pend_mask != 0)           // rows without a reference yet: every block is looked at
            return -1;
        int m = Lc + i_lo - 2 * KB + 1;
        if (cur_end <= split_key_end)
            m = min(m, cur_end - KB - 1);
        return m;
    };
    int calm = calm_limit();
    const size_t row_hq = (size_t)b * a.Hq + hq;
    // this lane's row in the per-segment table of this split; bucket s is s * Nq rows further
    float *seg_base = a.ws_seg
                          ? a.ws_seg + ((((size_t)sp * a.B * a.Hq + row_hq) * (a.Smax + 1)) * a.Nq + i_row) * 2
                          : nullptr;

    // A closed bucket's (sum, reference) pair is written one tile later, right
    // after the next barrier: a store issued just before a barrier would make
    // that barrier's wait for the tile loads wait for the store as well.
    float pend_tot = 0.f, pend_m = 0.f;
    int pend_bucket = -1;
    auto write_pending = [&]() {
        if (pend_bucket >= 0) {
            if (seg_base && row_valid && half == 0) {
                f32x2 v = {pend_tot, pend_m};
                *reinterpret_cast<f32x2 *>(seg_base + (size_t)(pend_bucket * a.Nq) * 2) = v;
            }
            pend_bucket = -1;
        }
    };
    auto close_bucket = [&]() {
        // the whole wave: bucket `cur` has been fully consumed (or is empty)
        if (cur_end > cur_begin) {
            write_pending();
            pend_tot = seg_part + xor32(seg_part);
            pend_m = has_ref ? m_ref : EN_NEG_INF;
            pend_bucket = cur;
        }
        seg_part = 0.f;
        ++cur;
        cur_begin = cur_end;
        cur_end = (cur <= S) ? nxt_end : 0x7fffffff;
        nxt_end = (cur + 1 <= S) ? bound_at(cur + 2) : 0x7fffffff;
    };

    // Scores of the 32-key block at byte offset blk_off of the K stages,
    // relative to m_ref, unpipelined (prologue and rare path).
    auto block_scores = [&](int blk_off, f32x16 &sv) {
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const bf16x8 fr = *reinterpret_cast<const bf16x8 *>(smem + kaddr[ks] + blk_off);
            if (ks == 0)
                sv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr, qf[0], negm, 0, 0, 0);
            else
                sv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr, qf[ks], sv, 0, 0, 0);
        }
    };
    // causal / padding mask of a block starting at key kb
    auto mask_block = [&](int kb, f32x16 &sv) {
        if (kb + KB - 1 > Lc + i_lo) {
            const int rel = Lc + i_row - kb - 4 * half;      // last visible key, block-relative
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (8 * (e / 4) + (e % 4) > rel)
                    sv[e] = EN_NEG_INF;
        }
    };

    // One phase for block jb = PAR of the tile in K stage ST (global block
    // j = 2 tile + PAR):
    //   S(j+1) = K(j+1) Q^T - m_ref      NKS matrix instructions (even steps)
    //   P(j)   = exp2(S(j))              vector ALU, EPS scores per pair of steps
    //   O     += V(j-1)^T-block P(j-1)   NKS matrix instructions (odd steps)
    // plus the loader blocks of the phase's job. Operand reads run PD steps ahead.
    constexpr int PD = 4;         // operand reads run PD steps ahead, across phases too
    bf16x8 fr[PD];
    auto operand = [&](auto par_tag, auto st_tag, auto k_tag) {
        constexpr int par = decltype(par_tag)::value, st = decltype(st_tag)::value, k = decltype(k_tag)::value;
        // operand of step k of the phase (par, st): even steps read K, odd steps V^T.
        // K of block j+1: par 0 -> second half of this tile, par 1 -> first half of the next.
        // V^T of block j-1: par 0 -> keys 32..63 of the previous tile, par 1 -> keys 0..31 of this one.
        if constexpr (k % 2 == 0) {
            constexpr int off = ((st + par) % NST) * KBYTES + (par ^ 1) * KB * ROWB;
            return *reinterpret_cast<const bf16x8 *>(smem + kaddr[k / 2] + off);
        } else {
            constexpr int i = k / 2, kk = i / NDB, d = i % NDB;
            constexpr int off = ((st + NST - 1 + par) % NST) * VBYTES + d * 32 * VROWB;
            return *reinterpret_cast<const bf16x8 *>(smem + vaddr[par ^ 1][kk] + off);
        }
    };
    auto phase = [&](auto par_tag, auto st_tag, int tile) {
        constexpr int PAR = decltype(par_tag)::value, ST = decltype(st_tag)::value;
        f32x16 &s_cur = sbuf[PAR];
        f32x16 &s_nxt = sbuf[PAR ^ 1];
        float rs = 0.f;
        bf16x2 pb_hold[EPS / 2];
        static_for<NSTEP>([&](auto k_tag) {
            constexpr int k = decltype(k_tag)::value;
            constexpr int i = k / 2;
            const bf16x8 cur_fr = fr[k % PD];
            if constexpr (k + PD < NSTEP)
                fr[k % PD] = operand(par_tag, st_tag, std::integral_constant<int, (k + PD) % NSTEP>{});
            else                               // first operands of the next phase
                fr[k % PD] = operand(std::integral_constant<int, PAR ^ 1>{},
                                     std::integral_constant<int, (ST + PAR) % NST>{},
                                     std::integral_constant<int, (k + PD) % NSTEP>{});
            if constexpr (k % 2 == 0) {
                if constexpr (i == 0)
                    s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur_fr, qf[0], negm, 0, 0, 0);
                else
                    s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur_fr, qf[i], s_nxt, 0, 0, 0);
                // exponentials of scores e0 .. e0+EPS-1 of the current block
#pragma unroll
                for (int u = 0; u < EPS; u += 2) {
                    const int e = i * EPS + u;
                    const f32x2 pp = {fast_exp2(s_cur[e]), fast_exp2(s_cur[e + 1])};
                    pb_hold[u / 2] = __builtin_convertvector(pp, bf16x2);
                    // plain adds: the dot-product instructions would occupy the matrix pipeline
                    rs += pp[0];
                    rs += pp[1];
                    // keep this work in this step (the optimiser would sink it below the loop)
                    asm volatile("" : "+v"(pb_hold[u / 2]), "+v"(rs));
                }
            } else {
                constexpr int kk = i / NDB, d = i % NDB;
                o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur_fr, pbuf[PAR ^ 1][kk], o[d], 0, 0, 0);
                // file the probabilities made in the previous step
#pragma unroll
                for (int u = 0; u < EPS; u += 2) {
                    const int e = i * EPS + u;
                    pbuf[PAR][e / 8][e % 8] = pb_hold[u / 2][0];
                    pbuf[PAR][e / 8][e % 8 + 1] = pb_hold[u / 2][1];
                }
            }
            if constexpr (k == 2 || k == NSTEP / 2 + 1) {
                using j_tag = std::integral_constant<int, (k == 2) ? 0 : 1>;
                if constexpr (PAR == 0)
                    dma_k(j_tag{}, std::integral_constant<int, (ST + 2) % NST>{});
                else
                    dma_v(j_tag{}, std::integral_constant<int, (ST + 1) % NST>{});
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        const int kb = tile * KT + PAR * KB;          // first key of block j
        // Rare cases, one branch for all of them: the next block needs the causal
        // mask, a bucket ends inside this block, or a row lacks a reference /
        // came near overflow (any magnitude below that is harmless: P keeps its
        // relative precision in bf16 and the accumulators are fp32).
        constexpr float BIG = 1.0e18f;            // 2^60
        const bool overflow = __builtin_amdgcn_ballot_w64(!(rs < BIG)) != 0;     // wave-uniform
        if (kb <= calm) {                 // also says that no row lacks a reference
            if (!overflow) {
                l_part += rs;
                seg_part += rs;           // the whole block lies inside bucket `cur`
                return;
            }
        }
        const bool odd_row = overflow || pend_mask != 0;
        const int ke = min(kb + KB, split_key_end);
        mask_block(kb + KB, s_nxt);
        // ---- reference check: the wave recomputes the scores of the block,
        // moves the affected rows to their current maximum, rescales what
        // they have accumulated and redoes the exponentials ----
        if (odd_row) {
            f32x16 sv;
            block_scores(ST * KBYTES + PAR * KB * ROWB, sv);
            mask_block(kb, sv);
            float mx = sv[0];
#pragma unroll
            for (int e = 1; e < 16; ++e)
                mx = fmaxf(mx, sv[e]);
            mx = pair_max(mx);
            // both lanes of a row must take the same decision
            const float want = (pending || !(rs < BIG)) ? 1.f : 0.f;
            const bool fix = pair_max(want) > 0.f && mx > EN_NEG_INF;
            const float delta = fix ? mx : 0.f;
            const float alpha = fix ? (has_ref ? fast_exp2(-delta) : 0.f) : 1.f;
#pragma unroll
            for (int d = 0; d < NDB; ++d)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    o[d][e] *= alpha;
            l_part *= alpha;
            seg_part *= alpha;
            m_ref += delta;
            has_ref = has_ref || fix;
            pending = pending && !fix;
            pend_mask = __builtin_amdgcn_ballot_w64(pending);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                negm[e] = -m_ref;
                s_nxt[e] -= delta;            // the next block was taken against the old reference
            }
            rs = 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const bf16_t pb = (bf16_t)fast_exp2(sv[e] - delta);
                pbuf[PAR][e / 8][e % 8] = pb;
                rs += (float)pb;
            }
        }
        l_part += rs;
        // ---- per-bucket partial sums ----
        if (cur_end > ke) {
            seg_part += rs;
        } else if (cur_end == ke && cur_begin <= kb) {
            // the bucket ends exactly with this block (segments aligned to 32 keys)
            seg_part += rs;
            while (cur <= S && cur_end <= ke)
                close_bucket();
        } else if (kb < split_key_end) {
            // buckets end inside the block: every bucket but the last one met takes the sum
            // of its keys, the last one what is left of the block's sum. The keys' sums can only
            // be taken from the rounded probabilities, so for this block the row sum is taken
            // from them too: a block must give the same total to the row and to its buckets
            // (with a dominant key the difference, up to 2^-9 of it, would otherwise land in
            // whatever bucket comes next, or be lost at the end of a split).
            float rs_hat = 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e)
                rs_hat += (float)pbuf[PAR][e / 8][e % 8];
            l_part += rs_hat - rs;
            rs = rs_hat;
            float rest = rs;
            while (true) {
                const int hi = min(cur_end, ke);
                if (cur_end > ke || cur > S) {
                    seg_part += rest;
                    break;
                }
                float part = 0.f;
                const int rhi = hi - kb - 4 * half;     // keys below `hi` not yet given away
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int kr = 8 * (e / 4) + (e % 4);
                    part += (kr < rhi) ? (float)pbuf[PAR][e / 8][e % 8] : 0.f;
                }
                // `part` is the sum over keys kb .. hi-1; what earlier buckets took is in rs - rest
                part -= rs - rest;
                seg_part += part;
                rest -= part;
                close_bucket();
            }
        }
        calm = calm_limit();
    };

    // ---- main loop: one barrier per tile. Tile t_begin + n lives in stage n % 3.
    // At the barrier of tile t everything issued so far has landed: K up to
    // tile t+1, V^T up to tile t. The two phases of tile t then issue K of tile
    // t+2 and V^T of tile t+1 into stages whose last readers finished before the
    // barrier. The first product uses a zero P^T with a zero-filled V^T stage. ----
    auto tile_body = [&](auto st_tag, int tile) {
        wait_all_memory();
        __builtin_amdgcn_s_barrier();
        lds_data_ready();
        write_pending();
        job_k(tile + 2);
        phase(std::integral_constant<int, 0>{}, st_tag, tile);
        job_v(tile + 1);
        phase(std::integral_constant<int, 1>{}, st_tag, tile);
    };
    using c0 = std::integral_constant<int, 0>;
    using c1 = std::integral_constant<int, 1>;
    using c2 = std::integral_constant<int, 2>;
    if (nt > 0) {
        wait_all_memory();
        __builtin_amdgcn_s_barrier();
        lds_data_ready();
        // scores of the first block
        block_scores(s0 * KBYTES, sbuf[0]);
        mask_block(t_begin * KT, sbuf[0]);
        // first operands of the first phase: K keys 32..63 of the first tile, the zero V^T stage
#pragma unroll
        for (int k = 0; k < PD; ++k) {
            if (k % 2 == 0) {
                fr[k] = *reinterpret_cast<const bf16x8 *>(smem + kaddr[k / 2] + s0 * KBYTES + KB * ROWB);
            } else {
                const int i = k / 2, kk = i / NDB, d = i % NDB;
                fr[k] = *reinterpret_cast<const bf16x8 *>(smem + vaddr[1][kk] + s2 * VBYTES + d * 32 * VROWB);
            }
        }
        int tile = t_begin;
        if (rem == 2) {
            tile_body(c1{}, tile);
            ++tile;
        }
        if (rem >= 1) {
            tile_body(c2{}, tile);
            ++tile;
        }
        for (; tile < t_end; tile += NST) {
            tile_body(c0{}, tile);
            tile_body(c1{}, tile + 1);
            tile_body(c2{}, tile + 2);
        }
        // the last pending product: keys 32..63 of the last tile (stage 2)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int d = 0; d < NDB; ++d) {
                const bf16x8 av =
                    *reinterpret_cast<const bf16x8 *>(smem + vaddr[1][kk] + 2 * VBYTES + d * 32 * VROWB);
                o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, pbuf[1][kk], o[d], 0, 0, 0);
            }
        // loads of the clamped tiles may still be in flight
        wait_all_memory();
    }

    if (!wave_valid)
        return;
    // Buckets of this split beyond the workgroup's causal frontier still get an
    // entry (zero mass); the bucket the loop stopped in gets what is pending.
    if (seg_base) {
        while (cur <= S && cur_begin < split_key_end)
            close_bucket();
        write_pending();
    }

    // ---- epilogue ----
    const float l_tot = l_part + xor32(l_part);
    const size_t row = row_hq * a.Nq + i_row;
    if (a.ws_ml && row_valid && half == 0) {
        f32x2 v = {has_ref ? m_ref : EN_NEG_INF, l_tot};
        *reinterpret_cast<f32x2 *>(a.ws_ml + ((size_t)sp * a.B * a.Hq * a.Nq + row) * 2) = v;
    }
    if (!row_valid)
        return;
    // One split: the output row. Several: this split's own softmax output
    // (normalised by its own sum), merged by the combine kernel.
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    bf16_t *op = (a.n_splits == 1)
                     ? (bf16_t *)a.out + (((size_t)b * a.Nq + i_row) * a.Hq + hq) * D
                     : (bf16_t *)a.ws_opart + ((size_t)sp * a.B * a.Hq * a.Nq + row) * D;
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                v[e] = (bf16_t)(o[d][4 * g + e] * inv);
            *reinterpret_cast<bf16x4 *>(op + 32 * d + 8 * g + 4 * half) = v;
        }
}

// ---------------------------------------------------------------------------
// attn_decode (bf16): few query rows per KV head (r * N_q <= 32, e.g. one new
// token per agent in the decode phase of a planning step, Section 3.2: about 40
// tokens are decoded per plan over the KV that was loaded once).
//
// This case is bound by reading the gathered K / V^T once from HBM, not by the
// matrix cores, so the work is cut for bandwidth: one wave per (agent, KV head,
// KV split), no workgroup barrier at all. All r * N_q query rows of the KV head
// are columns of the wave's one 32-column Q^T block (column c = head_local *
// N_q + i). The wave streams its key range in 64-key load tiles through its own
// two LDS stages (the loads of tile j+1 run while tile j is computed): 64 keys
// are one whole 128-byte line of every V^T row, and reading V^T in half lines
// costs a fifth of the bandwidth. A tile is two 32-key blocks whose score
// chains, exponentials and products are independent of each other, which is
// all the instruction-level parallelism a wave that is alone on its SIMD has:
// S^T = K Q^T, the exponentials and O^T += V^T P^T as in the prefill kernel. Partial results of the splits are merged by the same combine
// and mass kernels.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(64) void attn_decode_kernel(EnAttnArgs a)
{
    // two LDS stages; a third (two tiles in flight per wave) was tried for grids of at most one
    // wave per compute unit and changed nothing: a lone wave is bound by issuing its own
    // instructions (about 2 us per tile), not by waiting for its loads
    constexpr int NST = 2;
    constexpr int KB = 32;                       // keys per matrix-instruction block
    constexpr int LB = EN_KEY_TILE;              // keys per tile
    constexpr int NU = LB / KB;                  // blocks per tile
    constexpr int NKS = D / 16;
    constexpr int NDB = D / 32;
    constexpr int ROWB = 2 * D;
    constexpr int KSTR = ROWB + 16;              // padded K row in LDS
    constexpr int KCPR = KSTR / 16;
    constexpr int KCHUNKS = LB * KCPR;           // 16-byte chunks of a K tile
    constexpr int NBK = KCHUNKS / 64;            // loader blocks
    constexpr int KBYTES = NBK * 1024;
    constexpr int VSTR = LB * 2 + 16;            // padded V^T row in LDS (144 bytes)
    constexpr int VCPR = VSTR / 16;
    constexpr int VCHUNKS = D * VCPR;
    constexpr int NBV = VCHUNKS / 64;
    constexpr int VBYTES = NBV * 1024;
    constexpr int STAGE = KBYTES + VBYTES;
    static_assert(KCHUNKS % 64 == 0 && VCHUNKS % 64 == 0, "tiles must be whole loader blocks");
    static_assert(NBK + NBV < 64, "the loads of one tile must fit the counter of outstanding loads");
    __shared__ __attribute__((aligned(1024))) char smem[NST * STAGE];

    // no tile is shared between waves here, so consecutive workgroups (which go
    // to different XCDs) simply take consecutive (agent, KV head, split) units
    const int logical = blockIdx.x;
    if (logical >= a.total_wgs)
        return;
    int t = logical;
    const int sp = t % a.n_splits;
    t /= a.n_splits;
    const int kvh = t % a.Hkv;
    const int b = t / a.Hkv;

    const int lane = threadIdx.x;
    const int col = lane % 32, half = lane / 32;
    const int r = a.Hq / a.Hkv;
    const bool row_valid = col < r * a.Nq;
    const int hl = row_valid ? col / a.Nq : 0;
    const int i_row = row_valid ? col % a.Nq : 0;
    const int hq = kvh * r + hl;

    // the agent's header {S, L_c, ..} in one scalar load and, when they fit the wave, all bucket
    // bounds at once, one per lane: no chain of dependent trips to memory before the first tile
    const int32_t *bnd_g = a.bnd + (size_t)b * (a.Smax + 2);
    const bool bnd_in_lanes = a.Smax + 2 <= 64;
    int my_bnd = 0x7fffffff;
    if (bnd_in_lanes && lane <= a.Smax + 1)
        my_bnd = bnd_g[lane];
    const en_table_ptr hdr = as_table(a.hdr + 4 * (size_t)b);
    const int S = hdr[0];
    const en_table_ptr bnd = as_table(bnd_g);
    auto bound_at = [&](int s) {          // s is wave-uniform
        return bnd_in_lanes ? __builtin_amdgcn_readlane(my_bnd, s) : bnd[s];
    };
    const int Lc = hdr[1] + a.q_first;       // rows are new tokens q_first .. q_first+Nq-1
    const int Ltot = Lc + a.Nq;
    const int ntiles64 = (Ltot + EN_KEY_TILE - 1) / EN_KEY_TILE;
    // split boundaries are whole 64-key tiles, as everywhere else
    const int split_key_begin = (int)((long)sp * ntiles64 / a.n_splits) * EN_KEY_TILE;
    const int split_key_end = min((int)((long)(sp + 1) * ntiles64 / a.n_splits) * EN_KEY_TILE, Ltot);
    const int t_begin = split_key_begin, t_end = split_key_end;
    const int lt_begin = split_key_begin / LB;           // load tiles; splits begin on them
    const int lt_end = (split_key_end + LB - 1) / LB;    // context rows are zero up to a multiple of 64

    // ---- loader set-up ----
    const char *kg = (const char *)a.kc + ((size_t)b * a.Hkv + kvh) * (size_t)a.T * ROWB;
    const char *vg = (const char *)a.vt + ((size_t)b * a.Hkv + kvh) * (size_t)D * a.T * 2;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;
    uint32_t koff[NBK], voff[NBV];
#pragma unroll
    for (int j = 0; j < NBK; ++j) {
        const int q = j * 64 + lane;
        const int row = q / KCPR, c = q % KCPR;
        koff[j] = (uint32_t)(row * ROWB + (c < KCPR - 1 ? c : 0) * 16);      // the pad chunk re-reads chunk 0
    }
#pragma unroll
    for (int j = 0; j < NBV; ++j) {
        const int q = j * 64 + lane;
        const int d = q / VCPR, c = q % VCPR;
        voff[j] = (uint32_t)((size_t)d * a.T * 2 + (c < VCPR - 1 ? c : 0) * 16);
    }
    auto issue = [&](int tile, int stage) {
        const char *kt = kg + (size_t)tile * (LB * ROWB);
        const char *vtile = vg + (size_t)tile * (LB * 2);
        const uint32_t dst = lds0 + stage * STAGE;
#pragma unroll
        for (int j = 0; j < NBK; ++j)
            dma16(kt, koff[j], dst + j * 1024);
#pragma unroll
        for (int j = 0; j < NBV; ++j)
            dma16(vtile, voff[j], dst + KBYTES + j * 1024);
    };

    const int klane = col * KSTR + half * 16;
    const int vlane = KBYTES + col * VSTR + half * 16;

    // ---- the step's own keys and values join the context (decode steps): new token t sits at
    // position L_c + t, and the one wave whose key range holds that position writes it: the key
    // rotated there, the value as a column of V^T, exactly as ctx_append_kernel does. Nobody else
    // reads those lines in this launch (a 64-key tile belongs to one split, a KV head to one wave),
    // and the wave itself waits for its stores to be acknowledged before it loads a tile that
    // holds a new token. The first tile is on its way meanwhile if it holds none. ----
    const int first_new = max(Lc, split_key_begin);
    const bool owns_new = a.app_k != nullptr && first_new < split_key_end;
    const bool first_tile_old = first_new >= (lt_begin + 1) * LB;
    if (t_begin < t_end && !(owns_new && !first_tile_old))
        issue(lt_begin, 0);
    // Lane c owns the rotary pairs (c, c + D/2), c + 64, ... of a token. The first new token's
    // row is fetched here, together with the queries below; the stores follow the queries.
    constexpr int APP_J = (D / 2 + 63) / 64;
    float app_x1[APP_J], app_x2[APP_J], app_cs[APP_J], app_sn[APP_J];
    bf16_t app_v1[APP_J], app_v2[APP_J];
    auto app_load = [&](int t) {
        const int pos = Lc + t;
        const bf16_t *kr = (const bf16_t *)a.app_k + (((size_t)b * a.Nq + t) * a.Hkv + kvh) * D;
        const bf16_t *vr = (const bf16_t *)a.app_v + (((size_t)b * a.Nq + t) * a.Hkv + kvh) * D;
#pragma unroll
        for (int j = 0; j < APP_J; ++j) {
            const int c = min(lane + 64 * j, D / 2 - 1);
            app_cs[j] = a.cos_tab[(size_t)pos * (D / 2) + c];
            app_sn[j] = a.sin_tab[(size_t)pos * (D / 2) + c];
            app_x1[j] = (float)kr[c];
            app_x2[j] = (float)kr[c + D / 2];
            app_v1[j] = vr[c];
            app_v2[j] = vr[c + D / 2];
        }
    };
    auto app_store = [&](int t) {
        const int pos = Lc + t;
        bf16_t *kd = (bf16_t *)a.kc + (((size_t)b * a.Hkv + kvh) * a.T + pos) * D;
        // token j in column j with bits 2 and 3 exchanged
        const int vcol = (pos & ~0xC) | ((pos & 4) << 1) | ((pos & 8) >> 1);
        bf16_t *vd = (bf16_t *)a.vt + ((size_t)b * a.Hkv + kvh) * (size_t)D * a.T + vcol;
#pragma unroll
        for (int j = 0; j < APP_J; ++j) {
            const int c = lane + 64 * j;
            if (c < D / 2) {
                kd[c] = (bf16_t)(app_x1[j] * app_cs[j] - app_x2[j] * app_sn[j]);
                kd[c + D / 2] = (bf16_t)(app_x2[j] * app_cs[j] + app_x1[j] * app_sn[j]);
                vd[(size_t)c * a.T] = app_v1[j];
                vd[(size_t)(c + D / 2) * a.T] = app_v2[j];
            }
        }
    };
    if (owns_new)
        app_load(first_new - Lc);

    // ---- Q: load, rotate at L_c + i, scale, round to bf16 ----
    bf16x8 qf[NKS];
    {
        bf16x8 qraw[NKS];
        const bf16_t *qp = (const bf16_t *)a.q + (((size_t)b * a.Nq + i_row) * a.Hq + hq) * D + 8 * half;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            qraw[ks] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            if (row_valid)
                qraw[ks] = *reinterpret_cast<const bf16x8 *>(qp + 16 * ks);
        }
        const int pos = row_valid ? Lc + i_row : 0;
        const float *ct = a.cos_tab + (size_t)pos * (D / 2) + 8 * half;
        const float *st = a.sin_tab + (size_t)pos * (D / 2) + 8 * half;
        float cs[NKS / 2][8], sn[NKS / 2][8];
#pragma unroll
        for (int ks = 0; ks < NKS / 2; ++ks)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                cs[ks][j] = ct[16 * ks + j];
                sn[ks][j] = st[16 * ks + j];
            }
        // the new tokens' stores go out between the loads of the queries and the arithmetic on
        // them, so that their acknowledgement is under way while the queries are rotated
        if (owns_new) {
            int t = first_new - Lc;
            app_store(t);
            for (++t; t < a.Nq && Lc + t < split_key_end; ++t) {
                app_load(t);
                app_store(t);
            }
            if (!first_tile_old) {
                wait_all_memory();                   // stores included
                issue(lt_begin, 0);
            }
        }
        float qx[NKS][8];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                qx[ks][j] = (float)qraw[ks][j];
#pragma unroll
        for (int ks = 0; ks < NKS / 2; ++ks) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float x1 = qx[ks][j], x2 = qx[ks + NKS / 2][j];
                qx[ks][j] = (x1 * cs[ks][j] - x2 * sn[ks][j]) * a.scale_log2e;
                qx[ks + NKS / 2][j] = (x2 * cs[ks][j] + x1 * sn[ks][j]) * a.scale_log2e;
            }
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                qf[ks][j] = (bf16_t)qx[ks][j];
    }

    // ---- state (see the prefill kernel for the softmax reference scheme) ----
    f32x16 o[NDB];
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            o[d][e] = 0.f;
    float m_ref = 0.f;
    bool has_ref = false;
    bool pending = row_valid && Lc + i_row >= split_key_begin;
    f32x16 negm;
#pragma unroll
    for (int e = 0; e < 16; ++e)
        negm[e] = 0.f;
    float l_part = 0.f, seg_part = 0.f;

    const int tok0 = min(split_key_begin, Ltot - 1);
    int cur = bnd_in_lanes ? (int)__popcll(__ballot(lane <= S && my_bnd <= tok0)) - 1 : find_bucket(bnd, S, tok0);
    int cur_begin = bound_at(cur);
    int cur_end = bound_at(cur + 1);
    int nxt_end = (cur + 1 <= S) ? bound_at(cur + 2) : 0x7fffffff;
    const size_t row_hq = (size_t)b * a.Hq + hq;
    float *seg_base = a.ws_seg
                          ? a.ws_seg + (((size_t)sp * a.B * a.Hq + row_hq) * (a.Smax + 1)) * a.Nq * 2
                          : nullptr;
    auto close_bucket = [&]() {
        if (cur_end > cur_begin) {
            const float tot = seg_part + xor32(seg_part);
            if (seg_base && row_valid && half == 0) {
                f32x2 v = {tot, has_ref ? m_ref : EN_NEG_INF};
                *reinterpret_cast<f32x2 *>(seg_base + ((size_t)cur * a.Nq + i_row) * 2) = v;
            }
        }
        seg_part = 0.f;
        ++cur;
        cur_begin = cur_end;
        cur_end = (cur <= S) ? nxt_end : 0x7fffffff;
        nxt_end = (cur + 1 <= S) ? bound_at(cur + 2) : 0x7fffffff;
    };

    // the stores of new tokens are acknowledged before the loop loads the tile that holds them
    // (the loads of the queries went out in the meantime)
    if (owns_new && first_tile_old)
        wait_all_memory();
    int stage = 0;                               // of tile lt
    for (int lt = lt_begin; lt < lt_end; ++lt) {
        const char *stg = smem + stage * STAGE;
        // every LDS read of the previous tile has returned (its matrix
        // instructions consumed them), so its stage may be overwritten
        __builtin_amdgcn_s_waitcnt(0xc07f);                  // lgkmcnt(0)
        constexpr int PER_TILE = NBK + NBV;
        if (lt + 1 < lt_end) {
            issue(lt + 1, stage ^ 1);
            // this tile's loads have landed when at most the next tile's are outstanding
            __builtin_amdgcn_s_waitcnt((PER_TILE & 15) | ((PER_TILE >> 4) << 14) | 0x0f70);
        } else {
            __builtin_amdgcn_s_waitcnt(0x0f70);              // vmcnt(0)
        }
        lds_data_ready();
        const int kb = lt * LB;
        // ---- S^T = K Q^T - m_ref, the two 32-key blocks as independent chains ----
        f32x16 sv[NU];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const bf16x8 fr = *reinterpret_cast<const bf16x8 *>(stg + u * (KB * KSTR) + klane + ks * 32);
                sv[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr, qf[ks], ks == 0 ? negm : sv[u], 0, 0, 0);
            }
        // causal / padding mask; columns differ in i, so every tile that reaches
        // past L_c is checked. Element e of block u is key 32 u + 8 (e / 4) + e % 4 + 4 half of the tile.
        if (kb + LB - 1 > Lc) {
            const int rel = Lc + i_row - kb - 4 * half;
#pragma unroll
            for (int u = 0; u < NU; ++u)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    if (KB * u + 8 * (e / 4) + (e % 4) > rel)
                        sv[u][e] = EN_NEG_INF;
        }
        // ---- reference (first visible tile, or near overflow) ----
        constexpr float BIG = 1.0e18f;
        bf16x8 pf[NU][2];
        float rs = 0.f;
        {
            float p[NU][16];
#pragma unroll
            for (int u = 0; u < NU; ++u)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    p[u][e] = fast_exp2(sv[u][e]);
                    rs += p[u][e];
                }
            if (__any(pending || !(rs < BIG))) {
                float mx = sv[0][0];
#pragma unroll
                for (int u = 0; u < NU; ++u)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        mx = fmaxf(mx, sv[u][e]);
                mx = pair_max(mx);
                const float want = (pending || !(rs < BIG)) ? 1.f : 0.f;
                const bool fix = pair_max(want) > 0.f && mx > EN_NEG_INF;
                const float delta = fix ? mx : 0.f;
                const float alpha = fix ? (has_ref ? fast_exp2(-delta) : 0.f) : 1.f;
#pragma unroll
                for (int d = 0; d < NDB; ++d)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        o[d][e] *= alpha;
                l_part *= alpha;
                seg_part *= alpha;
                m_ref += delta;
                has_ref = has_ref || fix;
                pending = pending && !fix;
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    negm[e] = -m_ref;
#pragma unroll
                for (int u = 0; u < NU; ++u)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        p[u][e] = fast_exp2(sv[u][e] - delta);
            }
            // the sums use the rounded probabilities, like the products
            rs = 0.f;
#pragma unroll
            for (int u = 0; u < NU; ++u)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const bf16_t pb = (bf16_t)p[u][e];
                    pf[u][e / 8][e % 8] = pb;
                    rs += (float)pb;
                }
        }
        l_part += rs;
        // ---- per-bucket partial sums ----
        const int ke = min(kb + LB, split_key_end);
        if (cur_end > ke) {
            seg_part += rs;
        } else if (kb < split_key_end) {
            int lo = kb;
            while (true) {
                const int hi = min(cur_end, ke);
                float part = 0.f;
                const int rlo = lo - kb - 4 * half, rhi = hi - kb - 4 * half;
#pragma unroll
                for (int u = 0; u < NU; ++u)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int kr = KB * u + 8 * (e / 4) + (e % 4);
                        part += (kr >= rlo && kr < rhi) ? (float)pf[u][e / 8][e % 8] : 0.f;
                    }
                seg_part += part;
                if (cur_end > ke || cur > S)
                    break;
                close_bucket();
                lo = hi;
            }
        }
        // ---- O^T += V^T P^T ----
#pragma unroll
        for (int u = 0; u < NU; ++u)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                for (int d = 0; d < NDB; ++d) {
                    const bf16x8 av = *reinterpret_cast<const bf16x8 *>(stg + u * (KB * 2) + vlane + kk * 32 + d * 32 * VSTR);
                    o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, pf[u][kk], o[d], 0, 0, 0);
                }
        stage ^= 1;
    }

    if (seg_base)
        while (cur <= S && cur_begin < split_key_end)
            close_bucket();

    const float l_tot = l_part + xor32(l_part);
    const size_t row = row_hq * a.Nq + i_row;
    if (a.ws_ml && row_valid && half == 0) {
        f32x2 v = {has_ref ? m_ref : EN_NEG_INF, l_tot};
        *reinterpret_cast<f32x2 *>(a.ws_ml + ((size_t)sp * a.B * a.Hq * a.Nq + row) * 2) = v;
    }
    if (!row_valid)
        return;
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    bf16_t *op = (a.n_splits == 1)
                     ? (bf16_t *)a.out + (((size_t)b * a.Nq + i_row) * a.Hq + hq) * D
                     : (bf16_t *)a.ws_opart + ((size_t)sp * a.B * a.Hq * a.Nq + row) * D;
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                v[e] = (bf16_t)(o[d][4 * g + e] * inv);
            *reinterpret_cast<bf16x4 *>(op + 32 * d + 8 * g + 4 * half) = v;
        }
}

// ---------------------------------------------------------------------------
// attn_f32: one wave per (agent, head, query) row and KV split. Lanes stride
// over the keys with a private online softmax; lanes are merged at each bucket
// end (for the mass) and at the end of the row.
// grid: (ceil(rows/4), n_splits), 256 threads.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v += __shfl_xor(v, o, 64);
    return v;
}

template <int D>
__global__ __launch_bounds__(256) void attn_f32_kernel(EnAttnArgs a)
{
    __shared__ float qs[4][D];
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const size_t rows = (size_t)a.B * a.Hq * a.Nq;
    const size_t row = (size_t)blockIdx.x * 4 + wave;
    const int sp = blockIdx.y;
    const bool valid = row < rows;
    // row = (b*Hq + hq)*Nq + i
    const int i = valid ? (int)(row % a.Nq) : 0;
    const int hq = valid ? (int)((row / a.Nq) % a.Hq) : 0;
    const int b = valid ? (int)(row / ((size_t)a.Nq * a.Hq)) : 0;
    const int r = a.Hq / a.Hkv;
    const int kvh = hq / r;
    const int S = a.nseg[b];
    const int32_t *bnd = a.bnd + (size_t)b * (a.Smax + 2);
    const int Lc = bnd[S] + a.q_first;       // rows are new tokens q_first .. q_first+Nq-1
    const int Ltot = Lc + a.Nq;
    const int ntiles = (Ltot + EN_KEY_TILE - 1) / EN_KEY_TILE;
    const int kbeg = (int)((long)sp * ntiles / a.n_splits) * EN_KEY_TILE;
    const int kend_split = min((int)((long)(sp + 1) * ntiles / a.n_splits) * EN_KEY_TILE, Ltot);
    const int kend = min(kend_split, Lc + i + 1);       // causal limit

    // rotated, scaled query in LDS
    if (valid && lane < D / 2) {
        const float *qp = (const float *)a.q + (((size_t)b * a.Nq + i) * a.Hq + hq) * D;
        const int pos = Lc + i;
        const float cs = a.cos_tab[(size_t)pos * (D / 2) + lane];
        const float sn = a.sin_tab[(size_t)pos * (D / 2) + lane];
        const float x1 = qp[lane], x2 = qp[lane + D / 2];
        qs[wave][lane] = (x1 * cs - x2 * sn) * a.scale_log2e;
        qs[wave][lane + D / 2] = (x2 * cs + x1 * sn) * a.scale_log2e;
    }
    __syncthreads();
    if (!valid)
        return;

    const float *K = (const float *)a.kc + ((size_t)b * a.Hkv + kvh) * (size_t)a.T * D;
    const float *V = (const float *)a.vt + ((size_t)b * a.Hkv + kvh) * (size_t)a.T * D;
    float m = EN_NEG_INF, l = 0.f;
    float o[D];
#pragma unroll
    for (int d = 0; d < D; ++d)
        o[d] = 0.f;
    float *seg_base = a.ws_seg ? a.ws_seg + ((((size_t)sp * a.B + b) * a.Hq + hq) * (a.Smax + 1)) * a.Nq * 2
                               : nullptr;

    for (int bucket = 0; bucket <= S; ++bucket) {
        const int lo = max(bnd[bucket], kbeg);
        const int hi = min(bnd[bucket + 1], kend);
        const bool touches = bnd[bucket + 1] > bnd[bucket] && max(bnd[bucket], kbeg) < min(bnd[bucket + 1], kend_split);
        float seg = 0.f, seg_m = m;
        for (int j = lo + lane; j < hi; j += 64) {
            const float *kr = K + (size_t)j * D;
            float acc = 0.f;
#pragma unroll
            for (int d = 0; d < D; d += 4) {
                const f32x4 kv = *reinterpret_cast<const f32x4 *>(kr + d);
                acc += qs[wave][d] * kv[0] + qs[wave][d + 1] * kv[1] + qs[wave][d + 2] * kv[2] +
                       qs[wave][d + 3] * kv[3];
            }
            const float mn = fmaxf(m, acc);
            const float alpha = exp2f(m - mn);      // m = -inf -> 0
            const float p = exp2f(acc - mn);
            l = l * alpha + p;
            seg = seg * alpha + p;
            const float *vr = V + (size_t)j * D;
#pragma unroll
            for (int d = 0; d < D; d += 4) {
                const f32x4 vv = *reinterpret_cast<const f32x4 *>(vr + d);
                o[d] = o[d] * alpha + p * vv[0];
                o[d + 1] = o[d + 1] * alpha + p * vv[1];
                o[d + 2] = o[d + 2] * alpha + p * vv[2];
                o[d + 3] = o[d + 3] * alpha + p * vv[3];
            }
            m = mn;
        }
        seg_m = m;
        if (touches && seg_base) {
            // merge the lanes' partial sums of this bucket
            const float M = wave_max(seg_m);
            const float w = (seg_m == EN_NEG_INF) ? 0.f : exp2f(seg_m - M);
            const float tot = wave_sum(seg * w);
            if (lane == 0) {
                f32x2 v = {tot, M};
                *reinterpret_cast<f32x2 *>(seg_base + ((size_t)bucket * a.Nq + i) * 2) = v;
            }
        }
    }
    // merge lanes
    const float M = wave_max(m);
    const float w = (m == EN_NEG_INF) ? 0.f : exp2f(m - M);
    const float l_tot = wave_sum(l * w);
    if (a.ws_ml && lane == 0) {
        f32x2 v = {M, l_tot};
        *reinterpret_cast<f32x2 *>(a.ws_ml + ((size_t)sp * rows + row) * 2) = v;
    }
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    float *op = (a.n_splits == 1) ? (float *)a.out + (((size_t)b * a.Nq + i) * a.Hq + hq) * D
                                  : (float *)a.ws_opart + ((size_t)sp * rows + row) * D;
#pragma unroll
    for (int d = 0; d < D; ++d) {
        const float tot = wave_sum(o[d] * w);
        if (lane == (d & 63))
            op[d] = tot * inv;
    }
}

// ---------------------------------------------------------------------------
// combine: out = sum_sp w_sp y_sp / sum_sp w_sp with y_sp the split's own
// softmax output and w_sp = l_sp 2^(m_sp - m). One thread per 16 bytes of an
// output row. grid: ceil(rows * D / V / 256), V = elements in 16 bytes.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void mass_partial_block(const EnMassArgs &a, int blk, float *red);
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

// With many splits (decode over a long context by few agents) G = 4 or 16 neighbouring lanes
// share a (row, 16-byte chunk): lane g takes the splits g, g + G, ... and the G partial results
// are merged with lane shuffles, so that the chain of dependent loads is 1/G as long (with 16
// lanes, up to 64 splits are one batch of loads) and the few rows of such a step make G times
// as many workgroups.
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void combine_kernel(EnAttnArgs a, EnMassArgs m, int n_comb)
{
    // tail of the grid: per-head partial sums of the segment masses
    if ((int)blockIdx.x >= n_comb) {
        __shared__ float red[4 * EN_MASS_BG];
        mass_partial_block(m, blockIdx.x - n_comb, red);
        return;
    }
    constexpr int V = 16 / sizeof(T);
    typedef T tvec __attribute__((ext_vector_type(V)));
    typedef float fvec __attribute__((ext_vector_type(V)));
    const size_t rows = (size_t)a.B * a.Hq * a.Nq;
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
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
        const float keep = M == EN_NEG_INF ? 0.f : exp2f(M - Mb);
        l *= keep;
        acc *= keep;
        M = Mb;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            // a split that saw no key of this row left (-inf, 0) and an output that is not to be used
            const float w = ml[j][0] == EN_NEG_INF ? 0.f : ml[j][1] * exp2f(ml[j][0] - M);
            l += w;
            acc += w == 0.f ? (fvec)0.f : __builtin_convertvector(v[j], fvec) * w;
        }
    }
    if constexpr (G > 1) {
        float Mall = M;
#pragma unroll
        for (int o = 1; o < G; o <<= 1)
            Mall = fmaxf(Mall, __shfl_xor(Mall, o, 64));
        const float keep = M == EN_NEG_INF ? 0.f : exp2f(M - Mall);
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
    const float *p = (a.n_splits > 1 ? a.ws_mlfin : a.ws_ml) + row * 2;
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
    for (int sp0 = 0; sp0 < a.n_splits; sp0 += NB) {
        f32x2 ml[NB];
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            ml[j] = *reinterpret_cast<const f32x2 *>(a.ws_ml + ((size_t)(sp0 + j < a.n_splits ? sp0 + j : 0) * rows + row) * 2);
            if (sp0 + j >= a.n_splits)
                ml[j][0] = EN_NEG_INF;
        }
        float Mb = M;
#pragma unroll
        for (int j = 0; j < NB; ++j)
            Mb = fmaxf(Mb, ml[j][0]);
        if (Mb == EN_NEG_INF)
            continue;
        L *= M == EN_NEG_INF ? 0.f : exp2f(M - Mb);
        M = Mb;
#pragma unroll
        for (int j = 0; j < NB; ++j)
            L += ml[j][0] == EN_NEG_INF ? 0.f : ml[j][1] * exp2f(ml[j][0] - M);
    }
}

// Tiles of the KV splits, one split per lane (a plan has at most 64 splits): the attention
// kernels give split sp the tiles [sp * ntiles / n_splits, (sp + 1) * ntiles / n_splits). Code that
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
    const unsigned bgn = q * (unsigned)ntiles / (unsigned)n_splits;
    const unsigned end = (q + 1) * (unsigned)ntiles / (unsigned)n_splits;
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
// The same for one thread on its own (32-bit arithmetic: (t + 1) * n_splits <= Ltot + 64): the split
// that holds tile t is the largest sp whose first tile is <= t, ((t + 1) * n_splits - 1) / ntiles.
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
    lo = (int)(((t_lo + 1) * (unsigned)n_splits - 1) / (unsigned)ntiles);
    hi = (int)(((t_hi + 1) * (unsigned)n_splits - 1) / (unsigned)ntiles);
    for (int sp = lo; sp <= hi; ++sp)
        if ((unsigned)sp * (unsigned)ntiles / (unsigned)n_splits !=
            (unsigned)(sp + 1) * (unsigned)ntiles / (unsigned)n_splits)
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
        const f32x2 v = *reinterpret_cast<const f32x2 *>(
            a.ws_seg + (((((size_t)sp * a.B + b) * a.Hq + hq) * (a.Smax + 1) + bucket) * a.Nq + i) * 2);
        if (v[1] != EN_NEG_INF)
            acc += v[0] * exp2f(v[1] - M);
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
// of one head over the queries into partial[b][s][hq]. With several KV splits this runs as the
// tail of the combine launch (the partial sums are a by-product of the attention call, whatever
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
            const unsigned l = ((t_lo + 1) * n - 1) / ntiles, h = ((t_hi + 1) * n - 1) / ntiles;
            const unsigned e0 = l * ntiles / n, e1 = (l + 1) * ntiles / n, e2 = (l + 2) * ntiles / n;
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
        const bool simple = __ballot(live_v && hi_v - lo_v > 1) == 0;
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
        a.ws_red[((size_t)b * (a.Smax + 1) + s0 + j) * a.Hq + hq] =
            red[j] + red[BG + j] + red[2 * BG + j] + red[3 * BG + j];
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
// ctx_append: the keys and values of a decode step's new tokens join the
// gathered context at positions L_c + q_first + t (keys rotated there; values
// in the context's layout). grid: (n, Hkv, B), D/2 threads: thread c owns the
// rotary pair (c, c + D/2).
// ---------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(D / 2) void ctx_append_kernel(EnCtxAppendArgs a)
{
    const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int c = threadIdx.x;
    const int pos = a.hdr[4 * b + 1] + a.q_first + t;
    const T *kr = (const T *)a.k_rows + (((size_t)b * a.n + t) * a.Hkv + h) * D;
    const T *vr = (const T *)a.v_rows + (((size_t)b * a.n + t) * a.Hkv + h) * D;
    const float cs = a.cos_tab[(size_t)pos * (D / 2) + c], sn = a.sin_tab[(size_t)pos * (D / 2) + c];
    const float x1 = (float)kr[c], x2 = (float)kr[c + D / 2];
    T *kd = (T *)a.kc + (((size_t)b * a.Hkv + h) * a.T + pos) * D;
    kd[c] = (T)(x1 * cs - x2 * sn);
    kd[c + D / 2] = (T)(x2 * cs + x1 * sn);
    if constexpr (sizeof(T) == 4) {
        T *vd = (T *)a.vt + (((size_t)b * a.Hkv + h) * a.T + pos) * D;
        vd[c] = vr[c];
        vd[c + D / 2] = vr[c + D / 2];
    } else {
        // transposed layout [D][T], token j in column j with bits 2 and 3 exchanged
        const int col = (pos & ~0xC) | ((pos & 4) << 1) | ((pos & 8) >> 1);
        T *vd = (T *)a.vt + ((size_t)b * a.Hkv + h) * (size_t)D * a.T + col;
        vd[(size_t)c * a.T] = vr[c];
        vd[(size_t)(c + D / 2) * a.T] = vr[c + D / 2];
    }
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
// tier load: blocks of the pinned host store go to device slots (Section 3.2:
// the selected groups' KV is loaded from the slow store, once). The kernel
// reads host memory directly, 16 bytes per lane and four loads in flight per
// lane, so one launch moves every missing block of a step and, unlike a chain
// of copy commands, queues behind an event without holding up the host.
// grid: (chunks of 16 KB along a head's used rows, 2 * Hkv, blocks), 256 threads.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void tier_load_kernel(EnTierLoadArgs a)
{
    const int32_t *desc = reinterpret_cast<const int32_t *>(
        reinterpret_cast<uintptr_t>(__builtin_amdgcn_kernarg_segment_ptr()) + offsetof(EnTierLoadArgs, desc));
    const int m = blockIdx.z;
    const int group = desc[3 * m], slot = desc[3 * m + 1], tokens = desc[3 * m + 2];
    const int h = blockIdx.y >> 1, is_v = blockIdx.y & 1;
    const int units = tokens * (a.row_bytes / 16);           // 16-byte units of this head in use
    const int first = blockIdx.x * 1024 + threadIdx.x;
    if (blockIdx.x * 1024 >= units)
        return;
    const size_t head_off = (size_t)h * a.head_bytes;
    const uint4 *src = reinterpret_cast<const uint4 *>((is_v ? a.v_store : a.k_store) +
                                                       (size_t)group * a.block_bytes + head_off);
    uint4 *dst = reinterpret_cast<uint4 *>((is_v ? a.v_slots : a.k_slots) + (size_t)slot * a.block_bytes + head_off);
    uint4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (first + 256 * j < units)
            v[j] = src[first + 256 * j];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (first + 256 * j < units)
            dst[first + 256 * j] = v[j];
}

// ---------------------------------------------------------------------------
// append: rows [n, Hkv, D] go to tokens first .. first+n-1 of one group's block
// [Hkv, C, D] in both pool arrays (Section 3.2: new objects' KV is saved at the
// end of the group's cache). One thread per 16 bytes; grid.y: 0 keys, 1 values.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void append_kernel(EnAppendArgs a)
{
    // n rows of one group: n <= C, so the chunk count fits 32 bits with room to spare
    const unsigned idx = blockIdx.x * 256u + threadIdx.x;
    const unsigned total = (unsigned)a.n * a.Hkv * a.row_chunks;
    if (idx >= total)
        return;
    const unsigned rowi = idx / (unsigned)a.row_chunks;          // tok * Hkv + h
    const unsigned c = idx - rowi * (unsigned)a.row_chunks;
    const unsigned tok = rowi / (unsigned)a.Hkv;
    const unsigned h = rowi - tok * (unsigned)a.Hkv;
    const uint4 *src = reinterpret_cast<const uint4 *>(blockIdx.y == 0 ? a.k_rows : a.v_rows);
    uint4 *dst = reinterpret_cast<uint4 *>(blockIdx.y == 0 ? a.k_pool : a.v_pool);
    const size_t drow = ((size_t)a.group * a.Hkv + h) * a.C + a.first + tok;
    dst[drow * a.row_chunks + c] = src[(size_t)rowi * a.row_chunks + c];
}

// ---------------------------------------------------------------------------
// append to an 8-bit pool: one wave per (token, head) row and array. The row's
// largest magnitude fixes the scale (max|x| / 127), the codes are x / scale
// rounded to the nearest integer, ties to even, all in float32; a zero row has
// scale 0. grid: (n, Hkv, 2), 64 threads.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(64) void append_q8_kernel(EnAppendQ8Args a)
{
    constexpr int EPL = D / 64;               // elements per lane
    const int tok = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const bf16_t *src = (const bf16_t *)(blockIdx.z == 0 ? a.k_rows : a.v_rows) + ((size_t)tok * a.Hkv + h) * D;
    float x[EPL];
    float amax = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        x[e] = (float)src[lane * EPL + e];
        amax = fmaxf(amax, fabsf(x[e]));
    }
    amax = wave_max(amax);
    const float scale = amax / 127.0f;
    const size_t row = ((size_t)a.group * a.Hkv + h) * a.C + a.first + tok;
    int8_t *dst = (blockIdx.z == 0 ? a.k_pool : a.v_pool) + row * D;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        float q = scale > 0.f ? rintf(x[e] / scale) : 0.f;
        q = fminf(fmaxf(q, -127.f), 127.f);
        dst[lane * EPL + e] = (int8_t)(int)q;
    }
    if (lane == 0)
        (blockIdx.z == 0 ? a.k_scale : a.v_scale)[row] = scale;
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
int en_launch_gather(const en_pool *pool, EnGatherLaunch &g, int max_ctx_len, void *stream)
{
    const EnGatherArgs &a = g.a;
    hipStream_t st = (hipStream_t)stream;
    const int Lpad = (max_ctx_len + EN_KEY_TILE - 1) / EN_KEY_TILE * EN_KEY_TILE;
    const int nk = (Lpad + 31) / 32, nv = Lpad / EN_KEY_TILE;
    g.nk = nk;
    const dim3 blk(256);
    const int D = pool->d.head_dim;
    if (pool->d.dtype == EN_F32) {
        const dim3 grid(nk, a.Hkv, a.B);
        if (D == 64)
            hipLaunchKernelGGL((gather_kernel<float, 64>), grid, blk, 0, st, g);
        else
            hipLaunchKernelGGL((gather_kernel<float, 128>), grid, blk, 0, st, g);
    } else if (pool->d.dtype == EN_I8) {
        const dim3 grid(nk + nv, a.Hkv, a.B);
        if (D == 64)
            hipLaunchKernelGGL((gather_q8_kernel<64>), grid, blk, 0, st, g);
        else
            hipLaunchKernelGGL((gather_q8_kernel<128>), grid, blk, 0, st, g);
    } else {
        const dim3 grid(nk + nv, a.Hkv, a.B);
        if (D == 64)
            hipLaunchKernelGGL((gather_kernel<bf16_t, 64>), grid, blk, 0, st, g);
        else
            hipLaunchKernelGGL((gather_kernel<bf16_t, 128>), grid, blk, 0, st, g);
    }
    return (int)hipGetLastError();
}

int en_launch_attention(const en_pool *pool, const EnAttnArgs &a, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const int D = pool->d.head_dim;
    if (pool->d.dtype == EN_F32) {
        const size_t rows = (size_t)a.B * a.Hq * a.Nq;
        const dim3 grid((unsigned)((rows + 3) / 4), a.n_splits), blk(256);
        if (D == 64)
            hipLaunchKernelGGL((attn_f32_kernel<64>), grid, blk, 0, st, a);
        else
            hipLaunchKernelGGL((attn_f32_kernel<128>), grid, blk, 0, st, a);
    } else if (a.decode) {
        const dim3 grid((a.total_wgs + 7) / 8 * 8), blk(64);
        if (D == 64)
            hipLaunchKernelGGL((attn_decode_kernel<64>), grid, blk, 0, st, a);
        else
            hipLaunchKernelGGL((attn_decode_kernel<128>), grid, blk, 0, st, a);
    } else {
        const dim3 grid((a.total_wgs + 7) / 8 * 8), blk(64 * ATT_WAVES);
        if (D == 64)
            hipLaunchKernelGGL((attn_bf16_kernel<64>), grid, blk, 0, st, a);
        else
            hipLaunchKernelGGL((attn_bf16_kernel<128>), grid, blk, 0, st, a);
    }
    return (int)hipGetLastError();
}

int en_launch_combine(const en_pool *pool, const EnAttnArgs &a, const EnMassArgs &m, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const int D = pool->d.head_dim;
    const int vec = pool->d.dtype == EN_F32 ? 4 : 8;      // elements in 16 bytes
    const int G = a.n_splits > 32 ? 16 : (a.n_splits > 8 ? 4 : 1);     // lanes that share a (row, chunk)
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
        else                                                                                          \
            hipLaunchKernelGGL((combine_kernel<T, DD, 16>), grid, blk, 0, st, a, m, n_comb);          \
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

int en_launch_ctx_append(const en_pool *pool, const EnCtxAppendArgs &a, void *stream)
{
    const int D = pool->d.head_dim;
    const dim3 grid(a.n, a.Hkv, a.B), blk(D / 2);
    hipStream_t st = (hipStream_t)stream;
    if (pool->d.dtype == EN_F32) {
        if (D == 64)
            hipLaunchKernelGGL((ctx_append_kernel<float, 64>), grid, blk, 0, st, a);
        else
            hipLaunchKernelGGL((ctx_append_kernel<float, 128>), grid, blk, 0, st, a);
    } else {
        if (D == 64)
            hipLaunchKernelGGL((ctx_append_kernel<bf16_t, 64>), grid, blk, 0, st, a);
        else
            hipLaunchKernelGGL((ctx_append_kernel<bf16_t, 128>), grid, blk, 0, st, a);
    }
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

int en_launch_tier_load(const EnTierLoadArgs &a, int max_tokens, void *stream)
{
    const int units = max_tokens * (a.row_bytes / 16);
    const dim3 grid((units + 1023) / 1024, 2 * a.Hkv, a.n), blk(256);
    hipLaunchKernelGGL(tier_load_kernel, grid, blk, 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

int en_launch_append_q8(const en_pool *pool, const EnAppendQ8Args &a, void *stream)
{
    const dim3 grid(a.n, a.Hkv, 2), blk(64);
    if (pool->d.head_dim == 64)
        hipLaunchKernelGGL((append_q8_kernel<64>), grid, blk, 0, (hipStream_t)stream, a);
    else
        hipLaunchKernelGGL((append_q8_kernel<128>), grid, blk, 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

int en_launch_append(const en_pool *pool, const EnAppendArgs &a, void *stream)
{
    (void)pool;
    const size_t total = (size_t)a.n * a.Hkv * a.row_chunks;
    const dim3 grid((unsigned)((total + 255) / 256), 2), blk(256);
    hipLaunchKernelGGL(append_kernel, grid, blk, 0, (hipStream_t)stream, a);
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
        if (a.n_splits == 1 || a.Nq < EN_MASS_FEW_ROWS)
            hipLaunchKernelGGL(mass_partial_kernel, grid, blk, 0, st, a);
        const dim3 grid2((a.B * (a.Smax + 1) + 3) / 4);
        hipLaunchKernelGGL(mass_final_kernel, grid2, blk, 0, st, a);
    }
    return (int)hipGetLastError();
}
