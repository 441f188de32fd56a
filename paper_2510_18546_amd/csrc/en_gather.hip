// Data movement kernels of libefficientnav.so.
//
//   gather_k / gather_vt   index-driven gather of the selected K/V blocks into
//                          one contiguous context per agent; keys receive the
//                          rotary encoding of their concatenated position
//                          (Section 3.2 of arXiv 2510.18546: select, then load
//                          each group's KV once per planning step); the same
//                          from a pool of 8-bit codes
//   ctx_append             a decode step's own K/V rows join the context
//   tier_load              blocks of the host store go to device slots
//   append / append_q8     new objects' K/V rows join their group's block
#include "en_device.h"

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
// A block takes 32 token rows of HPB consecutive KV heads, kv0 onwards: where a
// row comes from and its cosines and sines (two fp32 table rows, twice the bytes
// of a bf16 key row) are the same for every head, so they are fetched once for
// the HPB heads (64 agents x 16 K tokens, keys only: 1.14 ms with the table read
// per head, 0.73 ms without the table, which is what the value half takes).
// 256 threads, 32 rows per pass.
// ---------------------------------------------------------------------------
template <typename T, int D, bool COPY_V, int HPB, typename P>
__device__ __forceinline__ void gather_k_rows(const EnGatherArgs &a, int tok, int kv0, P bnd, P sel, int S)
{
    constexpr int E = D / 16;
    const int b = blockIdx.z;
    const int c = threadIdx.x % 8;
    const int Ltot = bnd[S + 1];
    const int Lpad = (Ltot + EN_KEY_TILE - 1) / EN_KEY_TILE * EN_KEY_TILE;
    if (tok >= Lpad)
        return;
    typedef T tvec __attribute__((ext_vector_type(E)));
    typedef float fvec __attribute__((ext_vector_type(E)));
    // the rows of head kv0; head kv0 + h is h * hstride elements further, keys and values alike
    const T *ksrc = context_src<T, D>(a, bnd, sel, S, (const T *)a.k_pool, (const T *)a.k_new, b, kv0, tok);
    const T *vsrc = nullptr;
    if constexpr (COPY_V)
        vsrc = context_src<T, D>(a, bnd, sel, S, (const T *)a.v_pool, (const T *)a.v_new, b, kv0, tok);
    const size_t hstride = tok >= bnd[S] ? (size_t)D : (size_t)a.C * D;      // new tokens [.., Hkv, D], pool [.., Hkv, C, D]
    tvec x1[HPB], x2[HPB];
    fvec cs = 0.f, sn = 0.f;
    if (ksrc) {
#pragma unroll
        for (int h = 0; h < HPB; ++h) {
            x1[h] = *reinterpret_cast<const tvec *>(ksrc + h * hstride + c * E);
            x2[h] = *reinterpret_cast<const tvec *>(ksrc + h * hstride + D / 2 + c * E);
        }
        cs = *reinterpret_cast<const fvec *>(a.cos_tab + (size_t)tok * (D / 2) + c * E);
        sn = *reinterpret_cast<const fvec *>(a.sin_tab + (size_t)tok * (D / 2) + c * E);
    }
#pragma unroll
    for (int h = 0; h < HPB; ++h) {
        T *dst = (T *)a.kc + (((size_t)b * a.Hkv + kv0 + h) * a.T + tok) * D;
        fvec y1 = 0.f, y2 = 0.f;
        if (ksrc) {
            const fvec f1 = __builtin_convertvector(x1[h], fvec), f2 = __builtin_convertvector(x2[h], fvec);
            y1 = f1 * cs - f2 * sn;
            y2 = f2 * cs + f1 * sn;
        }
        *reinterpret_cast<tvec *>(dst + c * E) = __builtin_convertvector(y1, tvec);
        *reinterpret_cast<tvec *>(dst + D / 2 + c * E) = __builtin_convertvector(y2, tvec);
    }
    if constexpr (COPY_V) {
#pragma unroll
        for (int h = 0; h < HPB; ++h) {
            T *vdst = (T *)a.vt + (((size_t)b * a.Hkv + kv0 + h) * a.T + tok) * D;
            tvec v1 = (T)0.f, v2 = (T)0.f;
            if (vsrc) {
                v1 = *reinterpret_cast<const tvec *>(vsrc + h * hstride + c * E);
                v2 = *reinterpret_cast<const tvec *>(vsrc + h * hstride + D / 2 + c * E);
            }
            *reinterpret_cast<tvec *>(vdst + c * E) = v1;
            *reinterpret_cast<tvec *>(vdst + D / 2 + c * E) = v2;
        }
    }
}

// The key rows of 64-token tile `tile` for the heads kv0 .. kv0 + HPB - 1, 32 rows at a time:
// the halves first .. last of the tile.
template <typename T, int D, bool COPY_V, int HPB>
__device__ __forceinline__ void gather_k_block(const EnGatherArgs &a, int tile, int first, int last, int kv0,
                                               int32_t *lbnd)
{
    const int b = blockIdx.z;
    const int S = a.nseg[b];
    const EnGatherTables t = stage_tables(a, b, lbnd);
#pragma unroll 1
    for (int half = first; half <= last; ++half) {
        const int tok = tile * EN_KEY_TILE + half * 32 + threadIdx.x / 8;
        if (t.staged)
            gather_k_rows<T, D, COPY_V, HPB>(a, tok, kv0, (const int32_t *)lbnd,
                                             (const int32_t *)lbnd + EN_GATHER_TAB_LDS, S);
        else
            gather_k_rows<T, D, COPY_V, HPB>(a, tok, kv0, t.bnd, t.sel, S);
    }
}

// ---------------------------------------------------------------------------
// gather_vt (bf16): values of a 64-token tile are staged in LDS and written
// transposed, vt[d][column], where token j sits at column j with bits 2 and 3
// exchanged. 256 threads; bx = number of the 64-token tile.
// ---------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ void gather_vt_block(const EnGatherArgs &a, int bx, int kvh, int32_t *lbnd)
{
    constexpr int STR = D + 2;                 // LDS row stride in elements
    __shared__ uint16_t tile[EN_KEY_TILE * STR];
    __shared__ const uint16_t *srcs[EN_KEY_TILE];
    const int b = blockIdx.z;
    const int t0 = bx * EN_KEY_TILE;
    const int S = a.nseg[b];
    const EnGatherTables t = stage_tables(a, b, lbnd);
    const int32_t *lsel = lbnd + EN_GATHER_TAB_LDS;
    const int Ltot = t.staged ? lbnd[S + 1] : t.bnd[S + 1];
    if (t0 >= Ltot)                            // the same for the whole block
        return;
    if (a.v_rows) {
        // the values stay where they are: the tile's 64 row addresses instead (padding rows: the row of zeros)
        char *zero_row = (char *)a.vt + en_v_rows_table_bytes(a.B, a.Hkv, a.T);
        if (threadIdx.x < EN_KEY_TILE) {
            const uint16_t *vp = (const uint16_t *)a.v_pool, *vn = (const uint16_t *)a.v_new;
            const uint16_t *src =
                t.staged ? context_src<uint16_t, D>(a, (const int32_t *)lbnd, lsel, S, vp, vn, b, kvh, t0 + threadIdx.x)
                         : context_src<uint16_t, D>(a, t.bnd, t.sel, S, vp, vn, b, kvh, t0 + threadIdx.x);
            unsigned long long *tab = (unsigned long long *)a.vt + ((size_t)b * a.Hkv + kvh) * (size_t)a.T + t0;
            tab[threadIdx.x] = (unsigned long long)(uintptr_t)(src ? (const void *)src : (const void *)zero_row);
        } else if (bx == 0 && kvh == 0 && b == 0 && threadIdx.x < EN_KEY_TILE + D * 2 / 16) {
            reinterpret_cast<uint4 *>(zero_row)[threadIdx.x - EN_KEY_TILE] = make_uint4(0, 0, 0, 0);
        }
        return;
    }
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

// One launch for the whole gather. Grid (64-token tiles, units, agents); the units, head group
// by head group: the key units (the tile's key rows of HPB heads, which also copy fp32 values),
// then, for bf16, HPB value units (one head's transposed tile each). Workgroups are dispatched
// tile by tile along one unit, then the next unit: each unit is a sequential stream through
// memory (with the units of one tile side by side instead, the 8K-context gather took 18.8 us
// against 13.5), and key and value units of several heads are in flight together: they load
// different parts of a compute unit (vector memory and ALU against LDS), and a launch that ran
// all key units before all value units took the sum of the two instead of little more than the
// larger.
// When the launch carries the plan's descriptor block in its arguments, the
// tables are read from the argument segment and the first workgroup stores the
// block to device memory for the kernels that follow on the stream.
// Key units per head group: with one head per unit a 64-token tile is two units of 32 rows
// (more, shorter workgroups: what a small gather wants), with several heads one unit of two passes.
__host__ __device__ constexpr int en_gather_key_units(int hpb)
{
    return hpb == 1 ? 2 : 1;
}

// Queries prepared for the attention kernel (rows i of agent b, every head): rotated at L_c + i,
// scaled for the log2-domain softmax, rounded to bf16 once, exactly what a workgroup of the
// attention kernel would otherwise do for its own rows, once per KV split. The rows of an agent are
// dealt out over the gridDim.x workgroups of this unit; D/8 threads share a row, each takes four
// rotary pairs (k .. k+3, k + D/2 ..).
template <int D>
__device__ __forceinline__ void prepare_queries(const EnGatherArgs &a, int part, int n_parts, int b)
{
    constexpr int TPR = D / 8;                     // threads per row
    const int S = a.nseg[b];
    const int Lc = a.bnd[(size_t)b * (a.Smax + 2) + S];
    const int rows = a.Nq * a.Hq;
    const int per = (rows + n_parts - 1) / n_parts;
    const int r1 = min(rows, (part + 1) * per);
    const int t = threadIdx.x % TPR;
    for (int row = part * per + threadIdx.x / TPR; row < r1; row += 256 / TPR) {
        const int i = row / a.Hq;
        const size_t base = ((size_t)b * rows + row) * D;
        const bf16_t *src = (const bf16_t *)a.q + base;
        const bf16x4 x1 = *reinterpret_cast<const bf16x4 *>(src + 4 * t);
        const bf16x4 x2 = *reinterpret_cast<const bf16x4 *>(src + D / 2 + 4 * t);
        const size_t trow = (size_t)(Lc + i) * (D / 2) + 4 * t;
        const f32x4 c = *reinterpret_cast<const f32x4 *>(a.cos_tab + trow);
        const f32x4 sn = *reinterpret_cast<const f32x4 *>(a.sin_tab + trow);
        bf16x4 y1, y2;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float r1f, r2f;
            rope_scale_pair((float)x1[e], (float)x2[e], c[e], sn[e], a.scale_log2e, r1f, r2f);
            y1[e] = (bf16_t)r1f;
            y2[e] = (bf16_t)r2f;
        }
        bf16_t *dst = (bf16_t *)a.q_prep + base;
        *reinterpret_cast<bf16x4 *>(dst + 4 * t) = y1;
        *reinterpret_cast<bf16x4 *>(dst + D / 2 + 4 * t) = y2;
    }
}

template <typename T, int D, int HPB>
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
        {
            for (int i = threadIdx.x; i < g.n_inline; i += 256)
                g.desc_out[i] = img[i];
            for (int i = threadIdx.x; i < g.n_zero; i += 256)
                g.desc_out[g.n_inline + i] = 0;
        }
    }
    __shared__ int32_t lbnd[2 * EN_GATHER_TAB_LDS];       // bucket bounds, then selected groups
    const int tile = blockIdx.x;
    constexpr int KU = en_gather_key_units(HPB);
    constexpr int PER = KU + (sizeof(T) == 2 ? HPB : 0);      // units per head group
    int unit = blockIdx.y;
    if constexpr (sizeof(T) == 2) {
        // n_q_units more units along y, in front of the key and value units (dispatched first, so that
        // their short chains of loads run beside the streams and not behind them): the queries to prepare
        if (a.q) {
            if (unit < a.n_q_units) {
                prepare_queries<D>(a, unit * gridDim.x + tile, a.n_q_units * gridDim.x, blockIdx.z);
                return;
            }
            unit -= a.n_q_units;
        }
    }
    const int hg = unit / PER, r = unit % PER;
    if (r < KU)
        gather_k_block<T, D, sizeof(T) == 4, HPB>(a, tile, KU == 2 ? r : 0, KU == 2 ? r : 1, hg * HPB, lbnd);
    else if constexpr (sizeof(T) == 2)
        gather_vt_block<D>(a, tile, hg * HPB + r - KU, lbnd);
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
__device__ __forceinline__ void gather_q8_k_rows(const EnGatherArgs &a, const EnGatherTables &tabs, int tok, int kvh,
                                                 int32_t *lds)
{
    constexpr int E = D / 16;
    const int b = blockIdx.z;
    const int c = threadIdx.x % 8;
    const int S = a.nseg[b];
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
__device__ __forceinline__ void gather_q8_k_block(const EnGatherArgs &a, int tile, int kvh, int32_t *lds)
{
    const EnGatherTables tabs = stage_tables(a, blockIdx.z, lds);
#pragma unroll 1
    for (int half = 0; half < 2; ++half)
        gather_q8_k_rows<D>(a, tabs, tile * EN_KEY_TILE + half * 32 + threadIdx.x / 8, kvh, lds);
}

template <int D>
__device__ __forceinline__ void gather_q8_vt_block(const EnGatherArgs &a, int bx, int kvh, int32_t *lds)
{
    constexpr int STR = D + 2;                 // LDS row stride in elements
    __shared__ uint16_t tile[EN_KEY_TILE * STR];
    __shared__ size_t rows[EN_KEY_TILE];
    __shared__ int kinds[EN_KEY_TILE];
    const int b = blockIdx.z;
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
        {
            for (int i = threadIdx.x; i < g.n_inline; i += 256)
                g.desc_out[i] = img[i];
            for (int i = threadIdx.x; i < g.n_zero; i += 256)
                g.desc_out[g.n_inline + i] = 0;
        }
    }
    __shared__ int32_t ltab[2 * EN_GATHER_TAB_LDS];       // bucket bounds, then selected groups
    // the grid of gather_kernel with one head per key unit
    int unit = blockIdx.y;
    if (a.q) {
        if (unit < a.n_q_units) {      // the units in front: queries to prepare
            prepare_queries<D>(a, unit * gridDim.x + blockIdx.x, a.n_q_units * gridDim.x, blockIdx.z);
            return;
        }
        unit -= a.n_q_units;
    }
    const int tile = blockIdx.x, kvh = unit / 2;
    if (unit % 2 == 0)
        gather_q8_k_block<D>(a, tile, kvh, ltab);
    else
        gather_q8_vt_block<D>(a, tile, kvh, ltab);
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
// Heads per key unit: as many (8, 4, 2 that divide Hkv) as still leave 32 workgroups per compute unit.
static int gather_heads_per_unit(const en_pool *pool, const EnGatherArgs &a, int n_tiles, bool with_value_units)
{
    for (int hpb = 8; hpb > 1; hpb /= 2) {
        const long units = (long)(a.Hkv / hpb) * (en_gather_key_units(hpb) + (with_value_units ? hpb : 0));
        if (a.Hkv % hpb == 0 && units * n_tiles * a.B >= 32L * pool->n_cu)
            return hpb;
    }
    return 1;
}

template <typename T, int D>
static void launch_gather_kernel(int hpb, dim3 grid, hipStream_t st, const EnGatherLaunch &g)
{
    const dim3 blk(256);
    if (hpb == 8)
        hipLaunchKernelGGL((gather_kernel<T, D, 8>), grid, blk, 0, st, g);
    else if (hpb == 4)
        hipLaunchKernelGGL((gather_kernel<T, D, 4>), grid, blk, 0, st, g);
    else if (hpb == 2)
        hipLaunchKernelGGL((gather_kernel<T, D, 2>), grid, blk, 0, st, g);
    else
        hipLaunchKernelGGL((gather_kernel<T, D, 1>), grid, blk, 0, st, g);
}

int en_launch_gather(const en_pool *pool, EnGatherLaunch &g, int max_ctx_len, void *stream)
{
    const EnGatherArgs &a = g.a;
    hipStream_t st = (hipStream_t)stream;
    const int n_tiles = (max_ctx_len + EN_KEY_TILE - 1) / EN_KEY_TILE;
    const int D = pool->d.head_dim;
    if (pool->d.dtype == EN_I8) {
        const dim3 grid(n_tiles, 2 * a.Hkv + (a.q ? a.n_q_units : 0), a.B), blk(256);
        if (D == 64)
            hipLaunchKernelGGL((gather_q8_kernel<64>), grid, blk, 0, st, g);
        else
            hipLaunchKernelGGL((gather_q8_kernel<128>), grid, blk, 0, st, g);
        return (int)hipGetLastError();
    }
    const bool bf16 = pool->d.dtype != EN_F32;
    const int hpb = gather_heads_per_unit(pool, a, n_tiles, bf16);
    // (n_q_units more units along y when the launch also prepares the queries: bf16 contexts only)
    const dim3 grid(n_tiles, (a.Hkv / hpb) * (en_gather_key_units(hpb) + (bf16 ? hpb : 0)) + (bf16 && a.q ? a.n_q_units : 0), a.B);
    if (!bf16) {
        if (D == 64)
            launch_gather_kernel<float, 64>(hpb, grid, st, g);
        else
            launch_gather_kernel<float, 128>(hpb, grid, st, g);
    } else {
        if (D == 64)
            launch_gather_kernel<bf16_t, 64>(hpb, grid, st, g);
        else
            launch_gather_kernel<bf16_t, 128>(hpb, grid, st, g);
    }
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
