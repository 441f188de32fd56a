// attn_bf16: softmax(QK^T/sqrt(D))V of the new tokens over the gathered context
// (Appendix A of arXiv 2510.18546) on the bf16 matrix cores, with an online
// softmax and the per-segment partial sums of Section 3.3.
#include "en_device.h"

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

constexpr int ATT_WAVES = EN_WAVES;

// QPREP: the queries arrive prepared (rotated at L_c + i, scaled, bf16: the gather launch did it
// once), else the wave prepares its own 32 from the caller's unrotated ones.
// VPOOL: the values were not gathered. a.vt holds, per (agent, KV head, context row), the address of
// that row's D values where they are (a block of the pool, the new tokens, a row of zeros for the
// padding of the last tile). The loader fetches the 64 rows of a tile from there, so a V tile sits
// in LDS row-major, [64 keys][D], and the operand reads transpose it (ds_read_b64_tr_b16). Inside
// a tile the 16-byte chunks of a row are rotated (by four times the row number with 256-byte rows,
// by four times half the row number with 128-byte rows, two of which share a line of banks): the
// 32 lanes of one transposing read then touch 4 rows x 64 bytes on distinct banks.
template <int D, bool QPREP, bool VPOOL>
__global__ __launch_bounds__(64 * ATT_WAVES) void attn_bf16_kernel(EnAttnArgs a)
{
    constexpr int VCPR = D / 8;                  // VPOOL: 16-byte chunks per value row
    constexpr int VRPB = 1024 / (2 * D);         // VPOOL: value rows per loader block
    // VPOOL: rotation of row `row`'s chunks inside a tile (in chunks, taken mod VCPR)
    auto vrot = [](int row) { return D == 128 ? 4 * row : 4 * (row >> 1); };
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
    if (logical == 0 && a.red_zero)               // start of the reduced masses that later launches add up
        for (int i = threadIdx.x; i < a.n_red_zero; i += 64 * ATT_WAVES)
            a.red_zero[i] = 0ull;
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
    const int t_begin = (int)split_first_tile(sp, ntiles, a.n_splits);
    int t_end = (int)split_first_tile(sp + 1, ntiles, a.n_splits);
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
        voff[j] = VPOOL ? 0u : (uint32_t)((size_t)d * a.T * 2 + ((pos - d / 2) & 7) * 16);
    }
    // VPOOL: loader block blk = wave + 8 j of a tile is rows VRPB blk .. VRPB (blk + 1) - 1, lane L of it
    // position L % VCPR of row VRPB blk + L / VCPR, which holds chunk (L % VCPR - rotation) mod VCPR
    // of that row (the rotation of a row does not depend on blk: VRPB blk rows are whole lines of banks).
    const char *vtab = (const char *)a.vt + ((size_t)b * a.Hkv + kvh) * (size_t)a.T * 8;
    const uint32_t vtab_lane = (uint32_t)(VRPB * wave + lane / VCPR) * 8;      // this lane's first row of a tile
    const uint32_t vchunk = (uint32_t)((lane % VCPR - vrot(lane / VCPR)) & (VCPR - 1)) * 16;
    // Addresses of this lane's 16 bytes of the V tile to load next (vrow) and of the one after
    // (vnext, on its way from the table). The table is read with ordinary loads, which the compiler
    // waits for where it first uses the result: vrow_take is therefore called where everything in
    // flight has just been waited for anyway (right after a tile's barrier), one whole tile after
    // the request. (Between loader blocks, which the compiler does not see, it could only wait for
    // all of them.)
    unsigned long long vrow[VJ], vnext[VJ];
#pragma unroll
    for (int j = 0; j < VJ; ++j)
        vrow[j] = vnext[j] = 0;
    auto vrow_request = [&](int tile) {
        if constexpr (VPOOL) {
            const char *p = vtab + (size_t)min(tile, t_end - 1) * (KT * 8) + vtab_lane;
#pragma unroll
            for (int j = 0; j < VJ; ++j)
                vnext[j] = *reinterpret_cast<const unsigned long long *>(p + j * (VRPB * ATT_WAVES) * 8);
        }
    };
    auto vrow_take = [&]() {
        if constexpr (VPOOL) {
#pragma unroll
            for (int j = 0; j < VJ; ++j) {
                vrow[j] = vnext[j] | vchunk;
                asm volatile("" : "+v"(vrow[j]));      // here, not later
            }
        }
    };
    // Loader job of the current phase: one tile of K or of V^T, issued block by
    // block between the matrix instructions. A tile index past the end is
    // clamped: the last tile is fetched once more, into a stage nobody reads.
    uint32_t job_goff = 0;
    auto job_k = [&](int tile) { job_goff = (uint32_t)min(tile, t_end - 1) * KBYTES; };
    auto job_v = [&](int tile) {
        if constexpr (!VPOOL)
            job_goff = (uint32_t)min(tile, t_end - 1) * (KT * 2);
    };
    auto dma_k = [&](auto j_tag, auto stage_tag) {
        constexpr int j = decltype(j_tag)::value, stage = decltype(stage_tag)::value;
        if constexpr (j < KJ)
            dma16_imm<stage * KBYTES + j * ATT_WAVES * 1024>(kg, koff[j] + job_goff, lds_w);
    };
    auto dma_v = [&](auto j_tag, auto stage_tag) {
        constexpr int j = decltype(j_tag)::value, stage = decltype(stage_tag)::value;
        if constexpr (j < VJ) {
            if constexpr (VPOOL)
                dma16_addr_imm<VBASE + stage * VBYTES + j * ATT_WAVES * 1024>(vrow[j], lds_w);
            else
                dma16_imm<VBASE + stage * VBYTES + j * ATT_WAVES * 1024>(vg, voff[j] + job_goff, lds_w);
        }
    };

    // ---- first loads, issued before the queries are prepared so that both are in
    // flight together. The loop is unrolled over the three stages; the nt % 3
    // tiles that do not fill a round come first, so the first tile's stage s0
    // is chosen such that the last tile always sits in stage 2. ----
    const int rem = nt % NST;
    const int s0 = (NST - rem) % NST;
    const int s1 = (s0 + 1) % NST, s2 = (s0 + 2) % NST;
    if (nt > 0) {
        vrow_request(t_begin);       // (VPOOL) the first V tile waits for these: asked for first, loaded first
        char *vz = smem + VBASE + s2 * VBYTES;     // the first product reads a zero V^T stage
        for (int i = tid * 16; i < VBYTES; i += 64 * ATT_WAVES * 16)
            *reinterpret_cast<uint4 *>(vz + i) = make_uint4(0, 0, 0, 0);
        if constexpr (VPOOL) {
            vrow_take();
#pragma unroll
            for (int j = 0; j < VJ; ++j)
                dma16_addr(vrow[j], lds_w + VBASE + s0 * VBYTES + j * ATT_WAVES * 1024);
        }
        job_k(t_begin);
#pragma unroll
        for (int j = 0; j < KJ; ++j)
            dma16(kg, koff[j] + job_goff, lds_w + s0 * KBYTES + j * ATT_WAVES * 1024);
        job_k(t_begin + 1);
#pragma unroll
        for (int j = 0; j < KJ; ++j)
            dma16(kg, koff[j] + job_goff, lds_w + s1 * KBYTES + j * ATT_WAVES * 1024);
        job_v(t_begin);
        if constexpr (VPOOL) {
            vrow_request(t_begin + 1);
        } else {
#pragma unroll
            for (int j = 0; j < VJ; ++j)
                dma16(vg, voff[j] + job_goff, lds_w + VBASE + s0 * VBYTES + j * ATT_WAVES * 1024);
        }
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
    // VPOOL: the operand of a product is V^T[32 d + col][keys k0 + 4 half + {0..3}, k0 + 8 + 4 half + {0..3}]
    // (k0 = 32 h + 16 kk: the keys whose probabilities the lane holds), two transposing reads. In
    // one read the 16 lanes of a group point at 4 key rows x 16 values: lane j at row j / 4, values
    // 4 (j % 4) .., and lane i receives value i of the four rows.
    uint32_t vtaddr[NDB];
#pragma unroll
    for (int d = 0; d < NDB; ++d) {
        const int j = lane % 16, grp = lane / 16;
        const int row = 4 * half + j / 4;
        const int chunk = 4 * d + 2 * (grp % 2) + (j % 4) / 2;
        vtaddr[d] = (uint32_t)(VBASE + row * ROWB + ((chunk + vrot(row)) & (VCPR - 1)) * 16 + 8 * (j % 2));
    }
    // the operand of O^T block d from the keys k0 .. k0 + 15 of the V stage at byte offset stage_off
    auto v_operand = [&](int d, int stage_off, int k0) -> bf16x8 {
        typedef short s16x4 __attribute__((ext_vector_type(4)));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        typedef __attribute__((address_space(3))) s16x4 *lds_s16x4;
        char *p = smem + vtaddr[d] + stage_off + k0 * ROWB;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)p);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(p + 8 * ROWB));
        const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, both);
    };

    // ---- Q: prepared queries are loaded as they are; else load, rotate at L_c + i, scale, round to bf16 ----
    bf16x8 qf[NKS];
    if constexpr (QPREP) {
        const bf16_t *qp = (const bf16_t *)a.q + (((size_t)b * a.Nq + i_row) * a.Hq + hq) * D + 8 * half;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            qf[ks] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            if (row_valid)
                qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + 16 * ks);
        }
    } else
    {
        // The rotary rows (cosines and sines of position L_c + i, D/2 floats each) are the same for
        // the waves that share a query block, and they are twice the bytes of the queries
        // themselves: loaded per wave they are two thirds of what the compute unit's vector
        // memory path moves before the first tile (3 us of the launch). When the workgroup's
        // waves share at most two query blocks (Hq / Hkv >= 4, mostly), their 64 rows are
        // fetched once, into the K stage and the V^T stage that no tile load has touched yet
        // (64 rows of D/2 floats are exactly one stage), the 16-byte chunks of a row rotated by
        // the row number like those of a K tile, and every wave reads its rows from there.
        constexpr int TCPR = D / 8;                  // 16-byte chunks per table row
        const int qb_first = (ptile * ATT_WAVES) / r;
        const int qb_last = min((ptile * ATT_WAVES + ATT_WAVES - 1) / r, nqb - 1);
        const bool shared_tab = nt > 0 && qb_last - qb_first <= 1;
        // Order of the loads: the shared rotary rows first, then the wave's queries, so that the
        // rows go to LDS (and the workgroup meets at the barrier) while the queries are on their way.
        constexpr int TIT = TCPR / ATT_WAVES;        // chunks of either table per thread
        static_assert(TCPR % ATT_WAVES == 0, "rotary rows per thread");
        char *ctab = smem + s2 * KBYTES, *stab = smem + VBASE + s1 * VBYTES;
        f32x4 tc[TIT], tsn[TIT];
        if (shared_tab) {
            const int pos0 = Lc + qb_first * 32;
#pragma unroll
            for (int it = 0; it < TIT; ++it) {
                const int q = tid + it * 64 * ATT_WAVES;
                const int row = q / TCPR, c = q % TCPR;
                const size_t src = (size_t)min(pos0 + row, Ltot - 1) * (D / 2) + 4 * c;
                tc[it] = *reinterpret_cast<const f32x4 *>(a.cos_tab + src);
                tsn[it] = *reinterpret_cast<const f32x4 *>(a.sin_tab + src);
            }
        }
        bf16x8 qraw[NKS];
        const bf16_t *qp = (const bf16_t *)a.q + (((size_t)b * a.Nq + i_row) * a.Hq + hq) * D + 8 * half;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            qraw[ks] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            if (row_valid)
                qraw[ks] = *reinterpret_cast<const bf16x8 *>(qp + 16 * ks);
        }
        float cs[NKS / 2][8], sn[NKS / 2][8];
        if (shared_tab) {
#pragma unroll
            for (int it = 0; it < TIT; ++it) {
                const int q = tid + it * 64 * ATT_WAVES;
                const int row = q / TCPR, c = q % TCPR;
                const int dst = row * (2 * D) + ((c + row) % TCPR) * 16;
                *reinterpret_cast<f32x4 *>(ctab + dst) = tc[it];
                *reinterpret_cast<f32x4 *>(stab + dst) = tsn[it];
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);          // lgkmcnt(0): this wave's rows are in LDS
            __builtin_amdgcn_s_barrier();
            lds_data_ready();
            const int row = (wave_valid ? qb - qb_first : 0) * 32 + col;
#pragma unroll
            for (int ks = 0; ks < NKS / 2; ++ks)
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const int off = row * (2 * D) + ((4 * ks + 2 * half + jj + row) % TCPR) * 16;
                    const f32x4 c4 = *reinterpret_cast<const f32x4 *>(ctab + off);
                    const f32x4 s4 = *reinterpret_cast<const f32x4 *>(stab + off);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        cs[ks][4 * jj + e] = c4[e];
                        sn[ks][4 * jj + e] = s4[e];
                    }
                }
        } else {
            const int pos = row_valid ? Lc + i_row : 0;
            const float *ct = a.cos_tab + (size_t)pos * (D / 2) + 8 * half;
            const float *st = a.sin_tab + (size_t)pos * (D / 2) + 8 * half;
#pragma unroll
            for (int ks = 0; ks < NKS / 2; ++ks)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    cs[ks][j] = ct[16 * ks + j];
                    sn[ks][j] = st[16 * ks + j];
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
                rope_scale_pair(x1, x2, cs[ks][j], sn[ks][j], a.scale_log2e, qx[ks][j], qx[ks + NKS / 2][j]);
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
            if constexpr (VPOOL) {
                return v_operand(d, ((st + NST - 1 + par) % NST) * VBYTES, 32 * (par ^ 1) + 16 * kk);
            } else {
                constexpr int off = ((st + NST - 1 + par) % NST) * VBYTES + d * 32 * VROWB;
                return *reinterpret_cast<const bf16x8 *>(smem + vaddr[par ^ 1][kk] + off);
            }
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
        vrow_take();                  // (VPOOL) rows of V tile + 1, asked for a tile ago
        vrow_request(tile + 2);
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
                if constexpr (VPOOL)
                    fr[k] = v_operand(d, s2 * VBYTES, 32 + 16 * kk);
                else
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
                bf16x8 av;
                if constexpr (VPOOL)
                    av = v_operand(d, 2 * VBYTES, 32 + 16 * kk);
                else
                    av = *reinterpret_cast<const bf16x8 *>(smem + vaddr[1][kk] + 2 * VBYTES + d * 32 * VROWB);
                o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, pbuf[1][kk], o[d], 0, 0, 0);
            }
        // loads of the clamped tiles may still be in flight
        wait_all_memory();
    }
    // every wave is done with the tiles: their stages become the waves' staging areas for the
    // output rows (see the epilogue)
    __builtin_amdgcn_s_barrier();

    if (!wave_valid && !a.red_direct)
        return;
    float inv = 0.f;
    // (one split, reduced masses from this kernel: see below) the wave's pairs of 2 UB buckets
    constexpr int UB = 8;
    f32x2 pairs[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u)
        pairs[u] = f32x2{0.f, EN_NEG_INF};
    const bool red_direct = a.red_direct && seg_base;        // the same for the whole workgroup
    auto load_pairs = [&](int s0) {
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int sa = s0 + 2 * u;                         // wave-uniform
            const int nb = a.Smax + 1;
            const int b0 = bound_at(min(sa, nb)), b1 = bound_at(min(sa + 1, nb)), b2 = bound_at(min(sa + 2, nb));
            const bool live = half == 0 ? (sa <= S && b1 > b0) : (sa + 1 <= S && b2 > b1);
            pairs[u] = f32x2{0.f, EN_NEG_INF};
            if (live && row_valid)
                pairs[u] = *reinterpret_cast<const f32x2 *>(seg_base + (size_t)((sa + half) * a.Nq) * 2);
        }
    };
    if (wave_valid) {
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
    // One split: the output row. Several: this split's own softmax output
    // (normalised by its own sum), merged by the combine kernel.
    // A lane holds its row in pieces of 8 bytes, 32 rows per store instruction: written as they
    // are, a wave's 8 KB go out as 512 pieces of 16 bytes (2 - 3.5 us at the end of the launch,
    // when every wave does it at once). Staged through LDS, each store instruction writes whole
    // rows: 64 lanes x 16 bytes = four rows of 256 bytes.
    inv = (row_valid && l_tot > 0.f) ? 1.f / l_tot : 0.f;
    constexpr int OSTR = 2 * D + 16;             // bytes per staged row (padded: bank spread, 16-byte aligned)
    constexpr int OCPR = D / 8;                  // 16-byte chunks per row
    static_assert(ATT_WAVES * 32 * OSTR <= NST * (KBYTES + VBYTES), "staging areas must fit the tile stages");
    char *stage_o = smem + wave * (32 * OSTR);
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                v[e] = (bf16_t)(o[d][4 * g + e] * inv);
            *reinterpret_cast<bf16x4 *>(stage_o + col * OSTR + (32 * d + 8 * g + 4 * half) * 2) = v;
        }
    // the area is this wave's own: its writes only have to be complete (the compiler waits for them)
    if (red_direct) {
        // the pairs are read back here, behind the wave's last stores of them (waited for) and
        // ahead of the output rows' stores, so that their way from memory overlaps those
        wait_all_memory();
        load_pairs(0);
    }
#pragma unroll
    for (int k = 0; k < 32 * OCPR / 64; ++k) {
        const int idx = k * 64 + lane;
        const int rr = idx / OCPR, c = idx % OCPR;
        const int i = i_lo + rr;
        if (i < a.Nq) {
            const uint4 val = *reinterpret_cast<const uint4 *>(stage_o + rr * OSTR + c * 16);
            bf16_t *op = (a.n_splits == 1)
                             ? (bf16_t *)a.out + (((size_t)b * a.Nq + i) * a.Hq + hq) * D
                             : (bf16_t *)a.ws_opart + ((size_t)sp * a.B * a.Hq * a.Nq + row_hq * a.Nq + i) * D;
            *reinterpret_cast<uint4 *>(op + c * 8) = val;
        }
    }

    }      // wave_valid

    // ---- one split: the reduced masses [B, S+1] from here, without a further launch. The wave's
    // (sum, reference) pairs of every bucket are in the scratch (its own stores: waited for, then
    // read back, several buckets per batch of loads); with the rows' final references and sums in
    // registers a bucket's masses of the wave's 32 rows are summed (the two halves of the wave take
    // a bucket each), the workgroup's eight sums per bucket meet in LDS, and one thread per bucket
    // adds the workgroup's sum, as a fixed-point integer, to the plan's accumulator of
    // (agent, bucket): one arrival per workgroup (arrivals at one address take about 0.1 us each). ----
    if (red_direct) {
        constexpr int OAREA = ATT_WAVES * 32 * (2 * D + 16);      // the staging areas of the output rows
        float *red_w = reinterpret_cast<float *>(smem + OAREA);   // [waves][Smax + 1]
        static_assert(OAREA + ATT_WAVES * EN_RED_DIRECT_MAX_BUCKETS * 4 <= NST * (KBYTES + VBYTES), "sums of the buckets beside the staging areas");
        const int nb = a.Smax + 1;
        for (int s0 = 0; s0 < nb; s0 += 2 * UB) {
            if (s0 > 0 && wave_valid)
                load_pairs(s0);
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int s = s0 + 2 * u + half;
                float v = pairs[u][1] != EN_NEG_INF ? pairs[u][0] * fast_exp2(pairs[u][1] - m_ref) * inv : 0.f;
                v = half_sum(v);
                if (col == 0 && s < nb)
                    red_w[wave * nb + s] = v;
            }
        }
        __syncthreads();
        for (int s = tid; s < nb; s += 64 * ATT_WAVES) {
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < ATT_WAVES; ++w)
                v += red_w[w * nb + s];
            const size_t idx = (size_t)b * nb + s;
            const long long q = __float2ll_rn(ldexpf(v, a.red_shift));
            const unsigned long long add = ((unsigned long long)q << 10) + 1ull;
            const unsigned long long now = atomicAdd(a.red_direct + idx, add) + add;
            if ((int)(now & 1023ull) == a.red_target) {
                a.red_direct_out[idx] =
                    ldexpf((float)((long long)(now - (unsigned long long)a.red_target) >> 10), -a.red_shift);
                a.red_direct[idx] = 0ull;           // nobody arrives after the last: ready for the next call
            }
        }
    }
}

// ---------------------------------------------------------------------------
// launcher
// ---------------------------------------------------------------------------
int en_launch_attention_prefill(const en_pool *pool, const EnAttnArgs &a, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((a.total_wgs + 7) / 8 * 8), blk(64 * ATT_WAVES);
    if (pool->d.head_dim == 64) {
        if (a.v_rows) {
            if (a.q_prepared)
                hipLaunchKernelGGL((attn_bf16_kernel<64, true, true>), grid, blk, 0, st, a);
            else
                hipLaunchKernelGGL((attn_bf16_kernel<64, false, true>), grid, blk, 0, st, a);
        } else if (a.q_prepared)
            hipLaunchKernelGGL((attn_bf16_kernel<64, true, false>), grid, blk, 0, st, a);
        else
            hipLaunchKernelGGL((attn_bf16_kernel<64, false, false>), grid, blk, 0, st, a);
    } else if (a.v_rows) {
        if (a.q_prepared)
            hipLaunchKernelGGL((attn_bf16_kernel<128, true, true>), grid, blk, 0, st, a);
        else
            hipLaunchKernelGGL((attn_bf16_kernel<128, false, true>), grid, blk, 0, st, a);
    } else {
        if (a.q_prepared)
            hipLaunchKernelGGL((attn_bf16_kernel<128, true, false>), grid, blk, 0, st, a);
        else
            hipLaunchKernelGGL((attn_bf16_kernel<128, false, false>), grid, blk, 0, st, a);
    }
    return (int)hipGetLastError();
}
