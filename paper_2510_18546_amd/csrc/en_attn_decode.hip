// attn_decode: the same attention for steps of few query rows (the decode phase
// of a planning step, Section 3.2), bound by reading the context once; and
// attn_f32, the fp32 vector path of small configurations.
#include "en_device.h"

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
template <int D, int SUB>
__global__ __launch_bounds__(64 * SUB) void attn_decode_kernel(EnAttnArgs a)
{
    // SUB = 2: two waves share the unit's tiles (each issues half of a tile's loads and takes one
    // of its two 32-key blocks, with softmax state, partial output and segment sums of its own,
    // stored at partial-result index sp * 2 + wave). For steps that leave compute units idle: a
    // wave alone on its SIMD takes about 2 us per tile, and the tiles' LDS stages allow two
    // workgroups per compute unit, so this puts all four SIMDs to work.
    static_assert(SUB == 1 || SUB == 2, "one or two waves per unit");
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

    const int wave = SUB == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const int lane = threadIdx.x % 64;
    const int spw = sp * SUB + wave;             // index of this wave's partial results
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
    const int split_key_begin = (int)split_first_tile(sp, ntiles64, a.n_splits) * EN_KEY_TILE;
    const int split_key_end = min((int)split_first_tile(sp + 1, ntiles64, a.n_splits) * EN_KEY_TILE, Ltot);
    const int t_begin = split_key_begin, t_end = split_key_end;
    const int lt_begin = split_key_begin / LB;           // load tiles; splits begin on them
    const int lt_end = (split_key_end + LB - 1) / LB;    // context rows are zero up to a multiple of 64

    // ---- loader set-up ----
    const char *kg = (const char *)a.kc + ((size_t)b * a.Hkv + kvh) * (size_t)a.T * ROWB;
    const char *vg = (const char *)a.vt + ((size_t)b * a.Hkv + kvh) * (size_t)D * a.T * 2;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;
    // the waves take the loader blocks in turn; a wave that would run out repeats the last one
    constexpr int NKW = (NBK + SUB - 1) / SUB, NVW = (NBV + SUB - 1) / SUB;
    uint32_t koff[NKW], voff[NVW], kblk[NKW], vblk[NVW];
#pragma unroll
    for (int jj = 0; jj < NKW; ++jj) {
        const int j = min(wave + SUB * jj, NBK - 1);
        const int q = j * 64 + lane;
        const int row = q / KCPR, c = q % KCPR;
        koff[jj] = (uint32_t)(row * ROWB + (c < KCPR - 1 ? c : 0) * 16);      // the pad chunk re-reads chunk 0
        kblk[jj] = (uint32_t)j * 1024;
    }
#pragma unroll
    for (int jj = 0; jj < NVW; ++jj) {
        const int j = min(wave + SUB * jj, NBV - 1);
        const int q = j * 64 + lane;
        const int d = q / VCPR, c = q % VCPR;
        voff[jj] = (uint32_t)((size_t)d * a.T * 2 + (c < VCPR - 1 ? c : 0) * 16);
        vblk[jj] = (uint32_t)(KBYTES + j * 1024);
    }
    auto issue = [&](int tile, int stage) {
        const char *kt = kg + (size_t)tile * (LB * ROWB);
        const char *vtile = vg + (size_t)tile * (LB * 2);
        const uint32_t dst = lds0 + stage * STAGE;
#pragma unroll
        for (int jj = 0; jj < NKW; ++jj)
            dma16(kt, koff[jj], dst + kblk[jj]);
#pragma unroll
        for (int jj = 0; jj < NVW; ++jj)
            dma16(vtile, voff[jj], dst + vblk[jj]);
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
    const bool appends = owns_new && wave == 0;          // one wave writes, all wait for it
    if (appends)
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
        if (appends) {
            int t = first_new - Lc;
            app_store(t);
            for (++t; t < a.Nq && Lc + t < split_key_end; ++t) {
                app_load(t);
                app_store(t);
            }
        }
        if (owns_new && !first_tile_old) {
            if (appends)
                wait_all_memory();                   // stores included
            if (SUB > 1)
                __syncthreads();
            issue(lt_begin, 0);
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
                          ? a.ws_seg + (((size_t)spw * a.B * a.Hq + row_hq) * (a.Smax + 1)) * a.Nq * 2
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
    if (owns_new && first_tile_old) {
        if (appends)
            wait_all_memory();
        if (SUB > 1)
            __syncthreads();
    }
    constexpr int NUW = NU / SUB;                // 32-key blocks of a tile per wave
    const int u0 = wave * NUW;                   // this wave's first
    int stage = 0;                               // of tile lt
    for (int lt = lt_begin; lt < lt_end; ++lt) {
        const char *stg = smem + stage * STAGE;
        // every LDS read of the previous tile has returned (its matrix
        // instructions consumed them), so its stage may be overwritten
        __builtin_amdgcn_s_waitcnt(0xc07f);                  // lgkmcnt(0)
        if (SUB == 1) {
            constexpr int PER_TILE = NBK + NBV;
            if (lt + 1 < lt_end) {
                issue(lt + 1, stage ^ 1);
                // this tile's loads have landed when at most the next tile's are outstanding
                __builtin_amdgcn_s_waitcnt((PER_TILE & 15) | ((PER_TILE >> 4) << 14) | 0x0f70);
            } else {
                __builtin_amdgcn_s_waitcnt(0x0f70);              // vmcnt(0)
            }
        } else {
            // this wave's share of the tile has landed, and past the barrier the other's too, and
            // nobody reads the previous tile any more: the next one may overwrite it. It was a
            // whole tile's arithmetic ahead of its wait, as with one wave.
            __builtin_amdgcn_s_waitcnt(0x0f70);                  // vmcnt(0)
            __builtin_amdgcn_s_barrier();
            if (lt + 1 < lt_end)
                issue(lt + 1, stage ^ 1);
        }
        lds_data_ready();
        const int kb = lt * LB;
        const int kbw = kb + KB * u0;                // this wave's keys of the tile: [kbw, kbw + KB * NUW)
        // ---- S^T = K Q^T - m_ref, the two 32-key blocks as independent chains ----
        f32x16 sv[NUW];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
            for (int u = 0; u < NUW; ++u) {
                const bf16x8 fr = *reinterpret_cast<const bf16x8 *>(stg + (u0 + u) * (KB * KSTR) + klane + ks * 32);
                sv[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr, qf[ks], ks == 0 ? negm : sv[u], 0, 0, 0);
            }
        // causal / padding mask; columns differ in i, so every tile that reaches
        // past L_c is checked. Element e of block u is key 32 u + 8 (e / 4) + e % 4 + 4 half, counted from kbw.
        if (kbw + KB * NUW - 1 > Lc) {
            const int rel = Lc + i_row - kbw - 4 * half;
#pragma unroll
            for (int u = 0; u < NUW; ++u)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    if (KB * u + 8 * (e / 4) + (e % 4) > rel)
                        sv[u][e] = EN_NEG_INF;
        }
        // ---- reference (first visible tile, or near overflow) ----
        constexpr float BIG = 1.0e18f;
        bf16x8 pf[NUW][2];
        float rs = 0.f;
        {
            float p[NUW][16];
#pragma unroll
            for (int u = 0; u < NUW; ++u)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    p[u][e] = fast_exp2(sv[u][e]);
                    rs += p[u][e];
                }
            if (__any(pending || !(rs < BIG))) {
                float mx = sv[0][0];
#pragma unroll
                for (int u = 0; u < NUW; ++u)
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
                for (int u = 0; u < NUW; ++u)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        p[u][e] = fast_exp2(sv[u][e] - delta);
            }
            // the sums use the rounded probabilities, like the products
            rs = 0.f;
#pragma unroll
            for (int u = 0; u < NUW; ++u)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const bf16_t pb = (bf16_t)p[u][e];
                    pf[u][e / 8][e % 8] = pb;
                    rs += (float)pb;
                }
        }
        l_part += rs;
        // ---- per-bucket partial sums ----
        // (a wave that takes every other block closes the buckets that lie between its blocks
        // with what it had of them, possibly nothing: ranges below kbw select no element)
        const int ke = min(kbw + KB * NUW, split_key_end);
        if (cur_end > ke) {
            seg_part += rs;
        } else if (kbw < split_key_end) {
            int lo = kbw;
            while (true) {
                const int hi = min(cur_end, ke);
                float part = 0.f;
                const int rlo = lo - kbw - 4 * half, rhi = hi - kbw - 4 * half;
#pragma unroll
                for (int u = 0; u < NUW; ++u)
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
        for (int u = 0; u < NUW; ++u)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                for (int d = 0; d < NDB; ++d) {
                    const bf16x8 av = *reinterpret_cast<const bf16x8 *>(stg + (u0 + u) * (KB * 2) + vlane + kk * 32 + d * 32 * VSTR);
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
        *reinterpret_cast<f32x2 *>(a.ws_ml + ((size_t)spw * a.B * a.Hq * a.Nq + row) * 2) = v;
    }
    if (!row_valid)
        return;
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    bf16_t *op = (a.n_splits * SUB == 1)
                     ? (bf16_t *)a.out + (((size_t)b * a.Nq + i_row) * a.Hq + hq) * D
                     : (bf16_t *)a.ws_opart + ((size_t)spw * a.B * a.Hq * a.Nq + row) * D;
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
    const int kbeg = (int)split_first_tile(sp, ntiles, a.n_splits) * EN_KEY_TILE;
    const int kend_split = min((int)split_first_tile(sp + 1, ntiles, a.n_splits) * EN_KEY_TILE, Ltot);
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
// launcher: fp32 pools, steps that fit the decode kernel, everything else
// ---------------------------------------------------------------------------
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
        const dim3 grid((a.total_wgs + 7) / 8 * 8), blk(64 * a.sub);
        if (a.sub != 1 && a.sub != 2)
            return (int)hipErrorInvalidValue;
        if (D == 64) {
            if (a.sub == 1)
                hipLaunchKernelGGL((attn_decode_kernel<64, 1>), grid, blk, 0, st, a);
            else
                hipLaunchKernelGGL((attn_decode_kernel<64, 2>), grid, blk, 0, st, a);
        } else {
            if (a.sub == 1)
                hipLaunchKernelGGL((attn_decode_kernel<128, 1>), grid, blk, 0, st, a);
            else
                hipLaunchKernelGGL((attn_decode_kernel<128, 2>), grid, blk, 0, st, a);
        }
    } else {
        return en_launch_attention_prefill(pool, a, stream);
    }
    return (int)hipGetLastError();
}
