/*
 * CPU oracle for attention over retrieval-selected, discretely cached KV
 * segments (EfficientNav, arXiv 2510.18546).
 *
 * THIS IS TEST INFRASTRUCTURE. It is the plain definition of what the GPU
 * library computes, written out in float64 with explicit gather and explicit
 * rotary position encoding, and it shares no code with the GPU path. Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What is computed, and where the paper defines it:
 *   - every group of the navigation map owns a K/V block that was prefilled
 *     on its own, so blocks can be reused under any selection and order
 *     (Section 3.2, "Discrete Memory Caching");
 *   - the selected blocks are placed first and the new prompt tokens
 *     (instruction + trajectory) follow them (Appendix B, planning prompt);
 *   - attention is softmax(Q K^T / sqrt(D)) V (Appendix A; the source omits
 *     the trailing V, the standard product is taken);
 *   - the attention that new tokens pay to each existing group is the signal
 *     for attention-based memory clustering (Section 3.3).
 * Position handling (Section 3.2 refers to prompt-cache style re-positioning
 * without a formula): cached keys are stored unrotated and receive the rotary
 * encoding of their position in the NEW concatenation; new token j sits at
 * position L_c + j. Rotary pairs are (k, k + D/2), theta_k = base^(-2k/D).
 *
 * Inputs arrive as float32 (values already rounded to the storage type by the
 * input generator); all arithmetic below is double.
 *
 * Parity pins (tests/test_oracle_*.py): brute force with a materialised score
 * matrix, a library causal attention for S <= 1, closed forms for K = 0,
 * RoPE shift invariance, GQA expansion, segment permutation, dominance.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int en_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* offset[s] = sum of len[sel[j]] for j < s; offset[S] = L_c.
 * Returns 0, or -1 on a group id outside [0, G). */
int en_oracle_plan(int G, const int32_t *len, int S, const int32_t *sel,
                   int32_t *offset /* [S+1] */)
{
    int32_t acc = 0;
    for (int s = 0; s < S; ++s) {
        if (sel[s] < 0 || sel[s] >= G)
            return -1;
        offset[s] = acc;
        acc += len[sel[s]];
    }
    offset[S] = acc;
    return 0;
}

/* Rotary encoding of one row of D values at integer position pos. */
static void rope_row(double *x, int D, int64_t pos, double base)
{
    const int half = D / 2;
    for (int k = 0; k < half; ++k) {
        const double theta = pow(base, -2.0 * (double)k / (double)D);
        const double ang = (double)pos * theta;
        const double c = cos(ang), s = sin(ang);
        const double a = x[k], b = x[k + half];
        x[k] = a * c - b * s;
        x[k + half] = b * c + a * s;
    }
}

void en_oracle_rope(double *x, int D, int64_t pos, double base)
{
    rope_row(x, D, pos, base);
}

/*
 * Explicit gather for one agent.
 *   k_pool, v_pool : [G, Hkv, C, D] float32, keys unrotated
 *   k_new,  v_new  : [Nq, Hkv, D]   float32 for this agent
 *   kc, vc         : [Hkv, L, D]    double, L = L_c + Nq
 * Row j < L_c of head h is token (j - offset[s]) of group sel[s], the key
 * rotated at position j; rows L_c + j are the new tokens, keys rotated at
 * L_c + j. Values are copied unchanged.
 */
int en_oracle_gather_rope(int G, int Hkv, int C, int D,
                          const float *k_pool, const float *v_pool,
                          const int32_t *len, int S, const int32_t *sel,
                          int Nq, const float *k_new, const float *v_new,
                          double rope_base, double *kc, double *vc)
{
    int32_t *off = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S + 1));
    if (!off)
        return -2;
    if (en_oracle_plan(G, len, S, sel, off) != 0) {
        free(off);
        return -1;
    }
    const int Lc = off[S];
    const int L = Lc + Nq;
    for (int h = 0; h < Hkv; ++h) {
        for (int s = 0; s < S; ++s) {
            const int g = sel[s];
            for (int t = 0; t < len[g]; ++t) {
                const size_t src = (((size_t)g * Hkv + h) * C + t) * D;
                const size_t dst = ((size_t)h * L + off[s] + t) * D;
                for (int d = 0; d < D; ++d) {
                    kc[dst + d] = (double)k_pool[src + d];
                    vc[dst + d] = (double)v_pool[src + d];
                }
                rope_row(kc + dst, D, off[s] + t, rope_base);
            }
        }
        for (int j = 0; j < Nq; ++j) {
            const size_t src = ((size_t)j * Hkv + h) * D;
            const size_t dst = ((size_t)h * L + Lc + j) * D;
            for (int d = 0; d < D; ++d) {
                kc[dst + d] = (double)k_new[src + d];
                vc[dst + d] = (double)v_new[src + d];
            }
            rope_row(kc + dst, D, Lc + j, rope_base);
        }
    }
    free(off);
    return 0;
}

/*
 * The whole path for B agents.
 *   sel, sel_ptr : concatenated per-agent selections, sel_ptr[B+1]
 *   q            : [B, Nq, Hq, D] float32, unrotated
 *   k_new, v_new : [B, Nq, Hkv, D]
 *   rows         : NULL => every (b, i, hq); else n_rows triples (b, i, hq)
 *   out          : [n, D] double, n = B*Nq*Hq in (b, i, hq) order, or n_rows
 *   mass         : [n, Smax + 1] double; for agent b with S_b segments,
 *                  entry s < S_b is the probability mass on segment s, entry
 *                  S_b the mass on the new-token block, the rest 0.
 * Query head hq reads KV head hq / (Hq/Hkv). New token i sees every cached key
 * and new tokens j <= i.
 */
int en_oracle_attention(int B, int Hq, int Hkv, int D, int G, int C,
                        const float *k_pool, const float *v_pool,
                        const int32_t *len, const int32_t *sel,
                        const int32_t *sel_ptr, int Nq, const float *q,
                        const float *k_new, const float *v_new,
                        double rope_base, int Smax, int n_rows,
                        const int32_t *rows, double *out, double *mass)
{
    if (Hkv <= 0 || Hq % Hkv != 0 || D % 2 != 0)
        return -3;
    const int r = Hq / Hkv;
    const double scale = 1.0 / sqrt((double)D);
    const int M = Smax + 1;

    for (int b = 0; b < B; ++b) {
        const int S = sel_ptr[b + 1] - sel_ptr[b];
        const int32_t *sb = sel + sel_ptr[b];
        if (S > Smax)
            return -4;

        /* rows of this agent */
        int n_mine = 0;
        int32_t *mine = NULL;           /* indices into the output */
        if (rows) {
            mine = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_rows > 0 ? n_rows : 1));
            for (int n = 0; n < n_rows; ++n)
                if (rows[3 * n] == b)
                    mine[n_mine++] = n;
            if (n_mine == 0) {
                free(mine);
                continue;
            }
        } else {
            n_mine = Nq * Hq;
        }

        int32_t *off = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S + 1));
        if (en_oracle_plan(G, len, S, sb, off) != 0) {
            free(off);
            free(mine);
            return -1;
        }
        const int Lc = off[S];
        const int L = Lc + Nq;
        double *kc = (double *)malloc(sizeof(double) * (size_t)Hkv * L * D);
        double *vc = (double *)malloc(sizeof(double) * (size_t)Hkv * L * D);
        if (!kc || !vc)
            return -2;
        int rc = en_oracle_gather_rope(G, Hkv, C, D, k_pool, v_pool, len, S, sb, Nq,
                                       k_new + (size_t)b * Nq * Hkv * D,
                                       v_new + (size_t)b * Nq * Hkv * D,
                                       rope_base, kc, vc);
        if (rc != 0)
            return rc;

#pragma omp parallel
        {
            double *qr = (double *)malloc(sizeof(double) * (size_t)D);
            double *p = (double *)malloc(sizeof(double) * (size_t)L);
#pragma omp for schedule(dynamic, 8)
            for (int n = 0; n < n_mine; ++n) {
                int i, hq;
                size_t o;
                if (rows) {
                    o = (size_t)mine[n];
                    i = rows[3 * o + 1];
                    hq = rows[3 * o + 2];
                } else {
                    i = n / Hq;
                    hq = n % Hq;
                    o = ((size_t)b * Nq + i) * Hq + hq;
                }
                const int h = hq / r;
                const double *K = kc + (size_t)h * L * D;
                const double *V = vc + (size_t)h * L * D;
                const float *qs = q + (((size_t)b * Nq + i) * Hq + hq) * D;
                for (int d = 0; d < D; ++d)
                    qr[d] = (double)qs[d];
                rope_row(qr, D, Lc + i, rope_base);

                const int vis = Lc + i + 1;       /* keys 0 .. L_c + i are visible */
                double mx = -INFINITY;
                for (int j = 0; j < vis; ++j) {
                    double acc = 0.0;
                    for (int d = 0; d < D; ++d)
                        acc += qr[d] * K[(size_t)j * D + d];
                    p[j] = acc * scale;
                    if (p[j] > mx)
                        mx = p[j];
                }
                double sum = 0.0;
                for (int j = 0; j < vis; ++j) {
                    p[j] = exp(p[j] - mx);
                    sum += p[j];
                }
                for (int j = 0; j < vis; ++j)
                    p[j] /= sum;

                double *orow = out + o * D;
                for (int d = 0; d < D; ++d)
                    orow[d] = 0.0;
                for (int j = 0; j < vis; ++j)
                    for (int d = 0; d < D; ++d)
                        orow[d] += p[j] * V[(size_t)j * D + d];

                double *mrow = mass + o * M;
                for (int s = 0; s < M; ++s)
                    mrow[s] = 0.0;
                for (int s = 0; s < S; ++s)
                    for (int j = off[s]; j < off[s + 1]; ++j)
                        mrow[s] += p[j];
                for (int j = Lc; j < vis; ++j)
                    mrow[S] += p[j];
            }
            free(qr);
            free(p);
        }
        free(kc);
        free(vc);
        free(off);
        free(mine);
    }
    return 0;
}
