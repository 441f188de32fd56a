/*
 * efficientnav.h — C ABI of libefficientnav.so (MI355X / gfx950).
 *
 * Attention over discretely cached, retrieval-selected KV segments: the
 * data-parallel hot path of one planning step of EfficientNav
 * (arXiv 2510.18546).
 *
 *   kv_pool_create              one K/V block per navigation-map group, each
 *                               prefilled on its own (Section 3.2)
 *   segment_select[_scored]     which groups enter the prompt, in which order,
 *                               and where each lands (Section 3.4, Eq. (1))
 *   gather_rope[_queries]       load the selected blocks once per planning
 *                               step and re-position them (Section 3.2)
 *   segmented_prefill_attention new prompt tokens attend over
 *                               [selected segments || themselves]
 *                               (Appendix A; prompt order of Appendix B)
 *   segment_attention_mass      attention paid to each group, the clustering
 *                               signal of Section 3.3
 *   segment_cluster_assign      that signal per new object, and the join /
 *                               new-group decision
 *   kv_pool_append              new objects' KV saved at the end of their group
 *   segmented_decode_step       one decode step over the context gathered once
 *   kv_tier_*                   which groups are in device memory, loads of the
 *                               others from a host store, cache hit rate
 *
 * Conventions
 *   - Every call returns an en_status; en_last_error() gives the text of the
 *     calling thread's last failure. Nothing throws, nothing aborts.
 *   - "dev" pointers are device memory owned by the caller (e.g. the
 *     data_ptr() of a torch tensor on the GPU); "host" pointers are host
 *     memory. The library never frees or keeps caller host memory. It keeps
 *     the pool's k/v device pointers inside the en_pool until it is destroyed.
 *   - The library owns only small bookkeeping inside its opaque handles (the
 *     rotary table of a pool, the descriptor block of a plan). These are
 *     uploaded on first GPU use, so the select calls are pure host code.
 *   - Kernels are enqueued on the caller's hipStream_t (passed as void*, NULL
 *     = the default stream). No call synchronises the stream.
 *   - A pool should outlive its plans: of a plan whose pool has been destroyed
 *     only en_plan_destroy may still be called. Calls on one handle are
 *     serialised by the caller; a pool may be read by many plans.
 *   - Notation: G groups of capacity C token slots, len[g] <= C tokens in use,
 *     Hq query heads, Hkv KV heads (Hq % Hkv == 0, query head h reads KV head
 *     h / (Hq/Hkv)), head dimension D in {64, 128}, B agents (independent
 *     planning steps sharing the pool), S_b selected segments of agent b,
 *     offset[s] = sum_{j<s} len[sel[j]], L_c = offset[S_b], N_q new tokens at
 *     positions L_c .. L_c+N_q-1.
 */
#ifndef EFFICIENTNAV_H
#define EFFICIENTNAV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum en_status {
    EN_OK = 0,
    EN_ERR_INVALID_ARG = 1,   /* null pointer, negative size, bad enum        */
    EN_ERR_OUT_OF_RANGE = 2,  /* group id outside [0,G) or len outside [0,C]  */
    EN_ERR_DUPLICATE = 3,     /* a group twice in one agent's selection       */
    EN_ERR_CAPACITY = 4,      /* L_c + N_q exceeds max_ctx / buffer too small */
    EN_ERR_UNSUPPORTED = 5,   /* head_dim, head ratio, dtype or size not supported */
    EN_ERR_DEVICE = 6         /* a HIP call failed; see en_last_error()       */
} en_status;

typedef enum en_dtype {
    EN_F32 = 0,
    EN_BF16 = 1,
    EN_I8 = 2   /* pool of 8-bit codes with one float scale per (group, head, token),
                   see kv_pool_set_scales; contexts, queries, outputs are bf16 */
} en_dtype;

typedef struct en_pool en_pool; /* opaque */
typedef struct en_plan en_plan; /* opaque */

typedef struct en_pool_desc {
    int32_t n_groups;   /* G                                                  */
    int32_t capacity;   /* C                                                  */
    int32_t n_kv_heads; /* Hkv                                                */
    int32_t n_q_heads;  /* Hq                                                 */
    int32_t head_dim;   /* D: 64 or 128                                       */
    int32_t dtype;      /* en_dtype of pool, Q, new K/V, context and output   */
    int32_t max_ctx;    /* upper bound on L_c + N_q (rotary table rows)       */
    int32_t reserved;   /* must be 0                                          */
    double rope_base;   /* theta_k = rope_base^(-2k/D), pairs (k, k + D/2)    */
} en_pool_desc;

typedef struct en_plan_info {
    int32_t n_agents;     /* B                                                */
    int32_t n_new;        /* N_q                                              */
    int32_t max_segments; /* max_b S_b                                        */
    int32_t ctx_stride;   /* token stride of the context buffers (>= every
                             L_c + N_q, multiple of 64)                       */
    int32_t max_ctx_len;  /* max_b (L_c + N_q)                                */
    int32_t n_splits;     /* KV splits the attention kernel will use          */
    int64_t total_pairs;  /* visible (query,key) pairs over all agents, one
                             head: sum_b N_q*L_c + N_q(N_q+1)/2               */
    int64_t total_cached; /* sum_b L_c                                        */
} en_plan_info;

/* ------------------------------------------------------------------------
 * Pool of per-group K/V blocks (Section 3.2: the KV cache of each group is
 * computed individually, so it does not depend on which other groups are
 * selected or on their order).
 *   k_dev, v_dev : device, [G, Hkv, C, D] of desc->dtype; keys are stored
 *                  UNROTATED (no position encoding applied). Rows t >= len[g]
 *                  are never read.
 *   len_host     : host, int32 [G]; copied.
 * Errors: INVALID_ARG (null, non-positive sizes, reserved != 0),
 *         UNSUPPORTED (D not 64/128, Hq % Hkv != 0, unknown dtype),
 *         OUT_OF_RANGE (a len outside [0, C]).
 */
int kv_pool_create(const en_pool_desc *desc, void *k_dev, void *v_dev,
                   const int32_t *len_host, en_pool **out);

/* 8-bit pools (an option beside the paper's method, which names quantisation as
 * compatible with it, Section 2): with desc->dtype = EN_I8, k_dev / v_dev hold
 * int8 codes [G, Hkv, C, D] and every (group, head, token) row has a scale:
 * value = code * scale. Scales: device float [G, Hkv, C] for keys and for
 * values, owned by the caller like the pool arrays; set them before the first
 * gather_rope. gather_rope turns the selected rows into the same bf16 contexts
 * as for an EN_BF16 pool (keys: code * scale in float32, rotated, rounded once;
 * values: code * scale rounded to bf16); new tokens, queries, outputs and the
 * attention itself are bf16. kv_pool_append takes bf16 rows and stores codes and
 * scales: scale = max|x| / 127 over the row, code = x / scale rounded to the
 * nearest integer (ties to even), all in float32; a zero row gets scale 0.
 * Residency tiers do not take EN_I8 pools.
 * Errors: INVALID_ARG (null; pool is not EN_I8). */
int kv_pool_set_scales(en_pool *pool, float *k_scale_dev, float *v_scale_dev);

/* Record that group `group` now holds `len` tokens (the caller has written the
 * rows; Section 3.2: new objects are appended at the end of their group).
 * Plans made before the change keep the old length. */
int kv_pool_set_len(en_pool *pool, int32_t group, int32_t len);

/* Append to a group (Section 3.2, memory caching: when new objects join a
 * group only their KV is computed, and it is saved at the end of the group's
 * cache; the rows already there are not touched).
 *   k_rows_dev, v_rows_dev : device, [n_tokens, Hkv, D] in the pool dtype, keys
 *                            UNROTATED, e.g. a token range of a step's
 *                            new-token block; read on `stream`, not kept.
 * Enqueues on `stream` the copy of the rows to tokens len .. len+n_tokens-1 of
 * `group` in both pool arrays and then counts them in (host side, at once):
 * plans made after the call see the new length and must run on the same stream
 * or after it; plans made before keep the old one. n_tokens = 0 does nothing.
 * Errors: INVALID_ARG (null, n_tokens < 0), OUT_OF_RANGE (group),
 *         CAPACITY (len + n_tokens > C: nothing is copied), DEVICE.
 */
int kv_pool_append(en_pool *pool, int32_t group, const void *k_rows_dev, const void *v_rows_dev,
                   int32_t n_tokens, void *stream);

int kv_pool_destroy(en_pool *pool);

/* ------------------------------------------------------------------------
 * Selection, explicit form: the caller's ordered lists are honoured verbatim
 * (selection changes the order of context in the prompt, Section 3.2; cached
 * groups precede the new tokens, Appendix B).
 *   sel_host     : host, int32, the B lists concatenated
 *   sel_ptr_host : host, int32 [B+1], list b is sel[sel_ptr[b] .. sel_ptr[b+1])
 *   n_new        : N_q >= 1 new tokens per agent
 * Computes, per agent, offset[S_b+1] by exclusive prefix sum of the groups'
 * lengths. Pure host code. S_b = 0 and len = 0 groups are allowed.
 * Errors: OUT_OF_RANGE (id), DUPLICATE, CAPACITY (L_c + N_q > max_ctx),
 *         INVALID_ARG.
 */
int segment_select(const en_pool *pool, int32_t n_agents, const int32_t *sel_host,
                   const int32_t *sel_ptr_host, int32_t n_new, en_plan **out);

/* Selection, retrieval form (Section 3.4, Eq. (1)): maximise
 * sum_i (P_i - threshold) x_i subject to sum_i len_i x_i <= budget_tokens,
 * x_i in {0,1}; memory is counted in tokens. The objective is evaluated in
 * fixed point, value_i = nearest-even((double)P_i - (double)threshold) * 2^32,
 * so ties are exact; groups with value_i <= 0 are never taken; among optimal
 * sets the one with fewest tokens wins, then the lexicographically smallest
 * sorted id list. One agent; ids are emitted in ascending order.
 *   p_host        : host, float [G]
 *   sel_out_host  : host, int32 [G] (capacity), receives the ids
 *   n_sel_out     : receives the count
 *   out           : may be NULL (selection only); else as segment_select.
 * Errors: INVALID_ARG (null, budget < 0), CAPACITY.
 */
int segment_select_scored(const en_pool *pool, const float *p_host, float threshold,
                          int64_t budget_tokens, int32_t n_new, int32_t *sel_out_host,
                          int32_t *n_sel_out, en_plan **out);

int en_plan_get_info(const en_plan *plan, en_plan_info *info);

/* offsets_out_host: int32 [S_b + 1] (offset[S_b] = L_c); n_seg_out: S_b.
 * Either may be NULL. Exact integers, for bit-exact checks of the gather. */
int en_plan_query(const en_plan *plan, int32_t agent, int32_t *offsets_out_host,
                  int32_t *n_seg_out);

/* Override the number of KV splits chosen by segment_select (>= 1, clamped to
 * the number of 64-key tiles and to 64). Must precede en_workspace_bytes. */
int en_plan_set_splits(en_plan *plan, int32_t n_splits);

/* Prefill-only steps: leave the values where they are (Section 3.2 asks for each
 * selected group's KV to be loaded once; a step that no decode phase follows has no
 * second reader for a gathered copy of the values). With on = 1, gather_rope and
 * gather_rope_queries still write the rotated keys, but into vt_dev only, per
 * (agent, KV head, context row), the device address of that row's values in the
 * pool's block or in v_new_dev (8 bytes per row, [B, Hkv, T], then one row of
 * zeros for the padding of the last tile; the buffer keeps its size,
 * en_context_bytes), and segmented_prefill_attention[_prepared] fetch the rows
 * from there. Results are bit-identical to those of the gathered form. The pool's
 * values and v_new_dev must stay unchanged, and allocated, from the gather to the
 * end of the attention call. Set it before the gather; a change after the gather
 * makes the attention calls fail (INVALID_ARG) until the plan is gathered again.
 * Errors: INVALID_ARG (null, flag not 0 / 1, values not aligned to a row of
 * 2 * head_dim bytes: the pool's here, v_new_dev at the gather), UNSUPPORTED (not
 * an EN_BF16 pool; a plan of so few new tokens that its attention runs in the
 * decode kernel). segmented_decode_step[_static] and any step over a part of the
 * plan's rows return UNSUPPORTED on such a plan: they read gathered values. */
int en_plan_values_from_pool(en_plan *plan, int32_t on);

/* May be called while work that uses the plan is still queued on a stream,
 * provided later plans of the same pool are used on that same stream;
 * otherwise synchronise first. */
int en_plan_destroy(en_plan *plan);

/* ------------------------------------------------------------------------
 * Context buffers. gather_rope fills them, the attention kernel reads them.
 * Both have en_context_bytes(pool, plan) bytes. With T = ctx_stride:
 *   kc_dev : [B, Hkv, T, D]; row j < L_c is token j - offset[s] of group
 *            sel[s] with rotary encoding applied at position j; rows
 *            L_c + j are the new tokens' keys rotated at L_c + j; rows from
 *            L_c + N_q up to the next multiple of 64 are zero.
 *   vt_dev : EN_BF16: [B, Hkv, D, T], values transposed (token index
 *            fastest); token j is stored at column j with bits 2 and 3 of j
 *            exchanged (the order in which the PV matrix instruction consumes
 *            keys). EN_F32: [B, Hkv, T, D], plain copy. Padding as above.
 * Values are bit-exact copies of the pool / new-token values.
 */
size_t en_context_bytes(const en_pool *pool, const en_plan *plan);

/* Gather the selected blocks once per planning step (Section 3.2: select,
 * then load the required KV only once) and apply position encoding at the
 * concatenated positions.
 *   k_new_dev, v_new_dev : device, [B, N_q, Hkv, D], keys unrotated
 * Errors: INVALID_ARG, DEVICE.
 */
int gather_rope(en_pool *pool, en_plan *plan, const void *k_new_dev, const void *v_new_dev,
                void *kc_dev, void *vt_dev, void *stream);

/* gather_rope, and in the same launch the step's queries prepared for the
 * attention kernel: rotated at L_c + i, scaled by log2(e)/sqrt(D) (the softmax
 * runs in the log2 domain) and rounded to bf16 once, which
 * segmented_prefill_attention otherwise does in every workgroup, once per KV
 * split. For segmented_prefill_attention_prepared on the same plan.
 *   q_dev      : device, [B, N_q, Hq, D] bf16, unrotated
 *   q_prep_dev : device, [B, N_q, Hq, D] bf16, receives the prepared queries
 * EN_BF16 and EN_I8 pools. Errors: as gather_rope, UNSUPPORTED (EN_F32 pool).
 */
int gather_rope_queries(en_pool *pool, en_plan *plan, const void *k_new_dev, const void *v_new_dev,
                        const void *q_dev, void *kc_dev, void *vt_dev, void *q_prep_dev, void *stream);

/* Bytes of scratch the attention call needs for this plan: per-split running
 * (max, sum), per-(row, segment) partial sums, and, when n_splits > 1, partial
 * outputs (a step of few rows and few agents keeps two partial results per
 * split: the size accounts for it). */
size_t en_workspace_bytes(const en_pool *pool, const en_plan *plan);

/* softmax(Q K^T / sqrt(D)) V (Appendix A) of the N_q new tokens over the
 * gathered context: every cached key is visible, new token i also sees new
 * tokens j <= i. Q is rotated at L_c + i inside the kernel.
 *   q_dev   : device, [B, N_q, Hq, D], unrotated
 *   out_dev : device, [B, N_q, Hq, D]
 *   ws_dev  : device scratch of at least en_workspace_bytes; it receives the
 *             raw per-segment sums that segment_attention_mass turns into
 *             masses. NULL is allowed when the plan has n_splits == 1 and no
 *             masses are wanted.
 * Errors: INVALID_ARG, CAPACITY (ws_bytes too small), DEVICE.
 */
int segmented_prefill_attention(en_pool *pool, en_plan *plan, const void *q_dev,
                                const void *kc_dev, const void *vt_dev, void *out_dev,
                                void *ws_dev, size_t ws_bytes, void *stream);

/* segmented_prefill_attention over queries that gather_rope_queries prepared
 * (the arithmetic is the same, the results are bit for bit those of
 * segmented_prefill_attention on the unprepared queries), optionally with the
 * reduced masses in the same launches:
 *   q_prep_dev       : device, [B, N_q, Hq, D] bf16, from gather_rope_queries
 *   mass_red_out_dev : device float [B, Smax+1] or NULL: receives what
 *                      segment_attention_mass(reduce = 1) would write, without a
 *                      launch of its own. The heads' sums are added up as
 *                      fixed-point integers (in the scratch; with one KV split,
 *                      by the attention kernel itself in words that belong to
 *                      the plan, so calls on one plan must not overlap), so the
 *                      result does not depend on the order in which they arrive
 *                      and is the same from run to run; it may differ from what
 *                      segment_attention_mass(reduce = 1) gives (a float sum in
 *                      a fixed order) in the last bits. That call may still
 *                      follow, with either reduce mode. At most 1023 query
 *                      heads.
 * Plans whose steps have enough query rows for the matrix-core prefill kernel
 * (more than 32 rows per KV head); EN_BF16 and EN_I8 pools.
 * Errors: as segmented_prefill_attention, UNSUPPORTED (EN_F32 pool, or so few
 * rows that the decode kernel takes the step).
 */
int segmented_prefill_attention_prepared(en_pool *pool, en_plan *plan, const void *q_prep_dev,
                                         const void *kc_dev, const void *vt_dev, void *out_dev,
                                         float *mass_red_out_dev, void *ws_dev, size_t ws_bytes,
                                         void *stream);

/* Decode-phase reuse of a gathered context (Section 3.2: the selected KV is
 * loaded once per planning step, then about 40 tokens are decoded over it).
 * A plan made with n_new = N_q reserves N_q new-token slots behind the cached
 * segments; gather_rope fills the context once (the new-token rows it is given
 * may be placeholders, but must be finite); each call below then handles new
 * tokens q_first .. q_first+n_rows-1:
 *   1. their keys (rotated at positions L_c + q_first + t) and values are
 *      written into the context buffers,
 *   2. their queries attend over every key before and including them (the
 *      same arithmetic and kernels as segmented_prefill_attention; the result
 *      equals rows q_first .. of one prefill over all tokens up to them),
 *   3. if mass_out_dev is not NULL, their per-segment masses
 *      [B, n_rows, Hq, Smax+1] are written as by segment_attention_mass with
 *      reduce = 0 (bucket S_b = all new tokens visible to the row).
 * Steps must come in order of q_first on one stream (a step reads the rows
 * written by the earlier ones). All kernels are enqueued on `stream`; nothing
 * is allocated, so a sequence of steps can be captured into a HIP graph.
 *   q_dev                   : device, [B, n_rows, Hq, D], unrotated
 *   k_rows_dev, v_rows_dev  : device, [B, n_rows, Hkv, D], keys unrotated
 *   kc_dev, vt_dev          : the context buffers filled by gather_rope (updated)
 *   out_dev                 : device, [B, n_rows, Hq, D]
 *   ws_dev, ws_bytes        : scratch of at least en_decode_workspace_bytes(pool,
 *                             plan, n_rows) (the KV split count of a step is chosen
 *                             for n_rows, not for the plan's N_q)
 * Errors: INVALID_ARG, OUT_OF_RANGE (q_first + n_rows > N_q), CAPACITY, DEVICE.
 */
size_t en_decode_workspace_bytes(const en_pool *pool, const en_plan *plan, int32_t n_rows);
int segmented_decode_step(en_pool *pool, en_plan *plan, int32_t q_first, int32_t n_rows,
                          const void *q_dev, const void *k_rows_dev, const void *v_rows_dev,
                          void *kc_dev, void *vt_dev, void *out_dev, float *mass_out_dev,
                          void *ws_dev, size_t ws_bytes, void *stream);

/* segmented_decode_step for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * The same step, with the scratch taken from a static device array of
 * EN_STATIC_SCRATCH_BYTES (8 MiB) that is part of the library's code object
 * (every GPU the library runs on holds its own copy until the process ends).
 * This call allocates nothing and frees nothing, on the device or through any
 * library: the pool and the plan must already have been through gather_rope
 * (which is where the rotary table and the plan's descriptor block are created;
 * a decode step follows a gather anyway), else INVALID_ARG.
 * A step whose scratch (en_decode_workspace_bytes) exceeds the static array is
 * refused with CAPACITY: one agent over 8.7 K tokens needs 1.6 MB, 64 agents over
 * 16 K tokens 3.2 MB.
 * All calls on one GPU share that GPU's array, which keeps what the last call
 * left in it (the kernels write every entry they later read; nothing relies on
 * zeroes): calls that overlap in time on one GPU race, so keep them on one
 * stream or order them yourself. The step's masses come back through
 * mass_out_dev; segment_cluster_assign_rows reads a caller's workspace and does
 * not follow this call.
 * Other arguments and errors as segmented_decode_step.
 */
#define EN_STATIC_SCRATCH_BYTES ((size_t)8 << 20)
int segmented_decode_step_static(en_pool *pool, en_plan *plan, int32_t q_first, int32_t n_rows,
                                 const void *q_dev, const void *k_rows_dev, const void *v_rows_dev,
                                 void *kc_dev, void *vt_dev, void *out_dev, float *mass_out_dev,
                                 void *stream);

/* Per-segment attention mass (Section 3.3: the attention between newly
 * detected objects and an existing group) from the scratch left by the
 * attention call on the same plan and stream.
 *   reduce = 0 : mass_out_dev float [B, N_q, Hq, Smax+1]; for agent b entry
 *                s < S_b is the softmax probability mass that (query i,
 *                head h) puts on segment s, entry S_b the mass on the new
 *                block, entries beyond are 0; each row sums to 1.
 *   reduce = 1 : mass_out_dev float [B, Smax+1], the above summed over heads
 *                and query tokens (divide by Hq*N_q for the average).
 * The reduced form also writes a small part of the scratch (per-head partial
 * sums): two reduced calls on one scratch must not overlap in time.
 * Errors: INVALID_ARG, DEVICE.
 */
int segment_attention_mass(en_pool *pool, en_plan *plan, void *ws_dev, int32_t reduce,
                           float *mass_out_dev, void *stream);

/* Clustering signal and decision (Section 3.3, attention-based memory
 * clustering: a newly detected object joins the existing group it attends to
 * most if that attention passes a threshold, otherwise it founds a new group).
 * An object is a span of the new tokens; its score against cached segment s is
 * the mean, over the span's tokens and over the query heads, of the attention
 * mass on s (per_key = 0) or of that mass divided by the segment's length,
 * i.e. the mean attention weight per (query token, key token) pair
 * (per_key = 1). From the scratch left by the attention call on the same plan
 * and stream.
 *   n_obj, span_ptr_host : host int32 [n_obj+1], object o = new tokens
 *                          [span_ptr[o], span_ptr[o+1]), the same for every
 *                          agent; 0 <= span_ptr[o] < span_ptr[o+1] <= N_q
 *   accumulate           : 0 the scores are written; 1 they are added to what
 *                          score_dev holds (the paper averages the first tenth
 *                          of the layers: one call per layer)
 *   scale, threshold     : the decision looks at score * scale (e.g. 1/layers):
 *                          the cached segment s < S_b with the largest value,
 *                          the lowest s among equals, if that value >=
 *                          threshold, else -1 (new group). Empty segments and
 *                          the new tokens' own bucket never win.
 *   score_dev            : device float [B, n_obj, Smax+1] (bucket S_b = the new
 *                          tokens themselves, always a mass, never divided;
 *                          entries beyond it 0)
 *   assign_dev           : device int32 [B, n_obj], position in the agent's
 *                          selection list or -1; may be NULL (scores only)
 * Errors: INVALID_ARG (null, bad spans, per_key/accumulate not 0/1), DEVICE.
 */
int segment_cluster_assign(en_pool *pool, en_plan *plan, void *ws_dev, int32_t n_obj,
                           const int32_t *span_ptr_host, int32_t per_key, int32_t accumulate,
                           float scale, float threshold, float *score_dev, int32_t *assign_dev,
                           void *stream);

/* The same from the scratch that segmented_decode_step(q_first, n_rows) left:
 * for a plan that reserves rows for tokens still to be decoded, the prompt
 * tokens are such a step (q_first = 0). Spans count from the step's first row:
 * 0 <= span_ptr[o] < span_ptr[o+1] <= n_rows.
 * Errors: as above, OUT_OF_RANGE (q_first + n_rows > N_q). */
int segment_cluster_assign_rows(en_pool *pool, en_plan *plan, int32_t q_first, int32_t n_rows,
                                void *ws_dev, int32_t n_obj, const int32_t *span_ptr_host,
                                int32_t per_key, int32_t accumulate, float scale, float threshold,
                                float *score_dev, int32_t *assign_dev, void *stream);

/* ------------------------------------------------------------------------
 * Residency tier (Section 3.2: the KV cache of all groups is kept in a large,
 * slow store and only the selected groups are loaded into device memory, once
 * per planning step; a group selected in consecutive steps is already there.
 * Section 4, "memory caching distribution and cache hit rate": the share of the
 * selected groups found in device memory, as a function of the device budget).
 *
 * The tier owns a store of n_groups_total blocks in pinned host memory and
 * manages desc->n_groups device slots, each one block [Hkv, C, D] of K and of
 * V, in the caller's arrays k_dev / v_dev ([slots, Hkv, C, D], as for
 * kv_pool_create). kv_tier_pool() is an en_pool over those arrays whose group
 * ids are SLOT numbers: pass the slots that kv_tier_fetch returns to
 * segment_select / gather_rope. A device budget in bytes buys
 * budget / kv_tier_slot_bytes(desc) slots.
 * With k_dev = v_dev = NULL the tier only keeps the books (same decisions and
 * counters, no memory, no HIP call): for sizing a budget from a trace.
 *
 * Policy. A fetch first marks every asked-for group that is resident as used
 * now; then, in list order, each missing group takes the slot used least
 * recently (never-used slots first, lowest slot number among equals) and is
 * loaded. A group that was resident because of an earlier fetch counts as a
 * hit, one brought in by kv_tier_prefetch as prefetched, the others as misses:
 * hit rate = hits / requested.
 *
 * Ordering. Loads run on a stream of the tier's own. kv_tier_fetch makes
 * `stream` wait for the loads it needs, so work enqueued on `stream` after the
 * call sees the data. Before a slot is overwritten, the kernels that read it
 * must be done: all such reads are assumed to be enqueued on `stream` (the
 * same one in every call). kv_tier_fence(stream) says "every read of the slots
 * handed out so far is already enqueued on `stream`" (call it after
 * gather_rope: the attention kernels read the gathered context, not the
 * slots); loads then wait only for that point and run beside the kernels
 * enqueued after it. Without a fence a fetch that has to load waits for
 * everything enqueued on `stream` so far, which then counts as a fence covering
 * every earlier fetch.
 * kv_tier_prefetch loads groups that a later fetch is expected to ask for
 * (e.g. the same selection for the next layer) into slots whose readers the
 * last fence covers, least recently used first, and never waits for anything
 * else; it loads fewer groups than asked if such slots run out.
 *
 *   kv_tier_put   : k_host, v_host host [Hkv, len, D] in the pool dtype, keys
 *                   unrotated; copied into the store before the call returns
 *                   (waits for loads in flight). A device copy of the group
 *                   becomes stale and is dropped.
 *   kv_tier_append: as kv_pool_append (Section 3.2: new objects' KV is saved at
 *                   the end of the group's cache), for a group of the store:
 *                   k_rows_dev, v_rows_dev device [n_tokens, Hkv, D]. Enqueues
 *                   on `stream` the copy of the rows to the end of the block in
 *                   the store and, if the group is resident, in its slot, and
 *                   counts them in at once (plans made later see the new
 *                   length). Loads issued later wait for it. CAPACITY if the
 *                   block cannot hold them.
 *   kv_tier_select_scored : Eq. (1) as in segment_select_scored, over the
 *                   store's groups and lengths (groups never put are not
 *                   candidates); groups_out_host int32 [n_groups_total].
 *   kv_tier_fetch : groups_host int32 [n], distinct, n <= slots;
 *                   slots_out_host int32 [n] receives the slot of each.
 *   kv_tier_residency : slot_of_group_out_host int32 [n_groups_total], the
 *                   slot each group occupies or -1.
 * One tier is used by one thread at a time. The calls record and wait for events:
 * they are not for streams under graph capture.
 * Errors: INVALID_ARG, OUT_OF_RANGE (group outside the store or never put,
 *         len > C), DUPLICATE, CAPACITY (more groups than slots), UNSUPPORTED
 *         (as kv_pool_create), DEVICE.
 */
typedef struct en_tier en_tier;
typedef struct en_tier_stats {
    int64_t fetches;      /* kv_tier_fetch calls                               */
    int64_t requested;    /* groups they asked for                             */
    int64_t hits;         /* ... resident from an earlier fetch                */
    int64_t prefetched;   /* ... resident because of a prefetch                */
    int64_t misses;       /* ... loaded by the fetch itself                    */
    int64_t loads;        /* blocks copied, fetch and prefetch together        */
    int64_t bytes_loaded; /* their bytes (len tokens of K and V each)          */
    int64_t evictions;    /* loads that displaced a resident group             */
} en_tier_stats;

int64_t kv_tier_slot_bytes(const en_pool_desc *desc);
int kv_tier_create(const en_pool_desc *desc, int32_t n_groups_total, void *k_dev, void *v_dev,
                   en_tier **out);
en_pool *kv_tier_pool(en_tier *tier);
int kv_tier_put(en_tier *tier, int32_t group, const void *k_host, const void *v_host, int32_t len);
int kv_tier_append(en_tier *tier, int32_t group, const void *k_rows_dev, const void *v_rows_dev,
                   int32_t n_tokens, void *stream);
int kv_tier_select_scored(const en_tier *tier, const float *p_host, float threshold,
                          int64_t budget_tokens, int32_t *groups_out_host, int32_t *n_out);
int kv_tier_fetch(en_tier *tier, const int32_t *groups_host, int32_t n, int32_t *slots_out_host,
                  void *stream);
int kv_tier_fence(en_tier *tier, void *stream);
int kv_tier_prefetch(en_tier *tier, const int32_t *groups_host, int32_t n, int32_t *n_loaded_out);
int kv_tier_get_stats(const en_tier *tier, en_tier_stats *out);
int kv_tier_residency(const en_tier *tier, int32_t *slot_of_group_out_host);
int kv_tier_destroy(en_tier *tier);

/* ------------------------------------------------------------------------
 * Measurement aid for callers that need the duration of the attention kernel
 * itself (the kernel the roofline is quoted on), not of the whole call.
 * en_timing_enable(pool, n > 0) creates n pairs of HIP events in the pool; from
 * then on every segmented_prefill_attention / segmented_decode_step call on that
 * pool records one pair around its main kernel launch, on the stream it launches
 * on, until n pairs are used. en_timing_enable(pool, 0) frees them (so does
 * kv_pool_destroy). en_timing_collect waits for the recorded pairs, writes their
 * durations in milliseconds to ms_out_host (at most cap) and resets the record
 * count. The state belongs to the pool: calls on one pool are serialised by the
 * caller as for every other call. Not for streams under graph capture.
 * Errors: INVALID_ARG, CAPACITY (host memory), DEVICE.
 */
int en_timing_enable(en_pool *pool, int32_t max_records);
int en_timing_collect(en_pool *pool, float *ms_out_host, int32_t cap, int32_t *n_out);

/* ------------------------------------------------------------------------
 * Measured ceilings of the machine, for quoting beside the nominal peaks. They
 * compute nothing of the method; the caller times them (events on `stream`).
 *
 * en_ceiling_mfma_bf16: n_workgroups workgroups of 8 waves (two per SIMD), each
 *   wave `iters` rounds of 8 matrix instructions 32x32x16 bf16 and nothing else
 *   (operands in registers, 4 accumulators, 4 A and 2 B fragments in turn).
 *   constant_operands = 0: operand bits like normal-distributed data (random sign
 *   and mantissa); 1: every operand 0.5 (the clock of the chip depends on how many
 *   bits toggle). *flops_out receives the operations one launch performs.
 *   sink_dev: device scratch of n_workgroups * 2048 bytes (never written in
 *   practice).
 * en_ceiling_read_stream: n_workgroups workgroups read `bytes` (a multiple of 16,
 *   16-byte aligned) of device memory once, 16 bytes per lane and load, and keep
 *   nothing. sink_dev: 1024 bytes of device scratch.
 * Errors: INVALID_ARG, CAPACITY (sink too small), DEVICE.
 */
int en_ceiling_mfma_bf16(void *sink_dev, size_t sink_bytes, int32_t n_workgroups, int32_t iters,
                         int32_t constant_operands, double *flops_out, void *stream);
int en_ceiling_read_stream(const void *src_dev, size_t bytes, void *sink_dev, size_t sink_bytes,
                           int32_t n_workgroups, void *stream);

const char *en_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* EFFICIENTNAV_H */
