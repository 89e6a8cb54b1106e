/*
 * kvs.h -- C ABI of the MI355X (gfx950) library for the DHD KV-reuse hot path of KVShare
 * (Dual-Stage High Deviation token selection, Alg. 1 / Eq. (3); partial recomputation,
 * App. A; decode-stage re-check, Sec. 4.2).
 *
 * Conventions shared by every call
 * --------------------------------
 * Pointers marked [dev] are device (HBM) addresses, pointers marked [host] are ordinary host
 * memory that is read before the call returns.  The caller owns every buffer; the library
 * allocates nothing, reads no environment variable, and never synchronises.  The only state it
 * keeps between calls is, per device, which kernels have had their launch attributes set and the
 * device's compute-unit count (both written once, safely from several host threads).  Each call checks
 * its arguments on the host, enqueues its kernels on `stream` (a hipStream_t passed as
 * void*, NULL = the default stream) and returns.  Outputs are valid in stream order.
 *
 * Layouts are row-major and contiguous:
 *   K, V        [rows, n_kv_heads, head_dim]   element type given by kvs_shape.dtype
 *   Q           [rows, n_q_heads,  head_dim]
 *   dev_k/dev_v [n_kv_heads, rows] fp32        per-token, per-KV-head L1 deviation
 *   alpha       [n_kv_heads, rows] fp32        attention column mass, summed over the query
 *                                              heads that share the KV head
 *   score       [rows] fp32                    -inf for tokens that are not candidates
 * Query head h reads KV head h / (n_q_heads / n_kv_heads).  K/V/Q base addresses must be
 * 16-byte aligned.
 *
 * Errors: every function returns a kvs_status.  Argument errors are detected on the host
 * before anything is enqueued (KVS_EINVAL: NULL required pointer, negative size, k larger
 * than its row, n_q_heads not a multiple of n_kv_heads, unsorted offsets; KVS_EUNSUPPORTED:
 * head_dim/dtype combination that has no kernel; KVS_EWORKSPACE: workspace too small;
 * KVS_EHIP: the HIP runtime refused a launch).  kvs_last_error() returns a thread-local
 * description of the most recent failure.  Nothing throws or aborts across this boundary.
 *
 * Supported shapes: dtype KVS_BF16 or KVS_F32; head_dim 64 or 128; any n_q_heads that is a
 * multiple of n_kv_heads (n_kv_heads <= 64).
 */
#ifndef KVS_H
#define KVS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVS_API __attribute__((visibility("default")))

typedef enum {
    KVS_OK = 0,
    KVS_EINVAL = 1,
    KVS_EUNSUPPORTED = 2,
    KVS_EWORKSPACE = 3,
    KVS_EHIP = 4
} kvs_status;

typedef enum { KVS_F32 = 0, KVS_BF16 = 1 } kvs_dtype;

/* KVS_SCORE_V is the paper's score (value deviation only, Sec. 4.1 drops the key term);
 * KVS_SCORE_KV adds the key deviation's L1 norm under the same weight. */
typedef enum { KVS_SCORE_V = 0, KVS_SCORE_KV = 1 } kvs_score_mode;

typedef struct {
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t dtype; /* kvs_dtype */
} kvs_shape;

/*
 * kvs_deviation -- Alg. 1 step 3 / Eq. (3): the deviation impact score of every token.
 *
 *   dev_v[g,i] = sum_c | v_fresh[i,g,c] - v_cache[i,g,c] |        (L1 norm of Delta V_i on head g)
 *   dev_k[g,i] likewise on K (computed when mode == KVS_SCORE_KV or dev_k != NULL)
 *   score[i]   = sum_g alpha[g,i] * dev_v[g,i]                    mode KVS_SCORE_V
 *              = sum_g alpha[g,i] * (dev_k[g,i] + dev_v[g,i])     mode KVS_SCORE_KV
 *   score[i]   = -inf where reused[i] == 0 (the token was computed fresh, nothing to repair)
 *
 * n_tokens            rows of every tensor (0 is allowed: nothing is launched)
 * k_fresh, k_cache    [dev] may be NULL in mode KVS_SCORE_V with dev_k == NULL
 * v_fresh, v_cache    [dev] required
 * reused              [dev] uint8[n_tokens], NULL = every token is a candidate
 * alpha               [dev] fp32[n_kv_heads, n_tokens], NULL = 1 (magnitude-only ranking)
 * dev_k, dev_v, score [dev] outputs; each may be NULL if not wanted
 * All arithmetic is fp32 on exactly widened inputs, in a fixed order (bit-reproducible).
 */
KVS_API kvs_status kvs_deviation(const kvs_shape *shape, int64_t n_tokens,
                         const void *k_fresh, const void *v_fresh,
                         const void *k_cache, const void *v_cache,
                         const uint8_t *reused, const float *alpha, int32_t mode,
                         float *dev_k, float *dev_v, float *score, void *stream);

/*
 * kvs_deviation_topk -- Alg. 1 steps 3 and 4 in one call: the scores of kvs_deviation and, from
 * them, the k highest-scoring tokens of the one row of n_tokens scores, exactly as
 * kvs_select_topk(score, 1, {0, n_tokens}, {k}, idx_out) would return them (order (score
 * descending, index ascending), -0 equal to +0, -inf last, ascending indices out; bit-identical
 * to the two separate calls).  All arguments up to `score` are those of kvs_deviation.
 *
 * k        0 <= k <= n_tokens           idx_out [dev] int32[k]
 * score    [dev] fp32[n_tokens]; may be NULL only for rows of 12289 to 262144 tokens (outside that
 *          range the ranking reads the scores back from it)
 * workspace [dev] optional, as for kvs_select_topk: only used by rows above 262144 tokens
 *
 * Rows of up to 12288 tokens (one workgroup ranks them as fast) and above 262144 run as the two
 * separate calls.  Rows in between take three launches: the scoring kernel also stores every token's
 * order-preserving key and counts the keys' leading 13 bits into a histogram (integer atomics, so
 * the counts do not depend on arrival order and the result stays deterministic); then, with one
 * workgroup per 1024 keys, a launch that reads the threshold's bin off the histogram and sets the
 * few hundred keys of that bin aside, and a launch that resolves the other 19 bits on those and
 * writes the list.  Keys, histogram (32 KiB) and the records the launches exchange live in
 * device memory that belongs to the library (2.1 MB per device); the histogram is all zero
 * whenever no such call is in flight.  Calls that overlap in time on one device (two streams, two
 * host threads) would mix their counts: the caller serialises them.
 */
KVS_API kvs_status kvs_deviation_topk(const kvs_shape *shape, int64_t n_tokens,
                              const void *k_fresh, const void *v_fresh,
                              const void *k_cache, const void *v_cache,
                              const uint8_t *reused, const float *alpha, int32_t mode,
                              float *dev_k, float *dev_v, float *score,
                              int32_t k, int32_t *idx_out,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * kvs_select_topk -- Alg. 1 step 4: the k highest-scoring entries of each row.
 *
 * Row r of the ragged matrix is scores[row_off[r] .. row_off[r+1]).  The k_row[r] entries
 * that come first in the order (score descending, index ascending) are written as row-local
 * int32 indices, in ascending index order, at idx_out + sum(k_row[0..r)).  Scores compare as
 * real numbers (-0 equals +0); -inf entries rank last (still by index); NaN scores are a
 * caller error with unspecified (but memory-safe) results.  The result is exact and
 * deterministic.
 *
 * scores   [dev] fp32            row_off [host] int64[n_rows+1], non-decreasing
 * k_row    [host] int32[n_rows], 0 <= k_row[r] <= row length; rows longer than 2^31-1 are
 *          rejected
 * idx_out  [dev] int32[sum k_row]
 * workspace [dev] optional (NULL / 0 is valid), 256-byte aligned, kvs_workspace_size("select_topk",
 *          any valid shape, n_rows, total scores) bytes: rows longer than 49152 entries are then
 *          cut into parts of 32768 that run on workgroups of their own (four launches, 41 us
 *          instead of 105 us for 131072 entries); without it, or for a row of more than 64
 *          parts, such a row is handled by one workgroup.  The result is the same either way.
 */
KVS_API kvs_status kvs_select_topk(const float *scores, int32_t n_rows, const int64_t *row_off,
                           const int32_t *k_row, int32_t *idx_out,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * kvs_select_topk_static -- kvs_select_topk for callers that cannot allocate device memory (code
 * under stream capture, serving loops and harnesses that forbid hipMalloc): same arguments without
 * the workspace, same results.  Rows longer than 49152 scores, which kvs_select_topk spreads over
 * several workgroups only when given a workspace, here use a scratch buffer that belongs to the
 * library: a file-scope device array of 4.3 MB (each device the library runs on holds it until
 * the process ends).  The call allocates and frees nothing; on its first call on a device it asks
 * the runtime once for that device's address of the array (a call with n_rows = 0 does just
 * that and may be made ahead of time, e.g. before a stream capture begins).
 *
 * Limit: every row at most 1048576 (2^20) scores; a longer row returns KVS_EINVAL before anything
 * is launched.  All calls on one device share that device's scratch and the kernels overwrite what
 * they use before reading it, so nothing has to be cleared between calls; calls that overlap in
 * time on one device (different streams, or host threads) race on it and must be serialised by
 * the caller.
 */
KVS_API kvs_status kvs_select_topk_static(const float *scores, int32_t n_rows, const int64_t *row_off,
                                  const int32_t *k_row, int32_t *idx_out, void *stream);

/*
 * kvs_scatter_kv -- the KV Writer of App. A: recomputed K/V replace the reused entries.
 *
 *   k_cache[sel_pos[s]] = k_new[s],  v_cache[sel_pos[s]] = v_new[s]      for s in [0, n_sel)
 *   reused[sel_pos[s]] = 0           (if reused != NULL)  the token is no longer a candidate
 *   dev_v[g, sel_pos[s]] = 0         (if dev_v  != NULL)  its stored deviation is repaired
 *
 * n_rows     rows of the cache (and row stride of dev_v)
 * k_new,v_new [dev] [n_sel, n_kv_heads, head_dim]
 * sel_pos    [dev] int32[n_sel], global cache rows in [0, n_rows), all distinct (duplicates
 *            race: one of the writers wins per 16-byte piece)
 */
KVS_API kvs_status kvs_scatter_kv(const kvs_shape *shape, int64_t n_rows,
                          const void *k_new, const void *v_new,
                          const int32_t *sel_pos, int64_t n_sel,
                          void *k_cache, void *v_cache, uint8_t *reused, float *dev_v,
                          void *stream);

/*
 * kvs_partial_attention -- Eq. (1) restricted to the rows of the selected tokens (App. A:
 * only the selected tokens are computed, the others' KV is reused).
 *
 * Request b owns cache rows [ctx_off[b], ctx_off[b] + ctx_len[b]) and the selected tokens
 * [cu_sel[b], cu_sel[b+1]).  Selected token s sits at request-local position p = sel_pos[s]
 * and its query head h attends causally, by that original position, over the cache as it
 * stands (recomputed rows already scattered in):
 *
 *   out[s,h,:] = sum_{i <= p} softmax_i( scale * q_sel[s,h,:] . K[ctx_off[b]+i, g(h), :] )
 *                             * V[ctx_off[b]+i, g(h), :]
 *   lse[s,h]   = log sum_{i <= p} exp( scale * q . K_i )          (natural log; optional)
 *
 * ctx_off, ctx_len [host] int64[batch];  cu_sel [host] int64[batch+1], non-decreasing
 * q_sel   [dev] [n_sel, n_q_heads, head_dim]         sel_pos [dev] int32[n_sel], ascending
 *         within each request, each in [0, ctx_len[b])
 * out     [dev] [n_sel, n_q_heads, head_dim] in the shape's dtype
 * lse_out [dev] fp32[n_sel, n_q_heads] or NULL
 * workspace [dev] optional (NULL / 0 is valid), 256-byte aligned.  With at least
 *         kvs_workspace_size("partial_attention", ...) bytes, launches too small to fill the chip
 *         (few selected tokens over long contexts, e.g. the decode-stage recompute), and single
 *         requests whose K and V outgrow the last-level cache (above 192 MiB: then the size asked
 *         for is 528 bytes x 16 per output row), cut each row tile's key range into pieces
 *         handled by separate workgroups and merge them; results are the same up to fp32
 *         summation order.  With less, such launches keep whole key ranges.
 * bf16 inputs (head_dim 128, scale > 0) are contracted on the matrix cores with fp32 accumulation
 * and an fp32 softmax, the softmax weights entering the second product as bf16; every other case
 * takes an fp32 vector path.
 */
KVS_API kvs_status kvs_partial_attention(const kvs_shape *shape, int32_t batch,
                                 const int64_t *ctx_off, const int64_t *ctx_len,
                                 const int64_t *cu_sel,
                                 const void *q_sel, const int32_t *sel_pos,
                                 const void *k_cache, const void *v_cache, float scale,
                                 void *out, float *lse_out,
                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * kvs_decode_check -- Sec. 4.2: Alg. 1 re-run in the decode stage with alpha replaced by the
 * decoding token's current attention over the cache.
 *
 * For request b (its new token's K/V already appended, context ctx_len[b] rows):
 *   a[h,i]   = softmax_{i in [0, ctx_len[b])}( scale * q_new[b,h,:] . K[ctx_off[b]+i, g(h), :] )
 *   score[i] = sum_g ( sum_{h in group g} a[h,i] ) * dev_v[g, ctx_off[b]+i]   if reused, else -inf
 * and the k_req[b] best candidates (same order and tie rule as kvs_select_topk) are written
 * as ascending request-local indices at idx_out + sum(k_req[0..b)).
 *
 * n_rows    rows of the packed cache (row stride of dev_v, length of reused / score_out)
 * ctx_off, ctx_len [host] int64[batch]; every context lies inside [0, n_rows) and no two contexts
 *           share a cache row (KVS_EINVAL otherwise: scores and logits are kept per cache row)
 * q_new     [dev] [batch, n_q_heads, head_dim]
 * v_cache   [dev] only read when attn_out != NULL
 * dev_v     [dev] fp32[n_kv_heads, n_rows] as left by kvs_deviation / kvs_scatter_kv
 * reused    [dev] uint8[n_rows] or NULL (all candidates)
 * k_req     [host] int32[batch], 0 <= k_req[b] <= ctx_len[b]
 * score_out [dev] fp32[n_rows] or NULL; rows outside the contexts are not written
 * attn_out  [dev] [batch, n_q_heads, head_dim] (shape dtype) or NULL: sum_i a[h,i] * V_i
 * A call with one context of 12289..262144 rows selects the way kvs_deviation_topk does (keys and their
 * histogram from the scoring launch, two short selecting launches, same index list bit for bit) and, like it,
 * uses 2.1 MB of device memory that belongs to the library: such calls and kvs_deviation_topk calls on one
 * device must not overlap (one stream, or ordered by events).
 */
KVS_API kvs_status kvs_decode_check(const kvs_shape *shape, int32_t batch, int64_t n_rows,
                            const int64_t *ctx_off, const int64_t *ctx_len,
                            const void *q_new, const void *k_cache, const void *v_cache,
                            const float *dev_v, const uint8_t *reused, float scale,
                            const int32_t *k_req, int32_t *idx_out, float *score_out,
                            void *attn_out,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * kvs_attn_colsum -- Alg. 1 steps 1-2: the attention column mass of a whole prefill,
 *     alpha[g, i] = sum over the query heads h of KV head g, and over the rows j >= i, of A_h[j, i],
 *     A_h = row softmax over the keys i <= j of scale * q[j, h] . k[i, g]      (Eq. (3), causal),
 * i.e. the alpha that kvs_deviation takes.  Every row of A sums to 1, so sum_i alpha[g, i] =
 * n_tokens * n_q_heads / n_kv_heads.  The score matrix is never stored: one sweep leaves each
 * row's log-sum-exp in the workspace, a second one sums exp(score - lse) down the columns.
 * Cost: two passes of n_tokens^2 / 2 * head_dim * n_q_heads multiply-adds on the matrix cores.
 *
 * bf16 with head_dim 128 and a positive scale runs on the matrix cores (tensors below 4 GiB);
 * every other supported shape, fp32 included, takes a plain vector kernel that is only meant for
 * small problems.  Q and K as for the other calls: [n_tokens, heads, head_dim], 16-byte aligned.
 *
 * q         [dev] [n_tokens, n_q_heads, head_dim]
 * k         [dev] [n_tokens, n_kv_heads, head_dim] (the fresh keys)
 * alpha     [dev] fp32[n_kv_heads, n_tokens], written
 * workspace [dev] kvs_workspace_size("attn_colsum", shape, 1, n_tokens, 0) bytes, 256-byte
 *           aligned, required; contents on return are unspecified
 */
KVS_API kvs_status kvs_attn_colsum(const kvs_shape *shape, int64_t n_tokens, const void *q, const void *k,
                           float scale, float *alpha,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * kvs_first_order_impact -- Sec. 4.1, Eq. (2): the first-order expansion of the attention output's
 * deviation, dH ~ (dH/dK) dK + (dH/dV) dV, rated token by token.  With H = A V the correct (fresh,
 * causal) attention, dK = k_cache - k_fresh and dV = v_cache - v_fresh, reusing token i's cache
 * entry moves output row j >= i of query head h (KV head g) by
 *     A[h,j,i] * dV[g,i]  +  A[h,j,i] * scale * (q[j,h] . dK[g,i]) * (V[g,i] - H[h,j])
 * (value direction: dH/dV = A; key direction: the softmax Jacobian), and
 *     impact_v[i]  = sum over h, j of the L1 norm of the first term  (= Eq. (3): alpha * |dV|_1)
 *     impact_k[i]  = ... of the second term
 *     impact_kv[i] = ... of their sum
 * with -inf where reused[i] == 0.  The key direction is what the paper leaves out of Alg. 1 to save
 * work (it costs n_tokens^2 / 2 * n_q_heads * head_dim vector operations and is no matrix product);
 * this call exists to rank by it on check layers and to compare the two rankings (App. D.2).
 *
 * q        [dev] [n_tokens, n_q_heads, head_dim]
 * h_fresh  [dev] [n_tokens, n_q_heads, head_dim] (shape dtype): the causal attention of every row over
 *          the fresh K/V, e.g. from kvs_partial_attention with every token selected
 * lse      [dev] fp32[n_tokens, n_q_heads]: that attention's log-sum-exp (natural log), same call
 * reused   [dev] uint8[n_tokens] or NULL (every token is rated)
 * impact_* [dev] fp32[n_tokens], each may be NULL
 * workspace [dev] kvs_workspace_size("first_order_impact", shape, 1, n_tokens, 0) bytes, 256-byte aligned
 * All arithmetic is fp32 on exactly widened inputs in a fixed order (bit-reproducible); up to 2^20 tokens.
 */
KVS_API kvs_status kvs_first_order_impact(const kvs_shape *shape, int64_t n_tokens, const void *q,
                                  const void *k_fresh, const void *v_fresh,
                                  const void *k_cache, const void *v_cache,
                                  const void *h_fresh, const float *lse,
                                  const uint8_t *reused, float scale,
                                  float *impact_v, float *impact_k, float *impact_kv,
                                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * Token-sequence matching of the KV Retriever (Sec. 5.1; App. E Alg. 3 with the polynomial window
 * hash of Eq. (7)): which tokens of a new request (the target) also stand, in stretches that start
 * with a whole window of `window` equal-hash tokens, in an earlier request (the candidate), and where.
 * The result is the one the algorithm's sequential scan produces: a target position is matched once,
 * by the first pair of window starts (candidate window ascending, then target window ascending)
 * whose stretch of equal tokens reaches it; windows are compared by hash only, then token by
 * token, so two different windows with one hash contribute the equal tokens they begin with.
 * The paper names neither the base, the modulus nor the window: all three are arguments.
 *
 * target, candidate [dev] int32 token ids, non-negative (an id is hashed as an unsigned 32-bit number)
 * window            > 0; sequences shorter than the window match nothing
 * hash_base         b of Eq. (7), any 32-bit value
 * hash_modulus      m of Eq. (7), 1 .. 2^32-1
 * match_cand        [dev] int32[n_target] out: candidate position matched to each target position, -1: none
 * target_matches, candidate_matches
 *                   [dev] int32[n_target] out, each may be NULL: the matched pairs in the algorithm's
 *                   order of discovery (its two output lists); entries from *n_matches on are not written
 * n_matches         [dev] int64 out: number of matched target positions (hit rate = n_matches / n_target)
 * workspace         [dev] kvs_workspace_size("match_tokens", NULL, 1, n_target, n_candidate) bytes,
 *                   256-byte aligned (not needed when a sequence is shorter than the window)
 * Up to 2^26 tokens per sequence.  Integer work: the outputs are exact and do not depend on the
 * order in which the device's atomics arrive.  Six launches, no host synchronisation.  Cost grows
 * with the matched tokens, except for degenerate inputs (one token repeated throughout both
 * sequences makes every pair of windows a candidate: n_target x n_candidate steps).
 * Several earlier requests are matched in one call by concatenating them into one candidate with a token id
 * that occurs nowhere else between them (no window then spans two requests); partners index the concatenation.
 * The scheduler of Sec. 4.3 Alg. 2 needs no call of its own: the batch it sends on is
 * kvs_select_topk over the requests' hit rates (ties to the request that arrived first).
 */
KVS_API kvs_status kvs_match_tokens(const int32_t *target, int64_t n_target,
                                    const int32_t *candidate, int64_t n_candidate,
                                    int32_t window, uint32_t hash_base, uint32_t hash_modulus,
                                    int32_t *match_cand, int32_t *target_matches, int32_t *candidate_matches,
                                    int64_t *n_matches, void *workspace, size_t workspace_bytes, void *stream);

/*
 * A later layer's Q, K and V of the selected tokens (App. D.1: the tokens picked in an early layer are
 * the ones recomputed in the layers after it; their index list is simply passed on to this call,
 * kvs_scatter_kv and kvs_partial_attention of those layers).  Recomputing a token in a layer starts with
 * the layer's projection of its hidden state:
 *     y[m, f] = sum_c x[x_rows[m], c] * w_qkv[f, c],   f over (n_q_heads + 2 n_kv_heads) * head_dim features
 * in the order all Q heads, all K heads, all V heads.  With a rotary table, channel pair
 * (c, c + head_dim/2) of every Q and K head is turned by the table's angle for position sel_pos[m]:
 *     out[c] = y[c] cos - y[c + head_dim/2] sin,   out[c + head_dim/2] = y[c + head_dim/2] cos + y[c] sin
 * (the convention of the Llama / Qwen / Yi families the paper evaluates; the paper itself takes Q, K, V
 * as given).  One launch: gather, bf16 matrix product with fp32 accumulation, rotation in fp32, one
 * rounding to bf16 on the way out.
 *
 * x        [dev] bf16 [n_tokens, hidden] hidden states
 * x_rows   [dev] int32[n_sel] row of x for each selected token, or NULL (row m of x is selected token m:
 *          from the second recomputed layer on only the selected tokens have hidden states)
 * sel_pos  [dev] int32[n_sel] positions of the selected tokens (read only with a rotary table)
 * w_qkv    [dev] bf16 [(n_q_heads + 2 n_kv_heads) * head_dim, hidden], one row per output feature
 * rope     [dev] fp32 [rope_positions, head_dim/2, 2] = (cos, sin) per position and channel pair, or NULL
 * q_out    [dev] bf16 [n_sel, n_q_heads, head_dim]; k_out, v_out [dev] bf16 [n_sel, n_kv_heads, head_dim]:
 *          the layouts kvs_partial_attention and kvs_scatter_kv take
 * Built for bf16, head_dim 128, hidden a multiple of 64, an even number of heads in all, x and w below
 * 4 GiB each, a rotary table below 4 GiB (KVS_EUNSUPPORTED otherwise).  Tensors 16-byte aligned.  No workspace.  Row indices and
 * positions outside their ranges are clamped (memory safety only).
 */
KVS_API kvs_status kvs_project_qkv(const kvs_shape *shape, int32_t hidden, const void *x, int64_t n_tokens,
                                   const int32_t *x_rows, const int32_t *sel_pos, int64_t n_sel,
                                   const void *w_qkv, const float *rope, int64_t rope_positions,
                                   void *q_out, void *k_out, void *v_out, void *stream);

/*
 * Workspace a call needs, in bytes, for the given problem.  `call` is "select_topk",
 * "partial_attention", "decode_check", "attn_colsum", "first_order_impact" or "match_tokens" (anything else
 * returns 0).  n_rows_total is the total number of score / cache rows the call will see (match_tokens: the
 * target's tokens), n_sel_total the total number of selected tokens (partial_attention) or the candidate's
 * tokens (match_tokens, which ignores shape: it may be NULL there).  The answer is an upper bound valid for any split of the
 * totals over `batch` requests.
 */
KVS_API size_t kvs_workspace_size(const char *call, const kvs_shape *shape, int32_t batch,
                          int64_t n_rows_total, int64_t n_sel_total);

KVS_API const char *kvs_strerror(kvs_status status);
KVS_API const char *kvs_last_error(void);

/* Library build identification: "kvshare-hip gfx950 <n>" */
KVS_API const char *kvs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVS_H */
