/*
 * kvso.c -- CPU ORACLE for the DHD (Dual-Stage High Deviation) KV-reuse hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU library is
 * checked against.  It is called from tests, from the smoke check and from the benchmark's
 * cpu_baseline leg; the product path never routes through it.  It shares no code, header,
 * table or helper with the HIP sources.
 *
 * Every function follows the paper's own statement of the operation:
 *   kvso_deviation         Alg. 1 input "deviation matrix Delta V" and step 3; Eq. (3)
 *   kvso_alpha_prefill     Alg. 1 steps 1-2 (A = Softmax(QK^T/sqrt(d_k)), alpha = ColSum(A))
 *   kvso_select_topk       Alg. 1 step 4 (top-r% by Score)
 *   kvso_scatter_kv        the "KV Writer" of App. A: recomputed K/V replace reused entries
 *   kvso_partial_attention Eq. (1) restricted to the rows of the selected tokens (App. A:
 *                          only the selected tokens are computed, the others' KV is reused)
 *   kvso_decode_check      Sec. 4.2: Alg. 1 with alpha taken from the decoding token's
 *                          current attention over the cache
 *   kvso_first_order_impact Sec. 4.1, Eq. (2): the first-order expansion of the attention output's
 *                          deviation, token by token, in the value direction, the key direction
 *                          and both together
 *   kvso_exact_impact      Sec. 4.1 / App. D.2 "ideal index": the true change of the attention
 *                          output when one token's K/V alone is the reused one
 *   kvso_window_hash       App. E Eq. (7): polynomial hash of every window of a token sequence
 *   kvso_match_tokens      App. E Alg. 3: token-sequence matching over a hash index of the
 *                          target's windows, candidate windows in ascending order, matches
 *                          extended token by token, a target position matched at most once
 *   kvso_project_qkv       App. D.1 (the tokens selected in an early layer are the ones recomputed in
 *                          the later layers): a later layer's Q/K/V of the selected tokens, i.e. its
 *                          projection of their hidden states, with the rotary position factors of
 *                          the models the paper evaluates applied to Q and K
 *   kvso_schedule          Sec. 4.3 Alg. 2: the queue sorted by cache hit rate, descending; the
 *                          first N requests form the next batch
 *
 * Arithmetic: inputs are converted exactly to double (bf16 and fp32 are both subsets of
 * double), every sum and product is carried in double in the natural index order, and a result
 * is rounded once when it is stored as fp32.  No blocking, no fusion, no reordering.
 *
 * Layouts (all row-major, contiguous):
 *   K, V            [rows, n_kv_heads, head_dim]      dtype of the shape (fp32 or bf16 bits)
 *   Q               [rows, n_q_heads,  head_dim]
 *   dev_k, dev_v    [n_kv_heads, rows] fp32
 *   alpha           [n_kv_heads, rows] fp32 (column mass summed over the query heads that
 *                   share the KV head)
 *   score           [rows] fp32, -inf where the token is not a candidate
 * Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *
 * Return value: 0 on success, 1 on an invalid argument.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { KVSO_F32 = 0, KVSO_BF16 = 1 };
enum { KVSO_SCORE_V = 0, KVSO_SCORE_KV = 1 };

typedef struct {
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t dtype;
} kvso_shape;

static int shape_ok(const kvso_shape *s)
{
    if (!s) return 0;
    if (s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->head_dim <= 0) return 0;
    if (s->n_q_heads % s->n_kv_heads != 0) return 0;
    if (s->dtype != KVSO_F32 && s->dtype != KVSO_BF16) return 0;
    return 1;
}

/* exact widening load of element i */
static double ld(const void *p, int dtype, int64_t i)
{
    if (dtype == KVSO_F32) return (double)((const float *)p)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static size_t elem_size(int dtype) { return dtype == KVSO_F32 ? 4 : 2; }

/* ---------------------------------------------------------------------------------------
 * Deviation and score.  dev[g,i] = sum_c |fresh[i,g,c] - cache[i,g,c]|  (L1 norm of the
 * token's deviation on KV head g).  score_i = sum_g alpha[g,i] * dev_v[g,i]   (mode V, the
 * paper's Eq. (3) carried per head and summed), or with dev_k+dev_v in place of dev_v
 * (mode KV).  alpha == NULL means alpha = 1 (pure magnitude ranking).  Tokens with
 * reused[i] == 0 are not candidates and get score -inf; reused == NULL means all are.
 * ------------------------------------------------------------------------------------- */
int kvso_deviation(const kvso_shape *sh, int64_t n,
                   const void *k_fresh, const void *v_fresh,
                   const void *k_cache, const void *v_cache,
                   const uint8_t *reused, const float *alpha, int mode,
                   float *dev_k, float *dev_v, float *score)
{
    if (!shape_ok(sh) || n < 0 || !v_fresh || !v_cache) return 1;
    if (mode != KVSO_SCORE_V && mode != KVSO_SCORE_KV) return 1;
    int need_k = (mode == KVSO_SCORE_KV) || dev_k;
    if (need_k && (!k_fresh || !k_cache)) return 1;
    const int hk = sh->n_kv_heads, d = sh->head_dim, dt = sh->dtype;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double sc = 0.0;
        for (int g = 0; g < hk; ++g) {
            int64_t base = (i * hk + g) * (int64_t)d;
            double dv = 0.0, dk = 0.0;
            for (int c = 0; c < d; ++c)
                dv += fabs(ld(v_fresh, dt, base + c) - ld(v_cache, dt, base + c));
            if (need_k)
                for (int c = 0; c < d; ++c)
                    dk += fabs(ld(k_fresh, dt, base + c) - ld(k_cache, dt, base + c));
            if (dev_v) dev_v[(int64_t)g * n + i] = (float)dv;
            if (dev_k) dev_k[(int64_t)g * n + i] = (float)dk;
            double a = alpha ? (double)alpha[(int64_t)g * n + i] : 1.0;
            sc += a * (mode == KVSO_SCORE_KV ? dk + dv : dv);
        }
        if (score) score[i] = (!reused || reused[i]) ? (float)sc : -INFINITY;
    }
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * Prefill attention column mass.  For query head h and query row j the attention row is the
 * causal softmax over keys i <= j of scale * q[j,h] . k[i,g(h)].  alpha_h[h,i] is the sum of
 * column i over all rows j >= i; alpha_g[g,i] sums alpha_h over the heads of group g.
 * Two passes, each a direct transcription: (1) every row's max and normaliser, (2) every
 * column's sum of normalised weights.
 * alpha_h [n_q_heads, n] and alpha_g [n_kv_heads, n] are double; either may be NULL.
 * ------------------------------------------------------------------------------------- */
int kvso_alpha_prefill(const kvso_shape *sh, int64_t n, const void *q, const void *k,
                       double scale, double *alpha_h, double *alpha_g)
{
    if (!shape_ok(sh) || n < 0 || !q || !k) return 1;
    const int hq = sh->n_q_heads, hk = sh->n_kv_heads, d = sh->head_dim, dt = sh->dtype;
    const int grp = hq / hk;
    if (n == 0) return 0;
    double *row_max = malloc(sizeof(double) * (size_t)hq * n);
    double *row_sum = malloc(sizeof(double) * (size_t)hq * n);
    double *ah = alpha_h ? alpha_h : malloc(sizeof(double) * (size_t)hq * n);
    double *qd = malloc(sizeof(double) * (size_t)n * hq * d);
    double *kd = malloc(sizeof(double) * (size_t)n * hk * d);
    if (!row_max || !row_sum || !ah || !qd || !kd) return 1;
    for (int64_t e = 0; e < n * hq * d; ++e) qd[e] = ld(q, dt, e);
    for (int64_t e = 0; e < n * hk * d; ++e) kd[e] = ld(k, dt, e);

#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (int h = 0; h < hq; ++h) {
        for (int64_t j = 0; j < n; ++j) {
            const double *qv = qd + (j * hq + h) * (int64_t)d;
            const int g = h / grp;
            double m = -INFINITY;
            for (int64_t i = 0; i <= j; ++i) {
                const double *kv = kd + (i * hk + g) * (int64_t)d;
                double s = 0.0;
                for (int c = 0; c < d; ++c) s += qv[c] * kv[c];
                s *= scale;
                if (s > m) m = s;
            }
            double z = 0.0;
            for (int64_t i = 0; i <= j; ++i) {
                const double *kv = kd + (i * hk + g) * (int64_t)d;
                double s = 0.0;
                for (int c = 0; c < d; ++c) s += qv[c] * kv[c];
                z += exp(s * scale - m);
            }
            row_max[(int64_t)h * n + j] = m;
            row_sum[(int64_t)h * n + j] = z;
        }
    }
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (int h = 0; h < hq; ++h) {
        for (int64_t i = 0; i < n; ++i) {
            const int g = h / grp;
            const double *kv = kd + (i * hk + g) * (int64_t)d;
            double col = 0.0;
            for (int64_t j = i; j < n; ++j) {
                const double *qv = qd + (j * hq + h) * (int64_t)d;
                double s = 0.0;
                for (int c = 0; c < d; ++c) s += qv[c] * kv[c];
                col += exp(s * scale - row_max[(int64_t)h * n + j]) / row_sum[(int64_t)h * n + j];
            }
            ah[(int64_t)h * n + i] = col;
        }
    }
    if (alpha_g) {
        for (int g = 0; g < hk; ++g)
            for (int64_t i = 0; i < n; ++i) {
                double s = 0.0;
                for (int h = g * grp; h < (g + 1) * grp; ++h) s += ah[(int64_t)h * n + i];
                alpha_g[(int64_t)g * n + i] = s;
            }
    }
    free(row_max); free(row_sum); free(qd); free(kd);
    if (!alpha_h) free(ah);
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * Top-k selection.  Row r of the ragged score matrix is scores[row_off[r] .. row_off[r+1]).
 * The k_row[r] entries that come first in the order (score descending, index ascending) are
 * selected and written, as row-local indices in ascending order, at idx_out + sum(k_row[:r]).
 * Scores compare as real numbers (-0 == +0); -inf entries rank last; NaN is an error.
 * ------------------------------------------------------------------------------------- */
static const float *g_sort_scores; /* comparator context; select is not re-entrant */
#pragma omp threadprivate(g_sort_scores)

static int cmp_rank(const void *a, const void *b)
{
    int32_t ia = *(const int32_t *)a, ib = *(const int32_t *)b;
    float sa = g_sort_scores[ia], sb = g_sort_scores[ib];
    if (sa > sb) return -1;
    if (sa < sb) return 1;
    return (ia > ib) - (ia < ib);
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t ia = *(const int32_t *)a, ib = *(const int32_t *)b;
    return (ia > ib) - (ia < ib);
}

int kvso_select_topk(const float *scores, int32_t n_rows, const int64_t *row_off,
                     const int32_t *k_row, int32_t *idx_out)
{
    if (n_rows < 0 || (n_rows > 0 && (!scores || !row_off || !k_row))) return 1;
    int64_t *out_off = malloc(sizeof(int64_t) * ((size_t)n_rows + 1));
    if (!out_off) return 1;
    out_off[0] = 0;
    for (int32_t r = 0; r < n_rows; ++r) {
        int64_t len = row_off[r + 1] - row_off[r];
        if (len < 0 || len > INT32_MAX || k_row[r] < 0 || k_row[r] > len) { free(out_off); return 1; }
        out_off[r + 1] = out_off[r] + k_row[r];
    }
    if (out_off[n_rows] > 0 && !idx_out) { free(out_off); return 1; }
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : bad)
    for (int32_t r = 0; r < n_rows; ++r) {
        const float *row = scores + row_off[r];
        int64_t len = row_off[r + 1] - row_off[r];
        int32_t k = k_row[r];
        for (int64_t i = 0; i < len; ++i)
            if (isnan(row[i])) bad = 1;
        if (k == 0 || bad) continue;
        int32_t *order = malloc(sizeof(int32_t) * (size_t)len);
        for (int64_t i = 0; i < len; ++i) order[i] = (int32_t)i;
        g_sort_scores = row;
        qsort(order, (size_t)len, sizeof(int32_t), cmp_rank);
        qsort(order, (size_t)k, sizeof(int32_t), cmp_i32);
        memcpy(idx_out + out_off[r], order, sizeof(int32_t) * (size_t)k);
        free(order);
    }
    free(out_off);
    return bad;
}

/* ---------------------------------------------------------------------------------------
 * KV write-back.  For s in [0, n_sel): row sel_pos[s] of the cache takes row s of the
 * recomputed K/V; the token stops being a reuse candidate (reused cleared, stored deviation
 * zeroed).  sel_pos holds global row numbers of the packed cache, all distinct.
 * ------------------------------------------------------------------------------------- */
int kvso_scatter_kv(const kvso_shape *sh, int64_t n_rows,
                    const void *k_new, const void *v_new, const int32_t *sel_pos, int64_t n_sel,
                    void *k_cache, void *v_cache, uint8_t *reused, float *dev_v)
{
    if (!shape_ok(sh) || n_rows < 0 || n_sel < 0) return 1;
    if (n_sel > 0 && (!k_new || !v_new || !sel_pos || !k_cache || !v_cache)) return 1;
    const size_t row_bytes = (size_t)sh->n_kv_heads * sh->head_dim * elem_size(sh->dtype);
    for (int64_t s = 0; s < n_sel; ++s)
        if (sel_pos[s] < 0 || sel_pos[s] >= n_rows) return 1;
    for (int64_t s = 0; s < n_sel; ++s) {
        int64_t p = sel_pos[s];
        memcpy((char *)k_cache + p * row_bytes, (const char *)k_new + s * row_bytes, row_bytes);
        memcpy((char *)v_cache + p * row_bytes, (const char *)v_new + s * row_bytes, row_bytes);
        if (reused) reused[p] = 0;
        if (dev_v)
            for (int g = 0; g < sh->n_kv_heads; ++g) dev_v[(int64_t)g * n_rows + p] = 0.0f;
    }
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * Partial-recompute attention.  Request b owns cache rows ctx_off[b] .. ctx_off[b]+ctx_len[b])
 * and the selected tokens cu_sel[b] .. cu_sel[b+1]).  Selected token s sits at request-local
 * position p = sel_pos[s]; its query head h attends causally over keys 0..p of its request:
 *     o[s,h] = sum_{i<=p} softmax_i( scale * q[s,h] . K[i,g(h)] ) * V[i,g(h)]
 * on the cache as it stands (the caller has already blended recomputed rows in).
 * out [n_sel, n_q_heads, head_dim] double; lse [n_sel, n_q_heads] double (natural-log
 * sum-exp of the scaled logits), may be NULL.
 * ------------------------------------------------------------------------------------- */
int kvso_partial_attention(const kvso_shape *sh, int32_t batch,
                           const int64_t *ctx_off, const int64_t *ctx_len, const int64_t *cu_sel,
                           const void *q_sel, const int32_t *sel_pos,
                           const void *k_cache, const void *v_cache, double scale,
                           double *out, double *lse)
{
    if (!shape_ok(sh) || batch < 0) return 1;
    if (batch > 0 && (!ctx_off || !ctx_len || !cu_sel)) return 1;
    const int hq = sh->n_q_heads, hk = sh->n_kv_heads, d = sh->head_dim, dt = sh->dtype;
    const int grp = hq / hk;
    for (int32_t b = 0; b < batch; ++b) {
        if (cu_sel[b + 1] < cu_sel[b] || ctx_len[b] < 0 || ctx_off[b] < 0) return 1;
        for (int64_t s = cu_sel[b]; s < cu_sel[b + 1]; ++s)
            if (sel_pos[s] < 0 || sel_pos[s] >= ctx_len[b]) return 1;
    }
    if (batch > 0 && cu_sel[batch] > 0 && (!q_sel || !sel_pos || !k_cache || !v_cache || !out)) return 1;
    for (int32_t b = 0; b < batch; ++b) {
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
        for (int64_t s = cu_sel[b]; s < cu_sel[b + 1]; ++s) {
            for (int h = 0; h < hq; ++h) {
                const int g = h / grp;
                const int64_t p = sel_pos[s];
                const int64_t qb = (s * hq + h) * (int64_t)d;
                double *logit = malloc(sizeof(double) * (size_t)(p + 1));
                double m = -INFINITY;
                for (int64_t i = 0; i <= p; ++i) {
                    int64_t kb = ((ctx_off[b] + i) * hk + g) * (int64_t)d;
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c) acc += ld(q_sel, dt, qb + c) * ld(k_cache, dt, kb + c);
                    logit[i] = acc * scale;
                    if (logit[i] > m) m = logit[i];
                }
                double z = 0.0;
                for (int64_t i = 0; i <= p; ++i) { logit[i] = exp(logit[i] - m); z += logit[i]; }
                double *o = out + (s * hq + h) * (int64_t)d;
                for (int c = 0; c < d; ++c) o[c] = 0.0;
                for (int64_t i = 0; i <= p; ++i) {
                    int64_t vb = ((ctx_off[b] + i) * hk + g) * (int64_t)d;
                    double w = logit[i] / z;
                    for (int c = 0; c < d; ++c) o[c] += w * ld(v_cache, dt, vb + c);
                }
                if (lse) lse[s * hq + h] = m + log(z);
                free(logit);
            }
        }
    }
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * Decode-stage check.  The new token of request b (its K/V already appended, so the context
 * is ctx_len[b] rows long) attends over its whole context:
 *     a[h,i] = softmax_{i in [0,L)}( scale * q[b,h] . K[i,g(h)] )
 * and the reuse candidates are re-scored with that attention in place of the prefill column
 * mass:  score_i = sum_g ( sum_{h in g} a[h,i] ) * dev_v[g,i]   if reused[i], else -inf.
 * The k_req[b] best candidates (same order as kvso_select_topk, decided on the fp32-rounded
 * scores) are returned as ascending request-local indices, packed request after request.
 * dev_v [n_kv_heads, n_rows] and reused [n_rows] are indexed by global cache row.
 * score_out [n_rows] fp32 (only the rows of the batch's contexts are written) and
 * attn_out [batch, n_q_heads, head_dim] double (the decode attention output) may be NULL.
 * ------------------------------------------------------------------------------------- */
int kvso_decode_check(const kvso_shape *sh, int32_t batch, int64_t n_rows,
                      const int64_t *ctx_off, const int64_t *ctx_len,
                      const void *q_new, const void *k_cache, const void *v_cache,
                      const float *dev_v, const uint8_t *reused, double scale,
                      const int32_t *k_req, int32_t *idx_out, float *score_out, double *attn_out)
{
    if (!shape_ok(sh) || batch < 0 || n_rows < 0) return 1;
    if (batch > 0 && (!ctx_off || !ctx_len || !q_new || !k_cache || !dev_v || !k_req)) return 1;
    if (attn_out && !v_cache) return 1;
    const int hq = sh->n_q_heads, hk = sh->n_kv_heads, d = sh->head_dim, dt = sh->dtype;
    const int grp = hq / hk;
    int64_t out_base = 0;
    for (int32_t b = 0; b < batch; ++b) {
        const int64_t L = ctx_len[b], off = ctx_off[b];
        if (L < 0 || off < 0 || off + L > n_rows || k_req[b] < 0 || k_req[b] > L) return 1;
        double *a = malloc(sizeof(double) * (size_t)hq * (size_t)(L > 0 ? L : 1));
        float *sc = malloc(sizeof(float) * (size_t)(L > 0 ? L : 1));
        if (!a || !sc) return 1;
#pragma omp parallel for schedule(dynamic, 1)
        for (int h = 0; h < hq; ++h) {
            const int g = h / grp;
            double *ah = a + (int64_t)h * L;
            double m = -INFINITY;
            for (int64_t i = 0; i < L; ++i) {
                int64_t kb = ((off + i) * hk + g) * (int64_t)d;
                double acc = 0.0;
                for (int c = 0; c < d; ++c)
                    acc += ld(q_new, dt, ((int64_t)b * hq + h) * d + c) * ld(k_cache, dt, kb + c);
                ah[i] = acc * scale;
                if (ah[i] > m) m = ah[i];
            }
            double z = 0.0;
            for (int64_t i = 0; i < L; ++i) { ah[i] = exp(ah[i] - m); z += ah[i]; }
            for (int64_t i = 0; i < L; ++i) ah[i] /= z;
            if (attn_out) {
                double *o = attn_out + ((int64_t)b * hq + h) * d;
                for (int c = 0; c < d; ++c) o[c] = 0.0;
                for (int64_t i = 0; i < L; ++i) {
                    int64_t vb = ((off + i) * hk + g) * (int64_t)d;
                    for (int c = 0; c < d; ++c) o[c] += ah[i] * ld(v_cache, dt, vb + c);
                }
            }
        }
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < L; ++i) {
            double s = 0.0;
            for (int g = 0; g < hk; ++g) {
                double mass = 0.0;
                for (int h = g * grp; h < (g + 1) * grp; ++h) mass += a[(int64_t)h * L + i];
                s += mass * (double)dev_v[(int64_t)g * n_rows + off + i];
            }
            sc[i] = (!reused || reused[off + i]) ? (float)s : -INFINITY;
        }
        if (score_out && L > 0) memcpy(score_out + off, sc, sizeof(float) * (size_t)L);
        int64_t ro[2] = {0, L};
        int32_t kk = k_req[b];
        int rc = kvso_select_topk(sc, 1, ro, &kk, idx_out ? idx_out + out_base : NULL);
        free(a); free(sc);
        if (rc) return rc;
        out_base += kk;
    }
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * Full (fresh) causal attention of every row, helper of the two impact functions below:
 * A[h][j][i] for i <= j (row softmax of scale * q[j,h] . k[i,g(h)]) and H[h][j][:] = sum_i A V.
 * A is stored dense [hq][n][n] (zeros above the diagonal), so this is for small n only.
 * ------------------------------------------------------------------------------------- */
static int dense_attention(const kvso_shape *sh, int64_t n, const void *q, const void *k, const void *v,
                           double scale, double *A, double *H)
{
    const int hq = sh->n_q_heads, hk = sh->n_kv_heads, d = sh->head_dim, dt = sh->dtype;
    const int grp = hq / hk;
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
    for (int h = 0; h < hq; ++h) {
        for (int64_t j = 0; j < n; ++j) {
            const int g = h / grp;
            double *a = A + ((int64_t)h * n + j) * n;
            double m = -INFINITY;
            for (int64_t i = 0; i <= j; ++i) {
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += ld(q, dt, (j * hq + h) * (int64_t)d + c) * ld(k, dt, (i * hk + g) * (int64_t)d + c);
                a[i] = acc * scale;
                if (a[i] > m) m = a[i];
            }
            double z = 0.0;
            for (int64_t i = 0; i <= j; ++i) { a[i] = exp(a[i] - m); z += a[i]; }
            for (int64_t i = 0; i <= j; ++i) a[i] /= z;
            for (int64_t i = j + 1; i < n; ++i) a[i] = 0.0;
            double *o = H + ((int64_t)h * n + j) * d;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            for (int64_t i = 0; i <= j; ++i)
                for (int c = 0; c < d; ++c) o[c] += a[i] * ld(v, dt, (i * hk + g) * (int64_t)d + c);
        }
    }
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * First-order impact of each reused token on the attention output (Sec. 4.1, Eq. (2)).
 * H = A V is the correct attention (fresh K, V; causal); reusing token i's cache entry means
 * K_i -> K_i + dK_i, V_i -> V_i + dV_i with dK = K_cache - K_fresh, dV = V_cache - V_fresh.
 * To first order the output row j of query head h (KV head g) moves by
 *     value direction   A[h,j,i] * dV[g,i]                                     (dH/dV = A)
 *     key direction     A[h,j,i] * scale * (q[j,h] . dK[g,i]) * (V[g,i] - H[h,j])
 * (the second line is the softmax Jacobian: d A[j,m] = A[j,m] (delta_mi - A[j,i]) d s[j,i],
 * summed against V).  The impact of token i is the L1 norm of that movement over all rows j >= i,
 * all query heads and all channels:
 *     impact_v[i]  = sum_h sum_j | value term |_1   = sum_g alpha[g,i] * |dV[g,i]|_1   (Eq. (3))
 *     impact_k[i]  = sum_h sum_j | key term |_1
 *     impact_kv[i] = sum_h sum_j | value term + key term |_1
 * Tokens with reused[i] == 0 get -inf in all three (reused == NULL: every token is rated).
 * Each output is fp32 [n] and may be NULL.  O(n^2) memory: small n only.
 * ------------------------------------------------------------------------------------- */
int kvso_first_order_impact(const kvso_shape *sh, int64_t n, const void *q,
                            const void *k_fresh, const void *v_fresh,
                            const void *k_cache, const void *v_cache,
                            const uint8_t *reused, double scale,
                            float *impact_v, float *impact_k, float *impact_kv)
{
    if (!shape_ok(sh) || n < 0) return 1;
    if (n == 0) return 0;
    if (!q || !k_fresh || !v_fresh || !k_cache || !v_cache) return 1;
    const int hq = sh->n_q_heads, hk = sh->n_kv_heads, d = sh->head_dim, dt = sh->dtype;
    const int grp = hq / hk;
    double *A = malloc(sizeof(double) * (size_t)hq * n * n);
    double *H = malloc(sizeof(double) * (size_t)hq * n * d);
    if (!A || !H) { free(A); free(H); return 1; }
    dense_attention(sh, n, q, k_fresh, v_fresh, scale, A, H);
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < n; ++i) {
        double sv = 0.0, sk = 0.0, skv = 0.0;
        for (int h = 0; h < hq; ++h) {
            const int g = h / grp;
            const int64_t cell = (i * hk + g) * (int64_t)d;
            for (int64_t j = i; j < n; ++j) {
                const double a = A[((int64_t)h * n + j) * n + i];
                double ds = 0.0;
                for (int c = 0; c < d; ++c)
                    ds += ld(q, dt, (j * hq + h) * (int64_t)d + c) * (ld(k_cache, dt, cell + c) - ld(k_fresh, dt, cell + c));
                ds *= scale;
                const double *hj = H + ((int64_t)h * n + j) * d;
                for (int c = 0; c < d; ++c) {
                    const double dv = ld(v_cache, dt, cell + c) - ld(v_fresh, dt, cell + c);
                    const double tv = a * dv;
                    const double tk = a * ds * (ld(v_fresh, dt, cell + c) - hj[c]);
                    sv += fabs(tv);
                    sk += fabs(tk);
                    skv += fabs(tv + tk);
                }
            }
        }
        const int cand = !reused || reused[i];
        if (impact_v) impact_v[i] = cand ? (float)sv : -INFINITY;
        if (impact_k) impact_k[i] = cand ? (float)sk : -INFINITY;
        if (impact_kv) impact_kv[i] = cand ? (float)skv : -INFINITY;
    }
    free(A); free(H);
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * Exact impact of each reused token (the "ideal index" of Sec. 4.1 / App. D.2): the attention
 * is recomputed with token i's K and V taken from the cache and every other token fresh, and
 *     impact[i] = sum_h sum_j | H_i'[h,j] - H[h,j] |_1
 * is the true change of the output that reusing token i alone causes (no linearisation).
 * Tokens with reused[i] == 0 get -inf.  O(n^3 d) time: tiny n only.
 * ------------------------------------------------------------------------------------- */
int kvso_exact_impact(const kvso_shape *sh, int64_t n, const void *q,
                      const void *k_fresh, const void *v_fresh,
                      const void *k_cache, const void *v_cache,
                      const uint8_t *reused, double scale, float *impact)
{
    if (!shape_ok(sh) || n < 0) return 1;
    if (n == 0) return 0;
    if (!q || !k_fresh || !v_fresh || !k_cache || !v_cache || !impact) return 1;
    const int hq = sh->n_q_heads, hk = sh->n_kv_heads, d = sh->head_dim, dt = sh->dtype;
    const int grp = hq / hk;
    double *A = malloc(sizeof(double) * (size_t)hq * n * n);
    double *H = malloc(sizeof(double) * (size_t)hq * n * d);
    if (!A || !H) { free(A); free(H); return 1; }
    dense_attention(sh, n, q, k_fresh, v_fresh, scale, A, H);
    free(A);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n; ++i) {
        if (reused && !reused[i]) { impact[i] = -INFINITY; continue; }
        double total = 0.0;
        double *logit = malloc(sizeof(double) * (size_t)n);
        double *o = malloc(sizeof(double) * (size_t)d);
        for (int h = 0; h < hq; ++h) {
            const int g = h / grp;
            for (int64_t j = i; j < n; ++j) {           /* rows before i do not see token i */
                double m = -INFINITY;
                for (int64_t t = 0; t <= j; ++t) {
                    const void *kk = t == i ? k_cache : k_fresh;
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c) acc += ld(q, dt, (j * hq + h) * (int64_t)d + c) * ld(kk, dt, (t * hk + g) * (int64_t)d + c);
                    logit[t] = acc * scale;
                    if (logit[t] > m) m = logit[t];
                }
                double z = 0.0;
                for (int64_t t = 0; t <= j; ++t) { logit[t] = exp(logit[t] - m); z += logit[t]; }
                for (int c = 0; c < d; ++c) o[c] = 0.0;
                for (int64_t t = 0; t <= j; ++t) {
                    const void *vv = t == i ? v_cache : v_fresh;
                    const double wgt = logit[t] / z;
                    for (int c = 0; c < d; ++c) o[c] += wgt * ld(vv, dt, (t * hk + g) * (int64_t)d + c);
                }
                const double *hj = H + ((int64_t)h * n + j) * d;
                for (int c = 0; c < d; ++c) total += fabs(o[c] - hj[c]);
            }
        }
        impact[i] = (float)total;
        free(logit); free(o);
    }
    free(H);
    return 0;
}

/* ---------------------------------------------------------------------------------------------
 * App. E, Eq. (7): H = (t_0 b^(w-1) + t_1 b^(w-2) + ... + t_(w-1) b^0) mod m for the window of w
 * tokens that starts at every position i <= n - w.  The paper names neither b nor m: both are
 * arguments (2 <= m < 2^32 or m = 1, b < 2^32).  Tokens are non-negative.  Every window is
 * evaluated from its own definition (Horner over its w tokens): nothing rolls.
 * hash_out: [n - w + 1] (nothing is written when n < w).
 */
int kvso_window_hash(const int32_t *tokens, int64_t n, int32_t w, uint32_t b, uint32_t m, uint32_t *hash_out)
{
    if (n < 0 || w <= 0 || m == 0 || (n > 0 && !tokens) || (n >= w && !hash_out)) return 1;
    for (int64_t i = 0; i < n; ++i)
        if (tokens[i] < 0) return 1;
    for (int64_t i = 0; i + w <= n; ++i) {
        uint64_t h = 0;
        for (int32_t x = 0; x < w; ++x) h = (h * (uint64_t)b + (uint64_t)tokens[i + x]) % (uint64_t)m;
        hash_out[i] = (uint32_t)h;
    }
    return 0;
}

typedef struct { uint32_t h; int64_t i; } kvso_index_entry;

static int index_entry_cmp(const void *a, const void *b)
{
    const kvso_index_entry *x = (const kvso_index_entry *)a, *y = (const kvso_index_entry *)b;
    if (x->h != y->h) return x->h < y->h ? -1 : 1;
    return x->i < y->i ? -1 : (x->i > y->i ? 1 : 0);
}

/* ---------------------------------------------------------------------------------------------
 * App. E, Alg. 3.  Step 2: an index from hash value to the list of target window starts with
 * that hash, in ascending order (here: the (hash, start) pairs sorted, a list being a stretch of
 * equal hashes).  Step 3: candidate window starts j in ascending order; for every target start
 * i listed under the candidate window's hash, k runs from 0 while both positions exist and the
 * tokens agree; a target position i+k that has not been matched before is recorded together
 * with j+k and marked.  The algorithm compares hashes only, then tokens one at a time: two
 * windows that collide in the hash still contribute the stretch of equal tokens they start with.
 *
 * target_matches, candidate_matches: [n_target] each, filled in the order of discovery;
 * *n_matches: how many pairs were recorded.
 */
int kvso_match_tokens(const int32_t *target, int64_t n_target, const int32_t *candidate, int64_t n_candidate,
                      int32_t w, uint32_t b, uint32_t m,
                      int32_t *target_matches, int32_t *candidate_matches, int64_t *n_matches)
{
    if (n_target < 0 || n_candidate < 0 || w <= 0 || m == 0 || !n_matches) return 1;
    if (n_target > 0x7fffffff || n_candidate > 0x7fffffff) return 1;
    *n_matches = 0;
    const int64_t nt = n_target - w + 1, nc = n_candidate - w + 1;     /* window starts */
    for (int64_t i = 0; i < n_target; ++i) if (target[i] < 0) return 1;
    for (int64_t j = 0; j < n_candidate; ++j) if (candidate[j] < 0) return 1;
    if (nt <= 0 || nc <= 0) return 0;
    uint32_t *ht = (uint32_t *)malloc((size_t)nt * sizeof(uint32_t));
    uint32_t *hc = (uint32_t *)malloc((size_t)nc * sizeof(uint32_t));
    kvso_index_entry *index = (kvso_index_entry *)malloc((size_t)nt * sizeof(kvso_index_entry));
    unsigned char *matched = (unsigned char *)calloc((size_t)n_target, 1);
    if (!ht || !hc || !index || !matched) { free(ht); free(hc); free(index); free(matched); return 1; }
    kvso_window_hash(target, n_target, w, b, m, ht);
    kvso_window_hash(candidate, n_candidate, w, b, m, hc);
    for (int64_t i = 0; i < nt; ++i) { index[i].h = ht[i]; index[i].i = i; }
    qsort(index, (size_t)nt, sizeof(kvso_index_entry), index_entry_cmp);
    int64_t count = 0;
    for (int64_t j = 0; j < nc; ++j) {
        const uint32_t h = hc[j];
        /* first entry of the list under h */
        int64_t lo = 0, hi = nt;
        while (lo < hi) { const int64_t mid = (lo + hi) / 2; if (index[mid].h < h) lo = mid + 1; else hi = mid; }
        for (int64_t e = lo; e < nt && index[e].h == h; ++e) {
            const int64_t i = index[e].i;
            int64_t k = 0;
            while (i + k < n_target && j + k < n_candidate && target[i + k] == candidate[j + k]) {
                if (!matched[i + k]) {
                    target_matches[count] = (int32_t)(i + k);
                    candidate_matches[count] = (int32_t)(j + k);
                    ++count;
                    matched[i + k] = 1;
                }
                ++k;
            }
        }
    }
    *n_matches = count;
    free(ht); free(hc); free(index); free(matched);
    return 0;
}

/* ---------------------------------------------------------------------------------------------
 * Recomputing the selected tokens in a later layer (App. D.1): row m of the output is the layer's
 * projection of the hidden state of selected token m,
 *     y[m, f] = sum_c x[rows[m], c] * w[f, c]          f over (n_q_heads + 2 n_kv_heads) * head_dim features,
 * (w is stored as PyTorch stores a Linear weight: one row per output feature), split into Q, K, V by
 * heads.  With a rotary table, channel pair (c, c + head_dim/2) of every Q and K head is turned by the
 * angle the table holds for the token's position p = pos[m] and frequency c:
 *     out[c]              = y[c] cos - y[c + head_dim/2] sin
 *     out[c + head_dim/2] = y[c + head_dim/2] cos + y[c] sin,      (cos, sin) = rope[p, c, 0..1];
 * V is not turned.  The table is an input (the caller decides base and scaling of the frequencies).
 *
 * x [n_tokens, hidden], w [(n_q_heads + 2 n_kv_heads) * head_dim, hidden]: dtype of the shape
 * rows [n_sel] int32 or NULL (row m of x is token m), pos [n_sel] int32 (read only with a table)
 * rope [rope_positions, head_dim/2, 2] fp32 or NULL
 * q_out [n_sel, n_q_heads, head_dim], k_out, v_out [n_sel, n_kv_heads, head_dim]: fp64, not rounded
 */
int kvso_project_qkv(const kvso_shape *sh, int32_t hidden, const void *x, int64_t n_tokens,
                     const int32_t *rows, const int32_t *pos, int64_t n_sel, const void *w,
                     const float *rope, int64_t rope_positions,
                     double *q_out, double *k_out, double *v_out)
{
    if (!shape_ok(sh) || hidden <= 0 || n_tokens < 0 || n_sel < 0 || (sh->head_dim & 1)) return 1;
    if (n_sel == 0) return 0;
    if (!x || !w || !q_out || !k_out || !v_out || (rope && !pos)) return 1;
    const int d = sh->head_dim, hq = sh->n_q_heads, hk = sh->n_kv_heads, half = d / 2;
    const int64_t features = (int64_t)(hq + 2 * hk) * d;
    for (int64_t m = 0; m < n_sel; ++m) {
        const int64_t r = rows ? rows[m] : m;
        if (r < 0 || r >= n_tokens) return 1;
        if (rope && (pos[m] < 0 || pos[m] >= rope_positions)) return 1;
    }
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < n_sel; ++m) {
        const int64_t r = rows ? rows[m] : m;
        double *y = (double *)malloc((size_t)features * sizeof(double));
        if (!y) { bad = 1; continue; }
        for (int64_t f = 0; f < features; ++f) {
            double acc = 0.0;
            for (int32_t c = 0; c < hidden; ++c) acc += ld(x, sh->dtype, r * hidden + c) * ld(w, sh->dtype, f * hidden + c);
            y[f] = acc;
        }
        for (int h = 0; h < hq + 2 * hk; ++h) {
            double *yh = y + (int64_t)h * d;
            double *dst = h < hq ? q_out + (m * hq + h) * d
                        : h < hq + hk ? k_out + (m * hk + (h - hq)) * d
                                      : v_out + (m * hk + (h - hq - hk)) * d;
            const int turned = rope && h < hq + hk;
            for (int c = 0; c < half; ++c) {
                if (turned) {
                    const double cs = (double)rope[((int64_t)pos[m] * half + c) * 2 + 0];
                    const double sn = (double)rope[((int64_t)pos[m] * half + c) * 2 + 1];
                    dst[c] = yh[c] * cs - yh[c + half] * sn;
                    dst[c + half] = yh[c + half] * cs + yh[c] * sn;
                } else {
                    dst[c] = yh[c];
                    dst[c + half] = yh[c + half];
                }
            }
        }
        free(y);
    }
    return bad;
}

/* ---------------------------------------------------------------------------------------------
 * Sec. 4.3, Alg. 2: the queue sorted by cache hit rate, descending (requests of equal rate stay
 * in their order of arrival, which is their index), and the first N of it sent on as a batch.
 * order: [n] the whole queue after the sort; the batch is its first min(N, n) entries.
 */
int kvso_schedule(const float *hit_rate, int32_t n, int32_t *order)
{
    if (n < 0 || (n > 0 && (!hit_rate || !order))) return 1;
    for (int32_t r = 0; r < n; ++r) order[r] = r;
    /* insertion sort: stable, and the queue of Alg. 2 is built by insertions */
    for (int32_t r = 1; r < n; ++r) {
        const int32_t x = order[r];
        int32_t q = r;
        while (q > 0 && hit_rate[order[q - 1]] < hit_rate[x]) { order[q] = order[q - 1]; --q; }
        order[q] = x;
    }
    return 0;
}

int kvso_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
