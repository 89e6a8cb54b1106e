// Host-side pieces of the C ABI that are not tied to one kernel: error reporting, shape
// validation, workspace sizing and the kvs_partial_attention entry point, which validates the
// ragged batch description and dispatches to the matrix-core or the fp32 vector kernel.
#include "kvs_internal.h"
#include "attention.h"

#include <stdarg.h>
#include <stdio.h>
#include <string.h>

namespace kvs {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

kvs_status fail(kvs_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

kvs_status check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KVS_EHIP, "%s: %s", what, hipGetErrorString(e));
    return KVS_OK;
}

kvs_status check_shape(const kvs_shape *s)
{
    if (!s) return fail(KVS_EINVAL, "shape is NULL");
    if (s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->head_dim <= 0)
        return fail(KVS_EINVAL, "shape has a non-positive field (%d q heads, %d kv heads, head_dim %d)", s->n_q_heads, s->n_kv_heads, s->head_dim);
    if (s->n_q_heads % s->n_kv_heads != 0)
        return fail(KVS_EINVAL, "n_q_heads %d is not a multiple of n_kv_heads %d", s->n_q_heads, s->n_kv_heads);
    if (s->dtype != KVS_F32 && s->dtype != KVS_BF16) return fail(KVS_EINVAL, "unknown dtype %d", s->dtype);
    if (s->head_dim != 64 && s->head_dim != 128) return fail(KVS_EUNSUPPORTED, "head_dim %d (64 and 128 are built)", s->head_dim);
    return KVS_OK;
}

} // namespace kvs

extern "C" const char *kvs_strerror(kvs_status st)
{
    switch (st) {
    case KVS_OK: return "ok";
    case KVS_EINVAL: return "invalid argument";
    case KVS_EUNSUPPORTED: return "unsupported shape or dtype";
    case KVS_EWORKSPACE: return "workspace too small";
    case KVS_EHIP: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" const char *kvs_last_error(void) { return kvs::g_err; }

extern "C" const char *kvs_version(void) { return "kvshare-hip gfx950 1"; }

extern "C" size_t kvs_workspace_size(const char *call, const kvs_shape *shape, int32_t batch,
                                     int64_t n_rows_total, int64_t n_sel_total)
{
    if (!call || batch < 0 || n_rows_total < 0) return 0;
    if (strcmp(call, "match_tokens") == 0) return kvs::match_workspace_bytes(n_rows_total, n_sel_total);
    if (!shape) return 0;
    if (strcmp(call, "decode_check") == 0) return kvs::decode_workspace_bytes(shape, batch, n_rows_total);
    if (strcmp(call, "select_topk") == 0) return kvs::select_workspace_bytes(batch, n_rows_total);
    if (strcmp(call, "attn_colsum") == 0) return kvs::colsum_workspace_bytes(shape, n_rows_total);
    if (strcmp(call, "first_order_impact") == 0) return kvs::impact_workspace_bytes(shape, n_rows_total);
    if (strcmp(call, "partial_attention") == 0)
        return kvs::attention_mfma_supports(shape) ? kvs::attention_workspace_bytes(shape, batch, n_rows_total, n_sel_total) : 256;
    return 0;
}

extern "C" kvs_status kvs_partial_attention(const kvs_shape *shape, int32_t batch,
                                            const int64_t *ctx_off, const int64_t *ctx_len,
                                            const int64_t *cu_sel,
                                            const void *q_sel, const int32_t *sel_pos,
                                            const void *k_cache, const void *v_cache, float scale,
                                            void *out, float *lse_out,
                                            void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace kvs;
    kvs_status st = check_shape(shape);
    if (st != KVS_OK) return st;
    if (batch < 0) return fail(KVS_EINVAL, "kvs_partial_attention: batch < 0");
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return fail(KVS_EINVAL, "kvs_partial_attention: workspace must be 256-byte aligned");
    if (batch == 0) return KVS_OK;
    if (!ctx_off || !ctx_len || !cu_sel) return fail(KVS_EINVAL, "kvs_partial_attention: ctx_off/ctx_len/cu_sel is NULL");
    if (cu_sel[0] != 0) return fail(KVS_EINVAL, "kvs_partial_attention: cu_sel[0] must be 0");
    for (int32_t b = 0; b < batch; ++b) {
        if (ctx_off[b] < 0 || ctx_len[b] < 0) return fail(KVS_EINVAL, "kvs_partial_attention: negative context offset/length (request %d)", b);
        if (ctx_len[b] > 0x7fffffffLL) return fail(KVS_EINVAL, "kvs_partial_attention: context of request %d too long", b);
        if (cu_sel[b + 1] < cu_sel[b]) return fail(KVS_EINVAL, "kvs_partial_attention: cu_sel decreases at request %d", b);
        if (cu_sel[b + 1] - cu_sel[b] > ctx_len[b]) return fail(KVS_EINVAL, "kvs_partial_attention: request %d selects more tokens than its context holds", b);
    }
    const int64_t n_sel = cu_sel[batch];
    if (n_sel == 0) return KVS_OK;
    if (!q_sel || !sel_pos || !k_cache || !v_cache || !out) return fail(KVS_EINVAL, "kvs_partial_attention: NULL tensor pointer");
    if (!aligned16(q_sel) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out))
        return fail(KVS_EINVAL, "kvs_partial_attention: Q/K/V/out pointers must be 16-byte aligned");
    hipStream_t hs = (hipStream_t)stream;
    // the matrix-core kernel folds the scale into an exp2 argument and takes the row max before
    // scaling, which needs scale > 0; anything else goes to the vector kernel
    const bool mfma = attention_mfma_supports(shape) && scale > 0.f && scale < 3.0e38f;
    for (int32_t b0 = 0; b0 < batch; b0 += kAttnMaxReq) {
        const int nr = (batch - b0) < kAttnMaxReq ? (batch - b0) : kAttnMaxReq;
        AttnBatch bd;
        for (int i = 0; i < kAttnMaxReq; ++i) {
            const bool live = i < nr;
            bd.ctx_off[i] = live ? ctx_off[b0 + i] : 0;
            bd.ctx_len[i] = live ? ctx_len[b0 + i] : 0;
            bd.cu_sel[i] = live ? cu_sel[b0 + i] : cu_sel[b0 + nr];
        }
        bd.cu_sel[kAttnMaxReq] = cu_sel[b0 + nr];
        bd.sel_begin = cu_sel[b0];
        bd.n_req = nr;
        const int64_t ns = cu_sel[b0 + nr] - cu_sel[b0];
        if (ns == 0) continue;
        st = mfma ? launch_attention_mfma(shape, bd, ns, q_sel, sel_pos, k_cache, v_cache, scale, out, lse_out, workspace, workspace_bytes, hs)
                  : launch_attention_valu(shape, bd, ns, q_sel, sel_pos, k_cache, v_cache, scale, out, lse_out, hs);
        if (st != KVS_OK) return st;
    }
    return KVS_OK;
}
