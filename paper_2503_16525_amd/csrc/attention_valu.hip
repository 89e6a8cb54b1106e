// Partial-recompute attention, fp32 vector path (Eq. (1) restricted to the selected rows).
//
// Used for fp32 inputs (1e-4 tolerance, no matrix-core path for that type) and as the generic
// fallback for shapes the bf16 MFMA kernel does not cover.  One workgroup owns one selected
// token and one KV head, i.e. the up to 8 query heads that share that KV head; K/V tiles of 64 (or 32)
// keys are widened to fp32 in LDS once and reused by all of those heads.  Softmax is the usual
// running-max / running-sum form, all in fp32.
#include "kvs_internal.h"
#include "attention.h"

#include <math.h>

namespace kvs {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxG = 8;      // query heads handled per pass over the keys

template <int DTYPE>
__device__ __forceinline__ float load_elem(const void *p, int64_t i)
{
    if (DTYPE == KVS_F32) return ((const float *)p)[i];
    return __uint_as_float((uint32_t)((const uint16_t *)p)[i] << 16);
}

template <int DTYPE>
__device__ __forceinline__ void store_elem(void *p, int64_t i, float v)
{
    if (DTYPE == KVS_F32) ((float *)p)[i] = v;
    else ((uint16_t *)p)[i] = (uint16_t)f32_to_bf16_bits(v);
}

template <int DTYPE, int D>
__global__ __launch_bounds__(kThreads) void attn_valu_kernel(
    const AttnBatch bd, int n_q_heads, int n_kv_heads,
    const void *__restrict__ q_sel, const int32_t *__restrict__ sel_pos,
    const void *__restrict__ k_cache, const void *__restrict__ v_cache, float scale,
    void *__restrict__ out, float *__restrict__ lse_out)
{
    constexpr int kTile = D <= 64 ? 64 : 32;   // keys per LDS tile (keeps static LDS under 64 KiB)
    __shared__ float Ks[kTile][D + 1];
    __shared__ float Vs[kTile][D];
    __shared__ float q_s[kMaxG][D];
    __shared__ float p_s[kMaxG][kTile];
    __shared__ float m_s[kMaxG], l_s[kMaxG], corr_s[kMaxG];

    const int64_t s = bd.sel_begin + blockIdx.x;
    const int g = blockIdx.y;
    int b = 0;
    while (b + 1 < bd.n_req && s >= bd.cu_sel[b + 1]) ++b;   // requests per launch <= 64
    const int64_t row0 = bd.ctx_off[b];
    const int p = sel_pos[s];
    if (p < 0 || p >= bd.ctx_len[b]) return;                  // memory safety; caller guarantees range
    const int kv_len = p + 1;
    const int grp = n_q_heads / n_kv_heads;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    for (int h0 = 0; h0 < grp; h0 += kMaxG) {
        const int nh = min(kMaxG, grp - h0);
        for (int e = tid; e < nh * D; e += kThreads) {
            const int hh = e / D, c = e % D;
            q_s[hh][c] = load_elem<DTYPE>(q_sel, (s * n_q_heads + g * grp + h0 + hh) * (int64_t)D + c) * scale;
        }
        if (tid < kMaxG) { m_s[tid] = -INFINITY; l_s[tid] = 0.f; }
        float o[kMaxG * D / kThreads];
#pragma unroll
        for (int i = 0; i < kMaxG * D / kThreads; ++i) o[i] = 0.f;
        __syncthreads();

        for (int t0 = 0; t0 < kv_len; t0 += kTile) {
            for (int e = tid; e < kTile * D; e += kThreads) {
                const int j = e / D, c = e % D;
                const bool ok = t0 + j < kv_len;
                const int64_t gi = ((row0 + t0 + j) * n_kv_heads + g) * (int64_t)D + c;
                Ks[j][c] = ok ? load_elem<DTYPE>(k_cache, gi) : 0.f;
                Vs[j][c] = ok ? load_elem<DTYPE>(v_cache, gi) : 0.f;
            }
            __syncthreads();
            // logits + online softmax: wave w takes heads w, w+4; lane = key
            for (int hh = wave; hh < nh; hh += kThreads / 64) {
                float acc = 0.f;
                const int jr = lane < kTile ? lane : 0;
#pragma unroll 8
                for (int c = 0; c < D; ++c) acc += q_s[hh][c] * Ks[jr][c];
                const bool ok = lane < kTile && t0 + lane < kv_len;
                const float logit = ok ? acc : -INFINITY;
                const float m_old = m_s[hh];
                const float m_new = fmaxf(m_old, wave_max(logit));
                const float pj = ok ? expf(logit - m_new) : 0.f;
                const float corr = expf(m_old - m_new);        // exp(-inf) = 0 on the first tile
                const float psum = wave_sum(pj);
                if (lane < kTile) p_s[hh][lane] = pj;
                if (lane == 0) { m_s[hh] = m_new; l_s[hh] = l_s[hh] * corr + psum; corr_s[hh] = corr; }
            }
            __syncthreads();
            // o[hh][c] = o*corr + sum_j p[hh][j] * V[j][c]
#pragma unroll
            for (int i = 0; i < kMaxG * D / kThreads; ++i) {
                const int e = i * kThreads + tid;
                const int hh = e / D, c = e % D;
                if (hh < nh) {
                    float acc = o[i] * corr_s[hh];
#pragma unroll 8
                    for (int j = 0; j < kTile; ++j) acc += p_s[hh][j] * Vs[j][c];
                    o[i] = acc;
                }
            }
            __syncthreads();
        }
#pragma unroll
        for (int i = 0; i < kMaxG * D / kThreads; ++i) {
            const int e = i * kThreads + tid;
            const int hh = e / D, c = e % D;
            if (hh < nh) {
                const int h = g * grp + h0 + hh;
                store_elem<DTYPE>(out, (s * n_q_heads + h) * (int64_t)D + c, o[i] / l_s[hh]);
            }
        }
        if (lse_out && tid < nh) lse_out[s * n_q_heads + g * grp + h0 + tid] = m_s[tid] + logf(l_s[tid]);
        __syncthreads();
    }
}

} // namespace

kvs_status launch_attention_valu(const kvs_shape *shape, const AttnBatch &bd, int64_t n_sel,
                                 const void *q_sel, const int32_t *sel_pos, const void *k_cache,
                                 const void *v_cache, float scale, void *out, float *lse_out,
                                 hipStream_t st)
{
    if (n_sel == 0) return KVS_OK;
    if (n_sel > 0x7fffffffLL || shape->n_kv_heads > 65535) return fail(KVS_EINVAL, "kvs_partial_attention: grid too large");
    dim3 grid((unsigned)n_sel, (unsigned)shape->n_kv_heads), block(kThreads);
#define KVS_ATT_CASE(DT, DD)                                                                         \
    hipLaunchKernelGGL((attn_valu_kernel<DT, DD>), grid, block, 0, st, bd, shape->n_q_heads,          \
                       shape->n_kv_heads, q_sel, sel_pos, k_cache, v_cache, scale, out, lse_out)
    if (shape->dtype == KVS_F32 && shape->head_dim == 64) KVS_ATT_CASE(KVS_F32, 64);
    else if (shape->dtype == KVS_F32 && shape->head_dim == 128) KVS_ATT_CASE(KVS_F32, 128);
    else if (shape->dtype == KVS_BF16 && shape->head_dim == 64) KVS_ATT_CASE(KVS_BF16, 64);
    else if (shape->dtype == KVS_BF16 && shape->head_dim == 128) KVS_ATT_CASE(KVS_BF16, 128);
    else return fail(KVS_EUNSUPPORTED, "kvs_partial_attention: head_dim %d", shape->head_dim);
#undef KVS_ATT_CASE
    return check_launch("kvs_partial_attention(valu)");
}

} // namespace kvs
