// kvs_attn_colsum for the shapes the matrix-core kernel does not cover (fp32, head_dim 64, ...):
// the same two sweeps (row log-sum-exps, then column sums of exp(score - lse); Alg. 1 steps 1-2)
// on the vector units, one wavefront per output.  Plain and slow - it exists so that the tiny
// fp32 configuration runs the whole of Alg. 1 on the device; nothing large should come here.
#include "kvs_internal.h"

#include <math.h>

namespace kvs {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxD = 128;

template <int DTYPE>
__device__ __forceinline__ float load_elem(const void *p, int64_t i)
{
    if (DTYPE == KVS_F32) return ((const float *)p)[i];
    return __uint_as_float((uint32_t)((const uint16_t *)p)[i] << 16);
}

// one wave per (query token j, query head h): lse[j, h] = log sum_{i <= j} exp(scale * q . k_i)
template <int DTYPE>
__global__ __launch_bounds__(kThreads) void colsum_rows_valu(int n, int n_q_heads, int n_kv_heads, int d,
                                                             const void *__restrict__ q, const void *__restrict__ k,
                                                             float scale, float *__restrict__ lse)
{
    __shared__ float qs[kWaves][kMaxD];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * kWaves + wave;           // j * n_q_heads + h
    const bool live = row < (int64_t)n * n_q_heads;
    const int j = live ? (int)(row / n_q_heads) : 0, h = live ? (int)(row % n_q_heads) : 0;
    const int g = h / (n_q_heads / n_kv_heads);
    for (int c = lane; c < d; c += 64) qs[wave][c] = load_elem<DTYPE>(q, ((int64_t)j * n_q_heads + h) * d + c) * scale;
    __syncthreads();
    float m = -INFINITY, z = 0.f;
    for (int i = lane; i <= j; i += 64) {
        const int64_t kb = ((int64_t)i * n_kv_heads + g) * d;
        float s = 0.f;
        for (int c = 0; c < d; ++c) s = fmaf(qs[wave][c], load_elem<DTYPE>(k, kb + c), s);
        const float mn = fmaxf(m, s);
        z = z * expf(m - mn) + expf(s - mn);
        m = mn;
    }
    const float mw = wave_max(m);
    const float zw = wave_sum(m == -INFINITY ? 0.f : z * expf(m - mw));
    if (live && lane == 0) lse[row] = mw + logf(zw);
}

// one wave per (key i, KV head g): alpha[g, i] = sum over the group's heads and the rows j >= i
template <int DTYPE>
__global__ __launch_bounds__(kThreads) void colsum_cols_valu(int n, int n_q_heads, int n_kv_heads, int d,
                                                             const void *__restrict__ q, const void *__restrict__ k,
                                                             float scale, const float *__restrict__ lse,
                                                             float *__restrict__ alpha)
{
    __shared__ float ks[kWaves][kMaxD];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t col = (int64_t)blockIdx.x * kWaves + wave;           // g * n + i
    const bool live = col < (int64_t)n * n_kv_heads;
    const int g = live ? (int)(col / n) : 0, i = live ? (int)(col % n) : 0;
    const int grp = n_q_heads / n_kv_heads;
    for (int c = lane; c < d; c += 64) ks[wave][c] = load_elem<DTYPE>(k, ((int64_t)i * n_kv_heads + g) * d + c) * scale;
    __syncthreads();
    float acc = 0.f;
    const int64_t r_end = (int64_t)n * grp;
    for (int64_t r = (int64_t)i * grp + lane; r < r_end; r += 64) {    // flattened (token, head-in-group)
        const int64_t j = r / grp;
        const int h = g * grp + (int)(r - j * grp);
        const int64_t qb = (j * n_q_heads + h) * d;
        float s = 0.f;
        for (int c = 0; c < d; ++c) s = fmaf(ks[wave][c], load_elem<DTYPE>(q, qb + c), s);
        acc += expf(s - lse[j * n_q_heads + h]);
    }
    acc = wave_sum(acc);
    if (live && lane == 0) alpha[col] = acc;
}

} // namespace

kvs_status launch_colsum_valu(const kvs_shape *shape, int64_t n, const void *q, const void *k, float scale,
                              float *lse, float *alpha, hipStream_t st)
{
    const int d = shape->head_dim, hq = shape->n_q_heads, hk = shape->n_kv_heads;
    if (d > kMaxD) return fail(KVS_EUNSUPPORTED, "kvs_attn_colsum: head_dim %d", d);
    // quadratic work at a few percent of the matrix-core rate: refuse what would run for minutes
    if (n > 65536) return fail(KVS_EUNSUPPORTED, "kvs_attn_colsum: %lld tokens are too many for the vector path (this shape has no matrix-core kernel)", (long long)n);
    const dim3 block(kThreads);
    const dim3 g1((unsigned)((n * hq + kWaves - 1) / kWaves)), g2((unsigned)((n * hk + kWaves - 1) / kWaves));
    if (shape->dtype == KVS_F32) {
        hipLaunchKernelGGL(colsum_rows_valu<KVS_F32>, g1, block, 0, st, (int)n, hq, hk, d, q, k, scale, lse);
        hipLaunchKernelGGL(colsum_cols_valu<KVS_F32>, g2, block, 0, st, (int)n, hq, hk, d, q, k, scale, (const float *)lse, alpha);
    } else {
        hipLaunchKernelGGL(colsum_rows_valu<KVS_BF16>, g1, block, 0, st, (int)n, hq, hk, d, q, k, scale, lse);
        hipLaunchKernelGGL(colsum_cols_valu<KVS_BF16>, g2, block, 0, st, (int)n, hq, hk, d, q, k, scale, (const float *)lse, alpha);
    }
    return check_launch("kvs_attn_colsum(vector path)");
}

} // namespace kvs
