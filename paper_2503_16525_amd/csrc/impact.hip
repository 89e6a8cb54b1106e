// kvs_first_order_impact: the first-order expansion of the attention output's deviation (Sec. 4.1,
// Eq. (2)), token by token.  Reusing token i's cache entry moves output row j of query head h by
//     A[h,j,i] * dV[g,i]                                             value direction (dH/dV = A)
//   + A[h,j,i] * scale * (q[j,h] . dK[g,i]) * (V[g,i] - H[h,j])      key direction (softmax Jacobian)
// and the token's impact is the L1 norm of that movement over all rows j >= i, heads and channels,
// for the value term alone (which is Eq. (3): column mass times |dV|_1), the key term alone, and
// both together.  The paper drops the key term "to reduce computational overhead": unlike the value
// term it does not separate into (something of i) x (something of j) -- every (row, token) pair
// needs its own L1 norm over the channels -- so this is N^2/2 * H_q * d work on the vector units, not
// a contraction for the matrix cores (only the two dot products per pair are).  It is a diagnostic
// for check layers, not a step of the hot path.
//
// One workgroup owns 32 tokens (columns) of one KV head: their K, dK, V, dV rows sit in LDS as
// fp32, channel-major so that the 32 column lanes of a wave hit 32 banks.  Rows stream past in
// blocks of 64 flattened (query row, head-in-group) pairs, staged in LDS with their output rows
// H; thread (column c, row lane r) handles four pairs at a time: first the two dot products per
// pair (logit and q . dK), then, with a = exp(scale * logit - lse) and t = scale * (q . dK)
// known, the channel loop of the L1 norms (a and t factored out of the sums).  For bf16 the dot products
// are the one part that is a contraction: q . K_fresh and q . K_cache (both exact bf16 operands; their
// difference is q . dK) run on the matrix cores from bf16 copies of the rows and columns in LDS, every
// wave computing the 32 x 32 tile its lanes' four pairs lie in.  Sums are kept per thread in a fixed order and the 16
// row lanes of a column are added in a fixed order at the end: bit-reproducible.  Per-head
// partial sums go to the workspace; a second kernel adds the KV heads and applies the mask.
#include "kvs_internal.h"

#include <math.h>

namespace kvs {
namespace {

constexpr int kImpCols = 32;                 // tokens per workgroup
constexpr int kImpRowLanes = 16;
constexpr int kImpThreads = kImpCols * kImpRowLanes;    // 512
constexpr int kImpPairs = 4;                 // (row, head) pairs a thread handles at a time: a column value read from LDS serves all of them
constexpr int kImpBlock = kImpRowLanes * kImpPairs;      // 32 pairs staged per block

template <int DTYPE>
__device__ __forceinline__ float load_elem(const void *p, int64_t i)
{
    if (DTYPE == KVS_F32) return reinterpret_cast<const float *>(p)[i];
    return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(p)[i] << 16);
}

// grid: (column tiles, heaviest first) x kv heads
template <int DTYPE, int D>
__global__ __launch_bounds__(kImpThreads) void impact_kernel(
    int n, int n_q_heads, int n_kv_heads,
    const void *__restrict__ q, const void *__restrict__ k_fresh, const void *__restrict__ v_fresh,
    const void *__restrict__ k_cache, const void *__restrict__ v_cache,
    const void *__restrict__ h_fresh, const float *__restrict__ lse, float scale,
    float *__restrict__ part /* [3][n_kv_heads][n]: value, key, both */)
{
    extern __shared__ float lds[];
    constexpr bool MFMA_DOTS = DTYPE == KVS_BF16;
    // fp32, channel-major columns; K and dK (and the rows' Q) only where the dot products run on the vector units
    float *colV = lds;                        // [D][kImpCols]
    float *colDV = colV + D * kImpCols;
    float *colK = colDV + D * kImpCols;
    float *colDK = colK + (MFMA_DOTS ? 0 : D * kImpCols);
    float *rowH = colDK + (MFMA_DOTS ? 0 : D * kImpCols);       // [kImpBlock][D]
    float *rowQ = rowH + kImpBlock * D;
    float *rowL = rowQ + (MFMA_DOTS ? 0 : kImpBlock * D);       // [kImpBlock] lse; [kImpBlock] row index follows
    int *rowJ = reinterpret_cast<int *>(rowL + kImpBlock);
    float *red = reinterpret_cast<float *>(rowJ + kImpBlock);   // [3][kImpRowLanes][kImpCols]
    // bf16 copies for the matrix cores (DTYPE bf16 only): rows of 2 D bytes, 16-byte pieces XOR-swizzled by the row
    uint16_t *bfKf = reinterpret_cast<uint16_t *>(red + 3 * kImpRowLanes * kImpCols);   // [kImpCols][D]
    uint16_t *bfKc = bfKf + kImpCols * D;
    uint16_t *bfQ = bfKc + kImpCols * D;                                                  // [kImpBlock][D]
    constexpr int PIECES = D / 8;              // 16-byte pieces per bf16 row

    const int tid = threadIdx.x, col = tid % kImpCols, rl = tid / kImpCols;
    const int g = blockIdx.y;
    const int grp = n_q_heads / n_kv_heads;
    const int i0 = blockIdx.x * kImpCols;                  // first token of this workgroup (low tiles have the most rows)
    const int i = i0 + col;
    // ---- the tile's columns into LDS ----
    for (int e = tid; e < kImpCols * D; e += kImpThreads) {
        const int c = e % D, t = e / D;                    // consecutive threads read consecutive channels of a token
        const int tok = min(i0 + t, n - 1);
        const int64_t at = ((int64_t)tok * n_kv_heads + g) * D + c;
        const float kf = load_elem<DTYPE>(k_fresh, at), vf = load_elem<DTYPE>(v_fresh, at);
        if (!MFMA_DOTS) {
            colK[c * kImpCols + t] = kf;
            colDK[c * kImpCols + t] = load_elem<DTYPE>(k_cache, at) - kf;
        }
        colV[c * kImpCols + t] = vf;
        colDV[c * kImpCols + t] = load_elem<DTYPE>(v_cache, at) - vf;
    }
    if (MFMA_DOTS) {
        for (int e = tid; e < kImpCols * PIECES; e += kImpThreads) {
            const int pc = e % PIECES, t = e / PIECES;
            const int tok = min(i0 + t, n - 1);
            const int64_t at = ((int64_t)tok * n_kv_heads + g) * D + 8 * pc;
            const int dst = t * D + 8 * (pc ^ (t & (PIECES - 1)));
            *reinterpret_cast<uint4 *>(bfKf + dst) = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(k_fresh) + at);
            *reinterpret_cast<uint4 *>(bfKc + dst) = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(k_cache) + at);
        }
    }
    __syncthreads();
    float dv_l1 = 0.f;                                     // |dV_i|_1, fixed order
    for (int c = 0; c < D; ++c) dv_l1 += fabsf(colDV[c * kImpCols + col]);

    float acc_a = 0.f, acc_k = 0.f, acc_kv = 0.f;          // sum of A, key-term norm, combined norm for (column, row lane)
    const int64_t n_pairs = (int64_t)(n - i0) * grp;       // flattened (row j >= i0, head in group)
    // bf16: a block's rows (H and Q, 16-byte pieces; two of each per thread) are fetched into registers while
    // the block before is being worked on, and written to LDS between two barriers
    constexpr int kFetch = MFMA_DOTS ? kImpBlock * PIECES / kImpThreads : 1;
    static_assert(!MFMA_DOTS || kImpBlock * PIECES % kImpThreads == 0, "whole pieces per thread");
    uint4 h_next[kFetch], q_next[kFetch];
    float l_next = 0.f;
    int j_next = -1;
    auto fetch = [&](int64_t p0) {
#pragma unroll
        for (int f = 0; f < kFetch; ++f) {
            const int e = tid + f * kImpThreads, pc = e % PIECES, r = e / PIECES;
            const int64_t p = min(p0 + r, n_pairs - 1);
            const int j = i0 + (int)(p / grp), h = g * grp + (int)(p % grp);
            const int64_t at = ((int64_t)j * n_q_heads + h) * D + 8 * pc;
            h_next[f] = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(h_fresh) + at);
            q_next[f] = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(q) + at);
        }
        if (tid < kImpBlock) {
            const int64_t p = p0 + tid;
            const int64_t pc = min(p, n_pairs - 1);
            const int j = i0 + (int)(pc / grp), h = g * grp + (int)(pc % grp);
            l_next = lse[(int64_t)j * n_q_heads + h];
            j_next = p < n_pairs ? j : -1;                 // -1: past the end, contributes nothing
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int f = 0; f < kFetch; ++f) {
            const int e = tid + f * kImpThreads, pc = e % PIECES, r = e / PIECES;
            const uint4 w = h_next[f];
            float *dst = rowH + r * D + 8 * pc;
            *reinterpret_cast<float4 *>(dst) = make_float4(bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y));
            *reinterpret_cast<float4 *>(dst + 4) = make_float4(bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w));
            *reinterpret_cast<uint4 *>(bfQ + r * D + 8 * (pc ^ (r & (PIECES - 1)))) = q_next[f];
        }
        if (tid < kImpBlock) { rowL[tid] = l_next; rowJ[tid] = j_next; }
    };
    if constexpr (MFMA_DOTS) fetch(0);
    for (int64_t p0 = 0; p0 < n_pairs; p0 += kImpBlock) {
        __syncthreads();                                    // the block before has been consumed
        if constexpr (MFMA_DOTS) {
            commit();
        } else {
            for (int e = tid; e < kImpBlock * D; e += kImpThreads) {
                const int c = e % D, r = e / D;
                const int64_t p = min(p0 + r, n_pairs - 1);
                const int j = i0 + (int)(p / grp), h = g * grp + (int)(p % grp);
                const int64_t at = ((int64_t)j * n_q_heads + h) * D + c;
                rowQ[r * D + c] = load_elem<DTYPE>(q, at);
                rowH[r * D + c] = load_elem<DTYPE>(h_fresh, at);
            }
            if (tid < kImpBlock) {
                const int64_t p = p0 + tid;
                const int64_t pc = min(p, n_pairs - 1);
                const int j = i0 + (int)(pc / grp), h = g * grp + (int)(pc % grp);
                rowL[tid] = lse[(int64_t)j * n_q_heads + h];
                rowJ[tid] = p < n_pairs ? j : -1;              // -1: past the end, contributes nothing
            }
        }
        __syncthreads();
        if constexpr (MFMA_DOTS) {
            if (p0 + kImpBlock < n_pairs) fetch(p0 + kImpBlock);
        }
        float s[kImpPairs], ds[kImpPairs];
        if constexpr (MFMA_DOTS) {
            // this wave's lanes hold pairs 8 w + 4 hf + u of the block: rows 8 (w & 3) + 4 hf + u of 32-row tile w >> 2,
            // i.e. accumulator entries 4 (w & 3) + u of the 32 x 32 product of that tile with the 32 columns
            typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
            typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
            static_assert(kImpPairs == 4 && kImpCols == 32 && kImpBlock == 64, "the tile picture above");
            const int wave = tid >> 6, ln = tid & 31, hf = (tid >> 5) & 1;
            floatx16 sf, sc;
#pragma unroll
            for (int e = 0; e < 16; ++e) { sf[e] = 0.f; sc[e] = 0.f; }
            const int qrow = 32 * (wave >> 2) + ln;
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                const int pc = 2 * ks + hf;
                const bf16x8 qa = *reinterpret_cast<const bf16x8 *>(bfQ + qrow * D + 8 * (pc ^ (qrow & (PIECES - 1))));
                const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(bfKf + ln * D + 8 * (pc ^ (ln & (PIECES - 1))));
                const bf16x8 kc = *reinterpret_cast<const bf16x8 *>(bfKc + ln * D + 8 * (pc ^ (ln & (PIECES - 1))));
                sf = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf, sf, 0, 0, 0);
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kc, sc, 0, 0, 0);
            }
            const int jq = wave & 3;
#pragma unroll
            for (int u = 0; u < kImpPairs; ++u) {
                const float f = jq == 0 ? sf[u] : jq == 1 ? sf[4 + u] : jq == 2 ? sf[8 + u] : sf[12 + u];
                const float c = jq == 0 ? sc[u] : jq == 1 ? sc[4 + u] : jq == 2 ? sc[8 + u] : sc[12 + u];
                s[u] = f;
                ds[u] = c - f;
            }
        } else {
#pragma unroll
        for (int u = 0; u < kImpPairs; ++u) { s[u] = 0.f; ds[u] = 0.f; }
#pragma unroll 4
        for (int c = 0; c < D; c += 4) {
            float4 qv[kImpPairs];
#pragma unroll
            for (int u = 0; u < kImpPairs; ++u) qv[u] = *reinterpret_cast<const float4 *>(&rowQ[(rl * kImpPairs + u) * D + c]);
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                const float kk = colK[(c + cc) * kImpCols + col], dk = colDK[(c + cc) * kImpCols + col];
#pragma unroll
                for (int u = 0; u < kImpPairs; ++u) {
                    const float qe = cc == 0 ? qv[u].x : cc == 1 ? qv[u].y : cc == 2 ? qv[u].z : qv[u].w;
                    s[u] = fmaf(qe, kk, s[u]);
                    ds[u] = fmaf(qe, dk, ds[u]);
                }
            }
        }
        }
        // With a = A[h,j,i] and t = scale * (q . dK), the pair moves output row (j, h) by a * (dV + t * (V - H)):
        // |key term|_1 = a |t| * sum_c |V_c - H_c| and |both|_1 = a * sum_c |dV_c + t (V_c - H_c)|, so the channel
        // loop needs a subtraction, an fma and two |.|-adds per channel and the pair's weights enter once at the end.
        float a[kImpPairs], t[kImpPairs];
#pragma unroll
        for (int u = 0; u < kImpPairs; ++u) {
            const int r = rl * kImpPairs + u;
            const int j = rowJ[r];
            const bool live = j >= i && i < n;             // causal: row j sees token i; rows past the end carry -1
            a[u] = live ? __expf(scale * s[u] - rowL[r]) : 0.f;
            t[u] = scale * ds[u];
            acc_a += a[u];
        }
        float nk[kImpPairs], nkv[kImpPairs];
#pragma unroll
        for (int u = 0; u < kImpPairs; ++u) { nk[u] = 0.f; nkv[u] = 0.f; }
#pragma unroll 4
        for (int c = 0; c < D; c += 4) {
            float4 hv[kImpPairs];
#pragma unroll
            for (int u = 0; u < kImpPairs; ++u) hv[u] = *reinterpret_cast<const float4 *>(&rowH[(rl * kImpPairs + u) * D + c]);
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                const float vv = colV[(c + cc) * kImpCols + col], dv = colDV[(c + cc) * kImpCols + col];
#pragma unroll
                for (int u = 0; u < kImpPairs; ++u) {
                    const float he = cc == 0 ? hv[u].x : cc == 1 ? hv[u].y : cc == 2 ? hv[u].z : hv[u].w;
                    const float dd = vv - he;
                    nk[u] += fabsf(dd);
                    nkv[u] += fabsf(fmaf(t[u], dd, dv));
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kImpPairs; ++u) { acc_k += a[u] * fabsf(t[u]) * nk[u]; acc_kv += a[u] * nkv[u]; }
    }
    // ---- the 16 row lanes of each column, added in lane order ----
    red[(0 * kImpRowLanes + rl) * kImpCols + col] = acc_a;
    red[(1 * kImpRowLanes + rl) * kImpCols + col] = acc_k;
    red[(2 * kImpRowLanes + rl) * kImpCols + col] = acc_kv;
    __syncthreads();
    if (rl == 0 && i < n) {
        float sa = 0.f, sk = 0.f, skv = 0.f;
        for (int r = 0; r < kImpRowLanes; ++r) {
            sa += red[(0 * kImpRowLanes + r) * kImpCols + col];
            sk += red[(1 * kImpRowLanes + r) * kImpCols + col];
            skv += red[(2 * kImpRowLanes + r) * kImpCols + col];
        }
        const int64_t o = (int64_t)g * n + i, stride = (int64_t)n_kv_heads * n;
        part[o] = sa * dv_l1;             // value direction: (sum of A over rows and heads of the group) * |dV|_1
        part[stride + o] = sk;
        part[2 * stride + o] = skv;
    }
}

__global__ void impact_reduce_kernel(int n, int n_kv_heads, const float *__restrict__ part, const uint8_t *__restrict__ reused,
                                     float *__restrict__ impact_v, float *__restrict__ impact_k, float *__restrict__ impact_kv)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const bool cand = reused ? reused[i] != 0 : true;
    const int64_t stride = (int64_t)n_kv_heads * n;
    float s[3] = {0.f, 0.f, 0.f};
    for (int g = 0; g < n_kv_heads; ++g)
#pragma unroll
        for (int t = 0; t < 3; ++t) s[t] += part[t * stride + (int64_t)g * n + i];
    if (impact_v) impact_v[i] = cand ? s[0] : -INFINITY;
    if (impact_k) impact_k[i] = cand ? s[1] : -INFINITY;
    if (impact_kv) impact_kv[i] = cand ? s[2] : -INFINITY;
}

template <int DTYPE, int D>
constexpr size_t impact_lds_bytes()
{
    return DTYPE == KVS_BF16
               ? sizeof(float) * (2 * D * kImpCols + kImpBlock * D + 2 * kImpBlock + 3 * kImpRowLanes * kImpCols)
                     + sizeof(uint16_t) * (2 * kImpCols * D + kImpBlock * D)
               : sizeof(float) * (4 * D * kImpCols + 2 * kImpBlock * D + 2 * kImpBlock + 3 * kImpRowLanes * kImpCols);
}

} // namespace

size_t impact_workspace_bytes(const kvs_shape *shape, int64_t n_tokens)
{
    return sizeof(float) * 3 * (size_t)shape->n_kv_heads * (size_t)n_tokens + 256;
}

} // namespace kvs

extern "C" kvs_status kvs_first_order_impact(const kvs_shape *shape, int64_t n_tokens, const void *q,
                                             const void *k_fresh, const void *v_fresh,
                                             const void *k_cache, const void *v_cache,
                                             const void *h_fresh, const float *lse,
                                             const uint8_t *reused, float scale,
                                             float *impact_v, float *impact_k, float *impact_kv,
                                             void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace kvs;
    kvs_status st = check_shape(shape);
    if (st != KVS_OK) return st;
    if (n_tokens < 0) return fail(KVS_EINVAL, "kvs_first_order_impact: n_tokens < 0");
    if (n_tokens == 0) return KVS_OK;
    if (n_tokens > (1 << 20)) return fail(KVS_EUNSUPPORTED, "kvs_first_order_impact: more than 2^20 tokens");
    if (!q || !k_fresh || !v_fresh || !k_cache || !v_cache || !h_fresh || !lse) return fail(KVS_EINVAL, "kvs_first_order_impact: NULL tensor pointer");
    if (!(isfinite(scale))) return fail(KVS_EINVAL, "kvs_first_order_impact: scale is not finite");
    if (shape->n_kv_heads > 65535) return fail(KVS_EUNSUPPORTED, "kvs_first_order_impact: too many kv heads");
    const size_t need = impact_workspace_bytes(shape, n_tokens);
    if (!workspace || workspace_bytes < need) return fail(KVS_EWORKSPACE, "kvs_first_order_impact: workspace %zu < %zu bytes", workspace_bytes, need);
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(KVS_EINVAL, "kvs_first_order_impact: workspace must be 256-byte aligned");
    hipStream_t hs = (hipStream_t)stream;
    const int n = (int)n_tokens;
    float *part = (float *)workspace;
    const dim3 grid((unsigned)((n + kImpCols - 1) / kImpCols), (unsigned)shape->n_kv_heads), block(kImpThreads);
#define KVS_IMP(DT, DD)                                                                                                   \
    do {                                                                                                                  \
        static DeviceOnce once;                                                                                           \
        st = once_per_device(once, [] {                                                                                   \
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&impact_kernel<DT, DD>),              \
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)impact_lds_bytes<DT, DD>()); \
            return e == hipSuccess ? KVS_OK : fail(KVS_EHIP, "kvs_first_order_impact: hipFuncSetAttribute: %s", hipGetErrorString(e)); \
        });                                                                                                               \
        if (st != KVS_OK) return st;                                                                                      \
        hipLaunchKernelGGL((impact_kernel<DT, DD>), grid, block, (impact_lds_bytes<DT, DD>()), hs, n, shape->n_q_heads,         \
                           shape->n_kv_heads, q, k_fresh, v_fresh, k_cache, v_cache, h_fresh, lse, scale, part);          \
    } while (0)
    if (shape->dtype == KVS_BF16 && shape->head_dim == 128) KVS_IMP(KVS_BF16, 128);
    else if (shape->dtype == KVS_BF16 && shape->head_dim == 64) KVS_IMP(KVS_BF16, 64);
    else if (shape->dtype == KVS_F32 && shape->head_dim == 128) KVS_IMP(KVS_F32, 128);
    else KVS_IMP(KVS_F32, 64);
#undef KVS_IMP
    if ((st = check_launch("kvs_first_order_impact")) != KVS_OK) return st;
    hipLaunchKernelGGL(impact_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, hs, n, shape->n_kv_heads, part, reused,
                       impact_v, impact_k, impact_kv);
    return check_launch("kvs_first_order_impact(reduce)");
}
