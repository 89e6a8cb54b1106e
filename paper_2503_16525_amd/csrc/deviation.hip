// kvs_deviation: per-token, per-KV-head L1 deviation of the reused cache from freshly computed
// K/V, and the deviation impact score of Alg. 1 step 3 / Eq. (3).
//
// The kernel is a pure HBM stream: each (token, kv head) cell is one contiguous run of
// head_dim elements, consecutive cells are contiguous in memory, so the whole tensor is read
// as a flat sequence of 16-byte pieces, one per lane, LPH lanes per cell.  The LPH partial
// sums are combined with DPP row rotations (fixed order, no atomics), parked in LDS as
// [head][token-in-tile] and written out head-major so that dev_* and score stores are
// coalesced along the token axis.
#include "kvs_internal.h"

#include <math.h>

namespace kvs {
namespace {

constexpr int kDevThreads = 256;
constexpr int kDevTok = 32; // tokens per workgroup tile

template <int DTYPE>
__device__ __forceinline__ float l1_piece(const uint4 a, const uint4 b)
{
    if (DTYPE == KVS_BF16) {
        float s0 = fabsf(bf16_lo(a.x) - bf16_lo(b.x)) + fabsf(bf16_hi(a.x) - bf16_hi(b.x));
        float s1 = fabsf(bf16_lo(a.y) - bf16_lo(b.y)) + fabsf(bf16_hi(a.y) - bf16_hi(b.y));
        float s2 = fabsf(bf16_lo(a.z) - bf16_lo(b.z)) + fabsf(bf16_hi(a.z) - bf16_hi(b.z));
        float s3 = fabsf(bf16_lo(a.w) - bf16_lo(b.w)) + fabsf(bf16_hi(a.w) - bf16_hi(b.w));
        return (s0 + s1) + (s2 + s3);
    } else {
        float s0 = fabsf(__uint_as_float(a.x) - __uint_as_float(b.x));
        float s1 = fabsf(__uint_as_float(a.y) - __uint_as_float(b.y));
        float s2 = fabsf(__uint_as_float(a.z) - __uint_as_float(b.z));
        float s3 = fabsf(__uint_as_float(a.w) - __uint_as_float(b.w));
        return (s0 + s1) + (s2 + s3);
    }
}

template <int LPH>
__device__ __forceinline__ float group_sum(float v)
{
    if (LPH == 16) return row16_sum(v);
    if (LPH == 32) { v = row16_sum(v); return v + __shfl_xor(v, 16); }
    // LPH == 8
    v += __shfl_xor(v, 4);
    v += __shfl_xor(v, 2);
    v += __shfl_xor(v, 1);
    return v;
}

__device__ __forceinline__ uint4 stream_load(const uint4 *p) { return stream_load16(p); }

// One workgroup = kDevTok consecutive tokens = kDevTok * n_kv_heads cells.
// HIST (kvs_deviation_topk): every token's order-preserving key is stored beside its score and
// counted into the histogram of the keys' leading bits (finite scores only), which the selecting
// kernel consumes.
template <int DTYPE, int LPH, bool HAS_K, int UNROLL, bool HIST>
__global__ __launch_bounds__(kDevThreads) void deviation_kernel(
    int64_t n_tokens, int n_kv_heads,
    const uint4 *__restrict__ k_fresh, const uint4 *__restrict__ v_fresh,
    const uint4 *__restrict__ k_cache, const uint4 *__restrict__ v_cache,
    const uint8_t *__restrict__ reused, const float *__restrict__ alpha, int mode_kv,
    float *__restrict__ dev_k, float *__restrict__ dev_v, float *__restrict__ score,
    uint32_t *__restrict__ keys_out, uint32_t *__restrict__ key_hist)
{
    extern __shared__ float lds[]; // dv[n_kv_heads][kDevTok], then dk[n_kv_heads][kDevTok]
    float *dv_s = lds;
    float *dk_s = lds + n_kv_heads * kDevTok;

    constexpr int CPW = kWave / LPH;                    // cells per wave per step
    constexpr int CPB = CPW * (kDevThreads / kWave);    // cells per workgroup per step
    const int tid = threadIdx.x;
    const int sub = tid % LPH;                          // 16-byte piece within the cell
    const int cell_in_step = tid / LPH;
    const int64_t tok0 = (int64_t)blockIdx.x * kDevTok;
    const int tile_tok = (int)min((int64_t)kDevTok, n_tokens - tok0);
    const int tile_cells = tile_tok * n_kv_heads;
    const int64_t cell0 = tok0 * n_kv_heads;

    for (int base = 0; base < tile_cells; base += CPB * UNROLL) {
        uint4 vf[UNROLL], vc[UNROLL], kf[UNROLL], kc[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int c = base + u * CPB + cell_in_step;
            if (c < tile_cells) {
                const int64_t piece = (cell0 + c) * LPH + sub;
                vf[u] = stream_load(v_fresh + piece);
                vc[u] = stream_load(v_cache + piece);
                if (HAS_K) {
                    kf[u] = stream_load(k_fresh + piece);
                    kc[u] = stream_load(k_cache + piece);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int c = base + u * CPB + cell_in_step;   // uniform over the LPH lanes of a cell
            float sv = 0.f, sk = 0.f;
            if (c < tile_cells) {
                sv = l1_piece<DTYPE>(vf[u], vc[u]);
                if (HAS_K) sk = l1_piece<DTYPE>(kf[u], kc[u]);
            }
            sv = group_sum<LPH>(sv);
            if (HAS_K) sk = group_sum<LPH>(sk);
            if (c < tile_cells && sub == 0) {
                const int t = c / n_kv_heads, g = c - t * n_kv_heads;
                dv_s[g * kDevTok + t] = sv;
                if (HAS_K) dk_s[g * kDevTok + t] = sk;
            }
        }
    }
    __syncthreads();

    for (int e = tid; e < n_kv_heads * kDevTok; e += kDevThreads) {
        const int g = e / kDevTok, t = e % kDevTok;
        if (t < tile_tok) {
            const int64_t o = (int64_t)g * n_tokens + tok0 + t;
            if (dev_v) dev_v[o] = dv_s[e];
            if (HAS_K && dev_k) dev_k[o] = dk_s[e];
        }
    }
    if ((score || HIST) && tid < tile_tok) {
        const int64_t i = tok0 + tid;
        float s = 0.f;
        for (int g = 0; g < n_kv_heads; ++g) {
            float dev = dv_s[g * kDevTok + tid];
            if (HAS_K && mode_kv) dev = dk_s[g * kDevTok + tid] + dev;
            const float a = alpha ? alpha[(int64_t)g * n_tokens + i] : 1.0f;
            s += a * dev;
        }
        const bool cand = reused ? (reused[i] != 0) : true;
        const float sc = cand ? s : -INFINITY;
        if (score) score[i] = sc;
        if (HIST) {
            const uint32_t key = score_key(sc);
            keys_out[i] = key;
            key_hist_count<false>(key_hist, key, sc != -INFINITY);
        }
    }
}

template <int DTYPE, int LPH>
kvs_status launch(int64_t n, int hk, bool has_k, const void *kf, const void *vf, const void *kc,
                  const void *vc, const uint8_t *reused, const float *alpha, int mode_kv,
                  float *dev_k, float *dev_v, float *score, const FusedScratch *fs, hipStream_t st)
{
    const int64_t blocks = (n + kDevTok - 1) / kDevTok;
    if (blocks > 0x7fffffff) return fail(KVS_EINVAL, "kvs_deviation: too many tokens");
    const size_t lds = sizeof(float) * hk * kDevTok * 2;
    dim3 grid((unsigned)blocks), block(kDevThreads);
#define KVS_DEV_LAUNCH(HASK, UNR, HIST)                                                                          \
    hipLaunchKernelGGL((deviation_kernel<DTYPE, LPH, HASK, UNR, HIST>), grid, block, lds, st, n, hk,             \
                       (const uint4 *)kf, (const uint4 *)vf, (const uint4 *)kc, (const uint4 *)vc, reused, alpha, \
                       mode_kv, dev_k, dev_v, score, fs ? fs->keys : nullptr, fs ? fs->hist : nullptr)
    if (has_k) { if (fs) KVS_DEV_LAUNCH(true, 2, true); else KVS_DEV_LAUNCH(true, 2, false); }
    else { if (fs) KVS_DEV_LAUNCH(false, 4, true); else KVS_DEV_LAUNCH(false, 4, false); }
#undef KVS_DEV_LAUNCH
    return check_launch("kvs_deviation");
}

kvs_status deviation_call(const char *who, const kvs_shape *shape, int64_t n_tokens,
                          const void *k_fresh, const void *v_fresh, const void *k_cache, const void *v_cache,
                          const uint8_t *reused, const float *alpha, int32_t mode,
                          float *dev_k, float *dev_v, float *score, const FusedScratch *fs, hipStream_t hs)
{
    kvs_status st = check_shape(shape);
    if (st != KVS_OK) return st;
    if (n_tokens < 0) return fail(KVS_EINVAL, "%s: n_tokens < 0", who);
    if (mode != KVS_SCORE_V && mode != KVS_SCORE_KV) return fail(KVS_EINVAL, "%s: bad mode %d", who, mode);
    if (n_tokens == 0) return KVS_OK;
    if (!v_fresh || !v_cache) return fail(KVS_EINVAL, "%s: v_fresh/v_cache is NULL", who);
    const bool has_k = (mode == KVS_SCORE_KV) || dev_k != nullptr;
    if (has_k && (!k_fresh || !k_cache)) return fail(KVS_EINVAL, "%s: k_fresh/k_cache is NULL but the key deviation is needed", who);
    if (!aligned16(v_fresh) || !aligned16(v_cache) || (has_k && (!aligned16(k_fresh) || !aligned16(k_cache))))
        return fail(KVS_EINVAL, "%s: K/V pointers must be 16-byte aligned", who);
    if (shape->n_kv_heads > 64) return fail(KVS_EUNSUPPORTED, "%s: more than 64 kv heads", who);
    const int lph = (int)(shape->head_dim * elem_bytes(shape->dtype) / 16);
    const int mkv = mode == KVS_SCORE_KV;
    const int hk = shape->n_kv_heads;
#define KVS_DEV_CASE(DT, L) \
    return launch<DT, L>(n_tokens, hk, has_k, k_fresh, v_fresh, k_cache, v_cache, reused, alpha, mkv, dev_k, dev_v, score, fs, hs)
    if (shape->dtype == KVS_BF16) {
        if (lph == 8) KVS_DEV_CASE(KVS_BF16, 8);
        if (lph == 16) KVS_DEV_CASE(KVS_BF16, 16);
    } else {
        if (lph == 16) KVS_DEV_CASE(KVS_F32, 16);
        if (lph == 32) KVS_DEV_CASE(KVS_F32, 32);
    }
#undef KVS_DEV_CASE
    return fail(KVS_EUNSUPPORTED, "%s: head_dim %d with dtype %d", who, shape->head_dim, shape->dtype);
}

} // namespace
} // namespace kvs

extern "C" kvs_status kvs_deviation(const kvs_shape *shape, int64_t n_tokens,
                                    const void *k_fresh, const void *v_fresh,
                                    const void *k_cache, const void *v_cache,
                                    const uint8_t *reused, const float *alpha, int32_t mode,
                                    float *dev_k, float *dev_v, float *score, void *stream)
{
    return kvs::deviation_call("kvs_deviation", shape, n_tokens, k_fresh, v_fresh, k_cache, v_cache, reused, alpha, mode,
                               dev_k, dev_v, score, nullptr, (hipStream_t)stream);
}

extern "C" kvs_status kvs_deviation_topk(const kvs_shape *shape, int64_t n_tokens,
                                         const void *k_fresh, const void *v_fresh,
                                         const void *k_cache, const void *v_cache,
                                         const uint8_t *reused, const float *alpha, int32_t mode,
                                         float *dev_k, float *dev_v, float *score,
                                         int32_t k, int32_t *idx_out,
                                         void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace kvs;
    const char *who = "kvs_deviation_topk";
    if (n_tokens < 0) return fail(KVS_EINVAL, "%s: n_tokens < 0", who);
    if (k < 0 || k > n_tokens) return fail(KVS_EINVAL, "%s: k=%d outside [0,%lld]", who, k, (long long)n_tokens);
    if (k > 0 && !idx_out) return fail(KVS_EINVAL, "%s: idx_out is NULL", who);
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return fail(KVS_EINVAL, "%s: workspace must be 256-byte aligned", who);
    hipStream_t hs = (hipStream_t)stream;
    // (short rows: one workgroup ranks 8k scores in the time the two selecting launches take)
    if (k > 0 && n_tokens > kFusedMinTokens && n_tokens <= kFusedMaxTokens) {
        // scores, keys and the key histogram in one pass; one more launch turns them into the list
        FusedScratch fs;
        kvs_status st = fused_scratch(&fs);
        if (st != KVS_OK) return st;
        st = deviation_call(who, shape, n_tokens, k_fresh, v_fresh, k_cache, v_cache, reused, alpha, mode, dev_k, dev_v, score, &fs, hs);
        if (st != KVS_OK) return st;
        return launch_select_from_hist(fs, (int32_t)n_tokens, k, idx_out, hs);
    }
    // longer rows (and k = 0): the two calls one after the other; the ranking needs the scores in memory
    if (k > 0 && !score) return fail(KVS_EINVAL, "%s: rows of up to %d or above %d tokens need the score array", who, kFusedMinTokens, kFusedMaxTokens);
    kvs_status st = deviation_call(who, shape, n_tokens, k_fresh, v_fresh, k_cache, v_cache, reused, alpha, mode, dev_k, dev_v, score, nullptr, hs);
    if (st != KVS_OK || k == 0) return st;
    if (n_tokens > 0x7fffffffLL) return fail(KVS_EINVAL, "%s: row longer than 2^31-1", who);
    const int64_t begin = 0, len = n_tokens;
    return launch_select(score, 1, &begin, &len, &k, idx_out, workspace, workspace_bytes, hs);
}
