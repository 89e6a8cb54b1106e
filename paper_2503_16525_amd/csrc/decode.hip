// kvs_decode_check: decode-stage re-scoring of the reuse candidates (Sec. 4.2).  The new
// token's attention row over its whole context replaces the prefill column mass of Alg. 1:
//     score_i = sum_g ( sum_{h in g} softmax_i(scale * q_h . K_i) ) * dev_v[g,i]
//
// Kernels, all on the caller's stream:
//   1. logits     streams K once (16-byte pieces, LPH lanes per (token, kv head) cell, the group's
//                 query slices in registers, DPP reduction as in the deviation kernel), writes
//                 scale*q.K for every query head to the workspace as fp32 [n_q_heads][n_rows] and
//                 the (max, sum exp) of each 64-token tile;
//   2. stats      per (request, head): merges the tile partials into the softmax max / normaliser;
//   3. score      per token: normalised weights summed per group, times the stored deviation,
//                 masked to the candidates;
//   4. select     the same exact top-k kernel as kvs_select_topk, one row per request;
//   5. attn_out   (optional) sum_i a[h,i] * V_i.
#include "kvs_internal.h"
#include "attention.h"

#include <math.h>

namespace kvs {
namespace {

constexpr int kThreads = 256;
constexpr int kTok = 64;          // tokens per workgroup in the logits kernel (= one wavefront in the partials step)
constexpr int kMaxReq = kAttnMaxReq;

struct DecodeBatch {
    int64_t ctx_off[kMaxReq];
    int32_t ctx_len[kMaxReq];
    int32_t tile_begin[kMaxReq + 1];  // first token tile (of kTok) of request b in this launch's grid
    int32_t req0;                     // global index of the first request of this launch
    int32_t n_req;
};

// ---- 1. logits + per-tile softmax partials ---------------------------------------------------------
// LPH lanes per (token, kv head) cell (head_dim * elem / 16 bytes); EPL = elements per 16-byte piece.
// GRP > 0: the group size is a compile-time constant and every lane group always meets the same KV
// head (cells per step is a multiple of n_kv_heads), so its slice of the group's queries lives in
// registers.  GRP == 0: generic shapes, queries are read from LDS.
template <int DTYPE, int EPL>
__device__ __forceinline__ void unpack_piece(const uint4 w, float (&kx)[EPL])
{
    if constexpr (DTYPE == KVS_BF16) {
        kx[0] = bf16_lo(w.x); kx[1] = bf16_hi(w.x); kx[2] = bf16_lo(w.y); kx[3] = bf16_hi(w.y);
        kx[4] = bf16_lo(w.z); kx[5] = bf16_hi(w.z); kx[6] = bf16_lo(w.w); kx[7] = bf16_hi(w.w);
    } else {
        kx[0] = __uint_as_float(w.x); kx[1] = __uint_as_float(w.y);
        kx[2] = __uint_as_float(w.z); kx[3] = __uint_as_float(w.w);
    }
}

template <int LPH>
__device__ __forceinline__ float cell_sum(float acc)
{
    if (LPH == 16) return row16_sum(acc);
    if (LPH == 32) { acc = row16_sum(acc); return acc + __shfl_xor(acc, 16); }
    acc += __shfl_xor(acc, 4);
    acc += __shfl_xor(acc, 2);
    return acc + __shfl_xor(acc, 1);
}

template <int DTYPE, int LPH, int GRP>
__global__ __launch_bounds__(kThreads) void decode_logits_kernel(
    const DecodeBatch bd, int n_q_heads, int n_kv_heads, int64_t n_rows,
    const void *__restrict__ q_new, const uint4 *__restrict__ k_cache, float scale,
    float *__restrict__ logits, float2 *__restrict__ partial /* [tile][n_q_heads] (max, sum exp) */)
{
    constexpr int EPL = DTYPE == KVS_BF16 ? 8 : 4;
    constexpr int D = LPH * EPL;
#ifndef KVS_DEC_UNROLL
#define KVS_DEC_UNROLL 8
#endif
    constexpr int UNROLL = KVS_DEC_UNROLL;
    extern __shared__ float lds[];
    float *lg_s = lds;                             // [n_q_heads][kTok]
    float *q_s = lds + n_q_heads * kTok;           // [n_q_heads][D], pre-multiplied by scale (GRP == 0 only)

    int b = 0;
    while (b + 1 < bd.n_req && (int)blockIdx.x >= bd.tile_begin[b + 1]) ++b;
    const int tile = blockIdx.x - bd.tile_begin[b];
    const int len = bd.ctx_len[b];
    const int tok0 = tile * kTok;
    const int tile_tok = min(kTok, len - tok0);
    const int64_t row0 = bd.ctx_off[b] + tok0;
    const int grp = GRP > 0 ? GRP : n_q_heads / n_kv_heads;
    const int tid = threadIdx.x;
    constexpr int CPB = kThreads / LPH;             // cells per step
    const int sub = tid % LPH, cell_in_step = tid / LPH;
    const int tile_cells = tile_tok * n_kv_heads;
    const int64_t q_base = (int64_t)(bd.req0 + b) * n_q_heads * D;

    auto load_q = [&](int64_t gi) -> float {
        if (DTYPE == KVS_F32) return ((const float *)q_new)[gi] * scale;
        return __uint_as_float((uint32_t)((const uint16_t *)q_new)[gi] << 16) * scale;
    };

    constexpr int GR = GRP > 0 ? GRP : 1;
    float qr[GR][EPL];
    if constexpr (GRP > 0) {
        const int g = cell_in_step % n_kv_heads;   // fixed: CPB is a multiple of n_kv_heads
#pragma unroll
        for (int hh = 0; hh < GRP; ++hh)
#pragma unroll
            for (int i = 0; i < EPL; ++i) qr[hh][i] = load_q(q_base + (int64_t)(g * GRP + hh) * D + sub * EPL + i);
    } else {
        for (int e = tid; e < n_q_heads * D; e += kThreads) q_s[e] = load_q(q_base + e);
        __syncthreads();
    }

    for (int base = 0; base < tile_cells; base += CPB * UNROLL) {
        uint4 w[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int c = base + u * CPB + cell_in_step;
            if (c < tile_cells) {
                const int t = c / n_kv_heads, g = c - t * n_kv_heads;
                w[u] = stream_load16(k_cache + ((row0 + t) * n_kv_heads + g) * LPH + sub);
            } else {
                w[u] = make_uint4(0, 0, 0, 0);
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int c = base + u * CPB + cell_in_step;
            const bool live = c < tile_cells;
            const int t = live ? c / n_kv_heads : 0;
            const int g = live ? c - t * n_kv_heads : 0;
            float kx[EPL];
            unpack_piece<DTYPE, EPL>(w[u], kx);
            if constexpr (GRP > 0) {
#pragma unroll
                for (int hh = 0; hh < GRP; ++hh) {
                    float acc = 0.f;
#pragma unroll
                    for (int i = 0; i < EPL; ++i) acc = fmaf(qr[hh][i], kx[i], acc);
                    acc = cell_sum<LPH>(acc);
                    if (live && sub == 0) lg_s[(g * GRP + hh) * kTok + t] = acc;
                }
            } else {
                for (int hh = 0; hh < grp; ++hh) {
                    const float *qh = q_s + (g * grp + hh) * D + sub * EPL;
                    float acc = 0.f;
#pragma unroll
                    for (int i = 0; i < EPL; ++i) acc = fmaf(qh[i], kx[i], acc);
                    acc = cell_sum<LPH>(acc);
                    if (live && sub == 0) lg_s[(g * grp + hh) * kTok + t] = acc;
                }
            }
        }
    }
    __syncthreads();
    for (int e = tid; e < n_q_heads * kTok; e += kThreads) {
        const int h = e / kTok, t = e % kTok;
        if (t < tile_tok) logits[(int64_t)h * n_rows + row0 + t] = lg_s[e];
    }
    // softmax partials of this tile: wave w takes heads w, w+4, ...; lane = token
    const int lane = tid & 63, wave = tid >> 6;
    for (int h = wave; h < n_q_heads; h += kThreads / 64) {
        const float x = lane < tile_tok ? lg_s[h * kTok + lane] : -INFINITY;
        const float m = wave_max(x);
        const float z = wave_sum(lane < tile_tok ? expf(x - m) : 0.f);
        if (lane == 0) partial[(int64_t)blockIdx.x * n_q_heads + h] = make_float2(m, z);
    }
}

// ---- 2. softmax statistics per (request, head): merge the tile partials ------------------------------
__global__ __launch_bounds__(kThreads) void decode_stats_kernel(
    const DecodeBatch bd, int n_q_heads, const float2 *__restrict__ partial,
    float2 *__restrict__ stats /* [batch][n_q_heads] (max, sum) */)
{
    __shared__ float red[kThreads / 64];
    __shared__ float bc;
    const int b = blockIdx.x / n_q_heads, h = blockIdx.x % n_q_heads;
    const int t0 = bd.tile_begin[b], t1 = bd.tile_begin[b + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float m = -INFINITY;
    for (int t = t0 + tid; t < t1; t += kThreads) m = fmaxf(m, partial[(int64_t)t * n_q_heads + h].x);
    m = wave_max(m);
    if (lane == 0) red[wave] = m;
    __syncthreads();
    if (tid == 0) { float x = red[0]; for (int w = 1; w < kThreads / 64; ++w) x = fmaxf(x, red[w]); bc = x; }
    __syncthreads();
    m = bc;
    float z = 0.f;
    for (int t = t0 + tid; t < t1; t += kThreads) {
        const float2 p = partial[(int64_t)t * n_q_heads + h];
        z += p.y * expf(p.x - m);
    }
    z = wave_sum(z);
    __syncthreads();
    if (lane == 0) red[wave] = z;
    __syncthreads();
    if (tid == 0) {
        float x = 0.f;
        for (int w = 0; w < kThreads / 64; ++w) x += red[w];
        stats[(int64_t)(bd.req0 + b) * n_q_heads + h] = make_float2(m, x);
    }
}

// ---- 3. scores ---------------------------------------------------------------------------------
// One workgroup per kTok-token tile: lane = token, wave w takes KV heads w, w+4, ...; the waves'
// partial sums are added in a fixed order.
__global__ __launch_bounds__(kThreads) void decode_score_kernel(
    const DecodeBatch bd, int n_q_heads, int n_kv_heads, int64_t n_rows,
    const float *__restrict__ logits, const float2 *__restrict__ stats,
    const float *__restrict__ dev_v, const uint8_t *__restrict__ reused, float *__restrict__ score)
{
    static_assert(kTok == 64, "one token per lane");
    constexpr int NW = kThreads / 64;
    __shared__ float part[NW][kTok];
    int b = 0;
    while (b + 1 < bd.n_req && (int)blockIdx.x >= bd.tile_begin[b + 1]) ++b;
    const int tile = blockIdx.x - bd.tile_begin[b];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = tile * kTok + lane;
    const bool live = i < bd.ctx_len[b];
    const int64_t row = bd.ctx_off[b] + min(i, bd.ctx_len[b] - 1);
    const int grp = n_q_heads / n_kv_heads;
    const float2 *st = stats + (int64_t)(bd.req0 + b) * n_q_heads;
    float s = 0.f;
    for (int g = wave; g < n_kv_heads; g += NW) {
        float mass = 0.f;
        for (int hh = 0; hh < grp; ++hh) {
            const int h = g * grp + hh;
            const float2 ms = st[h];
            mass += __builtin_amdgcn_exp2f((logits[(int64_t)h * n_rows + row] - ms.x) * 1.4426950408889634f) * (1.0f / ms.y);
        }
        s += mass * dev_v[(int64_t)g * n_rows + row];
    }
    part[wave][lane] = s;
    __syncthreads();
    if (wave == 0 && live) {
        float t = part[0][lane];
#pragma unroll
        for (int w = 1; w < NW; ++w) t += part[w][lane];
        const bool cand = reused ? reused[row] != 0 : true;
        score[row] = cand ? t : -INFINITY;
    }
}

// ---- 5. optional decode attention output -------------------------------------------------------
// one workgroup per (request, kv head); thread = (half, channel); tokens split even/odd over halves
template <int DTYPE, int D>
__global__ __launch_bounds__(kThreads) void decode_attn_kernel(
    const DecodeBatch bd, int n_q_heads, int n_kv_heads, int64_t n_rows,
    const float *__restrict__ logits, const float2 *__restrict__ stats,
    const void *__restrict__ v_cache, void *__restrict__ attn_out)
{
    constexpr int MAXG = 8;
    constexpr int PARTS = kThreads / D;
    __shared__ float part[PARTS][MAXG][D];
    const int b = blockIdx.x / n_kv_heads, g = blockIdx.x % n_kv_heads;
    const int len = bd.ctx_len[b];
    const int64_t row0 = bd.ctx_off[b];
    const int grp = n_q_heads / n_kv_heads;
    const int c = threadIdx.x % D, part_id = threadIdx.x / D;
    const float2 *st = stats + (int64_t)(bd.req0 + b) * n_q_heads;
    for (int h0 = 0; h0 < grp; h0 += MAXG) {
        const int nh = min(MAXG, grp - h0);
        float acc[MAXG];
        float mx[MAXG], inv[MAXG];
#pragma unroll
        for (int hh = 0; hh < MAXG; ++hh) {
            acc[hh] = 0.f;
            const float2 ms = hh < nh ? st[g * grp + h0 + hh] : make_float2(0.f, 1.f);
            mx[hh] = ms.x;
            inv[hh] = 1.0f / ms.y;
        }
        for (int i = part_id; i < len; i += PARTS) {
            const int64_t gi = ((row0 + i) * n_kv_heads + g) * (int64_t)D + c;
            float v;
            if (DTYPE == KVS_F32) v = ((const float *)v_cache)[gi];
            else v = __uint_as_float((uint32_t)((const uint16_t *)v_cache)[gi] << 16);
#pragma unroll
            for (int hh = 0; hh < MAXG; ++hh)
                if (hh < nh) acc[hh] += expf(logits[(int64_t)(g * grp + h0 + hh) * n_rows + row0 + i] - mx[hh]) * inv[hh] * v;
        }
#pragma unroll
        for (int hh = 0; hh < MAXG; ++hh) part[part_id][hh][c] = acc[hh];
        __syncthreads();
        if (part_id == 0) {
            for (int hh = 0; hh < nh; ++hh) {
                float s = 0.f;
                for (int pp = 0; pp < PARTS; ++pp) s += part[pp][hh][c];
                const int64_t oi = ((int64_t)(bd.req0 + b) * n_q_heads + g * grp + h0 + hh) * D + c;
                if (DTYPE == KVS_F32) ((float *)attn_out)[oi] = s;
                else ((uint16_t *)attn_out)[oi] = (uint16_t)f32_to_bf16_bits(s);
            }
        }
        __syncthreads();
    }
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

} // namespace

size_t decode_workspace_bytes(const kvs_shape *shape, int32_t batch, int64_t n_rows)
{
    size_t logits = align_up(sizeof(float) * (size_t)shape->n_q_heads * (size_t)n_rows, 256);
    size_t stats = align_up(sizeof(float2) * (size_t)batch * (size_t)shape->n_q_heads, 256);
    size_t score = align_up(sizeof(float) * (size_t)n_rows, 256);
    size_t partial = align_up(sizeof(float2) * ((size_t)n_rows / kTok + (size_t)batch + 1) * (size_t)shape->n_q_heads, 256);
    return logits + stats + score + partial;
}

} // namespace kvs

extern "C" kvs_status kvs_decode_check(const kvs_shape *shape, int32_t batch, int64_t n_rows,
                                       const int64_t *ctx_off, const int64_t *ctx_len,
                                       const void *q_new, const void *k_cache, const void *v_cache,
                                       const float *dev_v, const uint8_t *reused, float scale,
                                       const int32_t *k_req, int32_t *idx_out, float *score_out,
                                       void *attn_out,
                                       void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace kvs;
    kvs_status st = check_shape(shape);
    if (st != KVS_OK) return st;
    if (batch < 0 || n_rows < 0) return fail(KVS_EINVAL, "kvs_decode_check: negative size");
    if (batch == 0) return KVS_OK;
    if (!ctx_off || !ctx_len || !k_req) return fail(KVS_EINVAL, "kvs_decode_check: ctx_off/ctx_len/k_req is NULL");
    if (!q_new || !k_cache || !dev_v) return fail(KVS_EINVAL, "kvs_decode_check: q_new/k_cache/dev_v is NULL");
    if (attn_out && !v_cache) return fail(KVS_EINVAL, "kvs_decode_check: attn_out needs v_cache");
    if (!aligned16(k_cache) || (v_cache && !aligned16(v_cache))) return fail(KVS_EINVAL, "kvs_decode_check: K/V pointers must be 16-byte aligned");
    int64_t total_k = 0;
    for (int32_t b = 0; b < batch; ++b) {
        if (ctx_off[b] < 0 || ctx_len[b] < 0 || ctx_off[b] + ctx_len[b] > n_rows)
            return fail(KVS_EINVAL, "kvs_decode_check: request %d context [%lld,+%lld) outside the %lld cache rows", b, (long long)ctx_off[b], (long long)ctx_len[b], (long long)n_rows);
        if (ctx_len[b] > 0x7fffffffLL) return fail(KVS_EINVAL, "kvs_decode_check: request %d context too long", b);
        if (k_req[b] < 0 || k_req[b] > ctx_len[b]) return fail(KVS_EINVAL, "kvs_decode_check: k_req[%d]=%d outside [0,%lld]", b, k_req[b], (long long)ctx_len[b]);
        if (ctx_len[b] == 0 && attn_out) return fail(KVS_EINVAL, "kvs_decode_check: attn_out with an empty context (request %d)", b);
        total_k += k_req[b];
    }
    if (total_k > 0 && !idx_out) return fail(KVS_EINVAL, "kvs_decode_check: idx_out is NULL");
    if (shape->n_q_heads > 256) return fail(KVS_EUNSUPPORTED, "kvs_decode_check: more than 256 query heads");
    const size_t need = decode_workspace_bytes(shape, batch, n_rows);
    if (!workspace || workspace_bytes < need) return fail(KVS_EWORKSPACE, "kvs_decode_check: workspace %zu < %zu bytes", workspace_bytes, need);
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(KVS_EINVAL, "kvs_decode_check: workspace must be 256-byte aligned");

    hipStream_t hs = (hipStream_t)stream;
    const int hq = shape->n_q_heads, hk = shape->n_kv_heads, d = shape->head_dim;
    char *ws = (char *)workspace;
    float *logits = (float *)ws;
    ws += align_up(sizeof(float) * (size_t)hq * (size_t)n_rows, 256);
    float2 *stats = (float2 *)ws;
    ws += align_up(sizeof(float2) * (size_t)batch * (size_t)hq, 256);
    float *score = score_out ? score_out : (float *)ws;
    ws += align_up(sizeof(float) * (size_t)n_rows, 256);
    float2 *partial = (float2 *)ws;
    const int lph = (int)(d * elem_bytes(shape->dtype) / 16);

    for (int32_t b0 = 0; b0 < batch; b0 += kMaxReq) {
        const int nr = (batch - b0) < kMaxReq ? (batch - b0) : kMaxReq;
        DecodeBatch bd_tok;   // tile table for kTok-token tiles
        int64_t tiles_tok = 0;
        for (int i = 0; i < kMaxReq; ++i) {
            const bool live = i < nr;
            const int64_t len = live ? ctx_len[b0 + i] : 0;
            bd_tok.ctx_off[i] = live ? ctx_off[b0 + i] : 0;
            bd_tok.ctx_len[i] = (int32_t)len;
            bd_tok.tile_begin[i] = (int32_t)tiles_tok;
            tiles_tok += (len + kTok - 1) / kTok;
            if (tiles_tok > 0x7fffffffLL) return fail(KVS_EINVAL, "kvs_decode_check: too many tokens in one launch");
        }
        bd_tok.tile_begin[kMaxReq] = (int32_t)tiles_tok;
        bd_tok.req0 = b0;
        bd_tok.n_req = nr;
        if (tiles_tok == 0) continue;
        const int grp = hq / hk;
        const bool regq = (kThreads / lph) % hk == 0;   // every lane group keeps one kv head
        const size_t lds = sizeof(float) * (size_t)hq * (kTok + (regq ? 0 : d));
        dim3 block(kThreads);
        // partials of this launch start at the launch's first tile: offset the pointer so that the
        // kernel can index by blockIdx
        float2 *part_l = partial;
#define KVS_DEC_LAUNCH(DT, L, G) hipLaunchKernelGGL((decode_logits_kernel<DT, L, G>), dim3((unsigned)tiles_tok), block, lds, hs, bd_tok, hq, hk, n_rows, q_new, (const uint4 *)k_cache, scale, logits, part_l)
#define KVS_DEC_CASE(DT, L)                                                    \
    do {                                                                       \
        if (regq && grp == 1) KVS_DEC_LAUNCH(DT, L, 1);                        \
        else if (regq && grp == 2) KVS_DEC_LAUNCH(DT, L, 2);                   \
        else if (regq && grp == 4) KVS_DEC_LAUNCH(DT, L, 4);                   \
        else if (regq && grp == 7) KVS_DEC_LAUNCH(DT, L, 7);                   \
        else if (regq && grp == 8) KVS_DEC_LAUNCH(DT, L, 8);                   \
        else KVS_DEC_LAUNCH(DT, L, 0);                                         \
    } while (0)
        if (shape->dtype == KVS_BF16 && lph == 16) KVS_DEC_CASE(KVS_BF16, 16);
        else if (shape->dtype == KVS_BF16 && lph == 8) KVS_DEC_CASE(KVS_BF16, 8);
        else if (shape->dtype == KVS_F32 && lph == 16) KVS_DEC_CASE(KVS_F32, 16);
        else if (shape->dtype == KVS_F32 && lph == 32) KVS_DEC_CASE(KVS_F32, 32);
        else return fail(KVS_EUNSUPPORTED, "kvs_decode_check: head_dim %d", d);
#undef KVS_DEC_CASE
#undef KVS_DEC_LAUNCH
        if ((st = check_launch("kvs_decode_check(logits)")) != KVS_OK) return st;
        hipLaunchKernelGGL(decode_stats_kernel, dim3((unsigned)(nr * hq)), block, 0, hs, bd_tok, hq, part_l, stats);
        if ((st = check_launch("kvs_decode_check(stats)")) != KVS_OK) return st;
        hipLaunchKernelGGL(decode_score_kernel, dim3((unsigned)tiles_tok), block, 0, hs, bd_tok, hq, hk, n_rows,
                           logits, stats, dev_v, reused, score);
        if ((st = check_launch("kvs_decode_check(score)")) != KVS_OK) return st;
        if (attn_out) {
            dim3 grid((unsigned)(nr * hk));
            if (shape->dtype == KVS_BF16 && d == 128) hipLaunchKernelGGL((decode_attn_kernel<KVS_BF16, 128>), grid, block, 0, hs, bd_tok, hq, hk, n_rows, logits, stats, v_cache, attn_out);
            else if (shape->dtype == KVS_BF16 && d == 64) hipLaunchKernelGGL((decode_attn_kernel<KVS_BF16, 64>), grid, block, 0, hs, bd_tok, hq, hk, n_rows, logits, stats, v_cache, attn_out);
            else if (shape->dtype == KVS_F32 && d == 128) hipLaunchKernelGGL((decode_attn_kernel<KVS_F32, 128>), grid, block, 0, hs, bd_tok, hq, hk, n_rows, logits, stats, v_cache, attn_out);
            else hipLaunchKernelGGL((decode_attn_kernel<KVS_F32, 64>), grid, block, 0, hs, bd_tok, hq, hk, n_rows, logits, stats, v_cache, attn_out);
            if ((st = check_launch("kvs_decode_check(attn)")) != KVS_OK) return st;
        }
    }
    if (total_k == 0) return KVS_OK;
    return launch_select(score, batch, ctx_off, ctx_len, k_req, idx_out, hs);
}
