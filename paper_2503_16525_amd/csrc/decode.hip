// kvs_decode_check: decode-stage re-scoring of the reuse candidates (Sec. 4.2).  The new
// token's attention row over its whole context replaces the prefill column mass of Alg. 1:
//     score_i = sum_g ( sum_{h in g} softmax_i(scale * q_h . K_i) ) * dev_v[g,i]
//
// Kernels, all on the caller's stream:
//   1. logits     streams K once and writes scale*q.K for every query head to the workspace as fp32
//                 [n_q_heads][n_rows], plus the (max, sum exp) of each 64-token tile.  bf16 with
//                 head_dim 128: on the matrix cores, K loaded straight into LDS (1b below); other
//                 shapes: 16-byte pieces, LPH lanes per (token, kv head) cell, the group's query
//                 slices in registers, DPP reduction as in the deviation kernel;
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

// ---- 1b. the same on the matrix cores (bf16, head_dim 128, groups of up to 32 query heads) ----------
// The vector kernel above spends ~60 instructions per 16 bytes of K and tops out near half of
// the HBM rate; here q . K is one v_mfma_f32_32x32x16_bf16 chain per 32 tokens of a KV head: A =
// the group's query heads as rows (the unused rows are zero), B = the K rows as columns, so a
// lane's column of the result is one token and its first registers are that token's logits for
// the group's heads - stores of one head are 32 consecutive floats.  Only 1/8 of the matrix work
// is useful at a group of 4, which is irrelevant: the kernel has to be memory-bound, and is.
// K goes from global memory straight into LDS (buffer loads with the LDS flag and the
// non-temporal hint: the cache is read once; 1 KiB = four
// 256-byte rows per instruction, 16-byte pieces XOR-swizzled by the row so that the operand reads
// are conflict-free).  A workgroup is still one 64-token tile; wave w takes KV heads w, w+4, ..,
// each as two units of 32 tokens that it stages and consumes by itself through its own two LDS
// slots, so there is no barrier anywhere: a wave only waits for its own loads.
// workgroups of the matrix-core logits launch at most: beyond that each takes several 64-token tiles (64-request
// batch, 10.9k tiles: 335 us per check with 1024 workgroups against 344 us with one per tile; 512 and 2048: 340, 339)
#ifndef KVS_DEC_PERSIST
#define KVS_DEC_PERSIST 1024
#endif
constexpr int kMmaUnitBytes = 32 * 256;            // 32 tokens x 256 bytes
constexpr int kMmaSlots = 2;
constexpr int kMmaLds = (kThreads / 64) * kMmaSlots * kMmaUnitBytes;

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 dec_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float dec_floatx16;

// max / sum over the 32 lanes of a half-wave (lanes 0-31 or 32-63), result in each of them
__device__ __forceinline__ float half_max(float v)
{
    v = fmaxf(v, dpp_f32<0x128>(v));
    v = fmaxf(v, dpp_f32<0x124>(v));
    v = fmaxf(v, dpp_f32<0x122>(v));
    v = fmaxf(v, dpp_f32<0x121>(v));
    return fmaxf(v, __shfl_xor(v, 16));
}
__device__ __forceinline__ float half_sum(float v)
{
    v = row16_sum(v);
    return v + __shfl_xor(v, 16);
}

__global__ __launch_bounds__(kThreads) void decode_logits_mfma_kernel(
    const DecodeBatch bd, int n_q_heads, int n_kv_heads, int64_t n_rows,
    const uint16_t *__restrict__ q_new, const uint16_t *__restrict__ k_cache, float scale,
    float *__restrict__ logits, float2 *__restrict__ partial /* [tile][n_q_heads] (max, sum exp) */, int n_tiles)
{
    constexpr int D = 128, ROW_B = 256;
    extern __shared__ __attribute__((aligned(16))) char lds_mma[];
    // a workgroup takes tiles blockIdx.x, blockIdx.x + gridDim.x, ...: nothing below synchronises the waves, and
    // every wave leaves a tile with its own loads and LDS reads complete
    for (int tile_id = blockIdx.x; tile_id < n_tiles; tile_id += gridDim.x) {
    int b = 0;
    while (b + 1 < bd.n_req && tile_id >= bd.tile_begin[b + 1]) ++b;
    const int tile = tile_id - bd.tile_begin[b];
    const int len = bd.ctx_len[b];
    const int tok0 = tile * kTok;
    const int tile_tok = min(kTok, len - tok0);
    const int64_t row0 = bd.ctx_off[b] + tok0;
    const int grp = n_q_heads / n_kv_heads;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hf = lane >> 5, ln = lane & 31;
    const uint16_t *qb = q_new + (int64_t)(bd.req0 + b) * n_q_heads * D;

    // the whole cache as one buffer (the host checks that it is below 4 GiB)
    const uint32_t row_bytes = (uint32_t)n_kv_heads * ROW_B;
    u32x4_t rs;
    {
        const uint64_t a = reinterpret_cast<uint64_t>(k_cache);
        rs.x = __builtin_amdgcn_readfirstlane((uint32_t)a);
        rs.y = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
        rs.z = __builtin_amdgcn_readfirstlane((uint32_t)n_rows * row_bytes);
        rs.w = 0x00020000u;
    }
    char *const my_lds = lds_mma + wave * (kMmaSlots * kMmaUnitBytes);
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)my_lds);
    // staging: instruction j moves rows 4j .. 4j+3 of the unit; lane = (row in the four, position);
    // piece p of row r sits at position p ^ (r & 15)
    const int st_r = lane >> 4, st_p = lane & 15;
    // This wave's KV heads are wave, wave + 4, ...; they are taken two at a time, and the four units
    // of a pair go (head A, tokens 0-31), (head B, 0-31), (A, 32-63), (B, 32-63): with two units in
    // flight per wave the four waves together are then reading all heads of the same 32 token rows,
    // i.e. one contiguous stretch of the cache, instead of every other 256-byte chunk of it.
    const int n_heads_w = (n_kv_heads - wave + 3) / 4;
    const int n_units = 2 * n_heads_w;
    // unit u of the wave -> (index of the head among the wave's heads, token half)
    auto unit_head = [&](int u) { const int pair = u >> 2, k = u & 3; return (n_heads_w - 2 * pair >= 2) ? 2 * pair + (k & 1) : 2 * pair; };
    auto unit_sub = [&](int u) { const int pair = u >> 2, k = u & 3; return (n_heads_w - 2 * pair >= 2) ? (k >> 1) : (k & 1); };
    auto stage_unit = [&](int u) {
        const int g = wave + 4 * unit_head(u), sub = unit_sub(u);
        const uint32_t slot = lds_base + (uint32_t)((u & (kMmaSlots - 1)) * kMmaUnitBytes);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = 4 * j + st_r;
            const int t = min(32 * sub + r, tile_tok - 1);          // rows past the context: its last row
            const uint32_t voff = (uint32_t)(row0 + t) * row_bytes + (uint32_t)g * ROW_B + (uint32_t)((st_p ^ (r & 15)) * 16);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen nt lds"
                         :: "s"(__builtin_amdgcn_readfirstlane(slot + (uint32_t)(j * 1024))), "v"(voff), "s"(rs));
        }
    };
    // B operand: K row ln, pieces 2*ks + hf
    const uint32_t b_read_off = (uint32_t)(ln * ROW_B + ((hf ^ (ln & 15)) * 16));
    const dec_floatx16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    if (n_units > 0) stage_unit(0);
    if (n_units > 1) stage_unit(1);
    for (int pair = 0; 2 * pair < n_heads_w; ++pair) {
        const int heads_here = min(2, n_heads_w - 2 * pair);
        // A operands: query head g*grp + ln of each head of the pair (rows past the group are zero)
        dec_bf16x8 qa[2][D / 16];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int g = wave + 4 * (2 * pair + min(i, heads_here - 1));
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (ln < grp) v = *reinterpret_cast<const u32x4_t *>(qb + (int64_t)(g * grp + ln) * D + 16 * ks + 8 * hf);
                qa[i][ks] = __builtin_bit_cast(dec_bf16x8, v);
            }
        }
        dec_floatx16 x[2][2];      // [head of the pair][token half]
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (k < 2 * heads_here) {
                const int u = 4 * pair + k;
                const int i = heads_here == 2 ? (k & 1) : 0, sub = heads_here == 2 ? (k >> 1) : (k & 1);
                // this unit's eight loads are older than the next unit's eight
                if (u + 1 < n_units) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                const char *slot = my_lds + (u & (kMmaSlots - 1)) * kMmaUnitBytes;
                dec_floatx16 acc = zero;
#pragma unroll
                for (int ks = 0; ks < D / 16; ++ks) {
                    const u32x4_t kb = *reinterpret_cast<const u32x4_t *>(slot + (b_read_off ^ (uint32_t)(32 * ks)));
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(i == 0 ? qa[0][ks] : qa[1][ks], __builtin_bit_cast(dec_bf16x8, kb), acc, 0, 0, 0);
                }
                if (i == 0) { if (sub == 0) x[0][0] = acc; else x[0][1] = acc; }
                else { if (sub == 0) x[1][0] = acc; else x[1][1] = acc; }
                // the slot is free once its reads have returned; refill it with the unit after next
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                if (u + kMmaSlots < n_units) stage_unit(u + kMmaSlots);
            }
        }
        // register r of half-wave hf is query head 8*(r/4) + 4*hf + r%4 of the group, column = token
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (i < heads_here) {
                const int g = wave + 4 * (2 * pair + i);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int hh = 8 * (r >> 2) + 4 * hf + (r & 3);
                    if (hh < grp) {                                      // uniform per half-wave
                        const int h = g * grp + hh;
                        float v[2];
#pragma unroll
                        for (int sub = 0; sub < 2; ++sub) {
                            const int t = 32 * sub + ln;
                            v[sub] = x[i][sub][r] * scale;
                            if (t < tile_tok) logits[(int64_t)h * n_rows + row0 + t] = v[sub];
                            else v[sub] = -INFINITY;
                        }
                        const float m = half_max(fmaxf(v[0], v[1]));
                        const float z = half_sum(__expf(v[0] - m) + __expf(v[1] - m));
                        if (ln == 0) partial[(int64_t)tile_id * n_q_heads + h] = make_float2(m, z);
                    }
                }
            }
        }
    }
    }   // tiles of this workgroup
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
// One wave per kTok-token tile, lane = token: every load is 64 consecutive floats, there is no
// LDS and no barrier, and the sum over the KV heads runs in head order.  GRP > 0: the group size
// is a compile-time constant, so the loads of two KV heads are in flight together.
// HIST (one context whose top-k then runs from the histogram, as in kvs_deviation_topk): the token's
// order-preserving key goes to keys_out[token index in the context] and is counted by its leading bits.
template <int GRP, bool HIST>
__global__ __launch_bounds__(kThreads) void decode_score_kernel(
    const DecodeBatch bd, int n_tiles, int n_q_heads, int n_kv_heads, int64_t n_rows,
    const float *__restrict__ logits, const float2 *__restrict__ stats,
    const float *__restrict__ dev_v, const uint8_t *__restrict__ reused, float *__restrict__ score,
    uint32_t *__restrict__ keys_out, uint32_t *__restrict__ key_hist)
{
    static_assert(kTok == 64, "one token per lane");
    const int lane = threadIdx.x & 63;
    const int tile_id = __builtin_amdgcn_readfirstlane((int)blockIdx.x * (kThreads / 64) + (int)(threadIdx.x >> 6));
    if (tile_id >= n_tiles) return;
    int b = 0;
    while (b + 1 < bd.n_req && tile_id >= bd.tile_begin[b + 1]) ++b;
    const int tile = tile_id - bd.tile_begin[b];
    const int i = tile * kTok + lane;
    const bool live = i < bd.ctx_len[b];
    const int64_t row = bd.ctx_off[b] + min(i, bd.ctx_len[b] - 1);
    const float2 *st = stats + (int64_t)(bd.req0 + b) * n_q_heads;
    float s = 0.f;
    if constexpr (GRP > 0) {
        constexpr int GB = 2;                       // KV heads per batch of loads
        for (int g0 = 0; g0 < n_kv_heads; g0 += GB) {
            float lg[GB][GRP], dv[GB];
#pragma unroll
            for (int j = 0; j < GB; ++j) {
                const int g = min(g0 + j, n_kv_heads - 1);
#pragma unroll
                for (int hh = 0; hh < GRP; ++hh) lg[j][hh] = logits[(int64_t)(g * GRP + hh) * n_rows + row];
                dv[j] = dev_v[(int64_t)g * n_rows + row];
            }
#pragma unroll
            for (int j = 0; j < GB; ++j) {
                if (g0 + j < n_kv_heads) {
                    float mass = 0.f;
#pragma unroll
                    for (int hh = 0; hh < GRP; ++hh) {
                        const float2 ms = st[(g0 + j) * GRP + hh];
                        mass += __builtin_amdgcn_exp2f((lg[j][hh] - ms.x) * 1.4426950408889634f) * (1.0f / ms.y);
                    }
                    s += mass * dv[j];
                }
            }
        }
    } else {
        const int grp = n_q_heads / n_kv_heads;
        for (int g = 0; g < n_kv_heads; ++g) {
            float mass = 0.f;
            for (int hh = 0; hh < grp; ++hh) {
                const int h = g * grp + hh;
                const float2 ms = st[h];
                mass += __builtin_amdgcn_exp2f((logits[(int64_t)h * n_rows + row] - ms.x) * 1.4426950408889634f) * (1.0f / ms.y);
            }
            s += mass * dev_v[(int64_t)g * n_rows + row];
        }
    }
    if (live) {
        const bool cand = reused ? reused[row] != 0 : true;
        const float sc = cand ? s : -INFINITY;
        score[row] = sc;
        if (HIST) {
            const uint32_t key = score_key(sc);
            keys_out[i] = key;
            key_hist_count<true>(key_hist, key, sc != -INFINITY);
        }
    }
}

// ---- 5. optional decode attention output -------------------------------------------------------
// sum_i a[h, i] * V_i.  The V stream is cut into tiles of kAttTok tokens; a workgroup takes one
// tile of one KV head (LPH lanes per 256-byte row, 16 bytes per lane, several rows in flight per
// lane), computes the tile's weights once from the stored logits and the softmax statistics, and leaves the
// tile's share of the group's outputs in the workspace; a second kernel adds the tiles of a
// request in order.  (One workgroup per (request, KV head), as this used to be, took 14 ms for a
// single 32k context: eight workgroups on a 256-unit chip.)
constexpr int kAttTok = 256;
constexpr int kAttMaxG = 8;        // query heads of a group handled per sweep over V

template <int DTYPE, int LPH>
__global__ __launch_bounds__(kThreads) void decode_attn_partial_kernel(
    const DecodeBatch bd /* tile_begin counts kAttTok-token tiles */, int n_q_heads, int n_kv_heads, int64_t n_rows,
    const float *__restrict__ logits, const float2 *__restrict__ stats,
    const uint4 *__restrict__ v_cache, float *__restrict__ part /* [tile][n_q_heads][D] */)
{
    constexpr int EPL = DTYPE == KVS_BF16 ? 8 : 4;
    constexpr int D = LPH * EPL;
    constexpr int SLOTS = kThreads / LPH;          // rows a workgroup works on at once
    constexpr int UNROLL = 4;
    __shared__ float red[kThreads / 64][kAttMaxG][D];
    __shared__ __align__(16) float wts[kAttTok][kAttMaxG];
    static_assert(kAttTok == kThreads, "one token per thread in the weights step");
    const int g = blockIdx.x % n_kv_heads;
    const int tile_id = blockIdx.x / n_kv_heads;
    int b = 0;
    while (b + 1 < bd.n_req && tile_id >= bd.tile_begin[b + 1]) ++b;
    const int tok0 = (tile_id - bd.tile_begin[b]) * kAttTok;
    const int ntok = min(kAttTok, bd.ctx_len[b] - tok0);
    const int64_t row0 = bd.ctx_off[b] + tok0;
    const int grp = n_q_heads / n_kv_heads;
    const int tid = threadIdx.x, sub = tid % LPH, slot = tid / LPH, wave = tid >> 6, lane = tid & 63;
    const float2 *st = stats + (int64_t)(bd.req0 + b) * n_q_heads;
    for (int h0 = 0; h0 < grp; h0 += kAttMaxG) {
        const int nh = min(kAttMaxG, grp - h0);
        float acc[kAttMaxG][EPL];
#pragma unroll
        for (int hh = 0; hh < kAttMaxG; ++hh)
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[hh][e] = 0.f;
        // the tile's weights once, one token per thread (the logits of a head are contiguous over tokens)
        if (tid < ntok) {
#pragma unroll
            for (int hh = 0; hh < kAttMaxG; ++hh) {
                float a = 0.f;
                if (hh < nh) {
                    const float2 ms = st[g * grp + h0 + hh];
                    const float lg = logits[(int64_t)(g * grp + h0 + hh) * n_rows + row0 + tid];
                    a = __builtin_amdgcn_exp2f((lg - ms.x) * 1.4426950408889634f) / ms.y;
                }
                wts[tid][hh] = a;
            }
        }
        __syncthreads();
        for (int t0 = slot; t0 < ntok; t0 += SLOTS * UNROLL) {
            uint4 w[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int t = min(t0 + u * SLOTS, ntok - 1);
                w[u] = stream_load16(v_cache + ((row0 + t) * n_kv_heads + g) * LPH + sub);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int t = t0 + u * SLOTS;
                if (t < ntok) {                         // uniform over the LPH lanes of a row
                    float vx[EPL];
                    unpack_piece<DTYPE, EPL>(w[u], vx);
                    const float4 a0 = *reinterpret_cast<const float4 *>(&wts[t][0]);
                    const float4 a1 = *reinterpret_cast<const float4 *>(&wts[t][4]);
                    const float a[kAttMaxG] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
                    for (int hh = 0; hh < kAttMaxG; ++hh) {
                        if (hh < nh) {
#pragma unroll
                            for (int e = 0; e < EPL; ++e) acc[hh][e] = fmaf(a[hh], vx[e], acc[hh][e]);
                        }
                    }
                }
            }
        }
        // add the row slots: inside a wave by shuffles, across the waves through LDS, fixed order
#pragma unroll
        for (int hh = 0; hh < kAttMaxG; ++hh)
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                float v = acc[hh][e];
#pragma unroll
                for (int o = LPH; o < 64; o <<= 1) v += __shfl_xor(v, o);
                acc[hh][e] = v;
            }
        if (lane < LPH) {
#pragma unroll
            for (int hh = 0; hh < kAttMaxG; ++hh)
#pragma unroll
                for (int e = 0; e < EPL; ++e) red[wave][hh][sub * EPL + e] = acc[hh][e];
        }
        __syncthreads();
        for (int i = tid; i < nh * D; i += kThreads) {
            const int hh = i / D, c = i - hh * D;
            float s = 0.f;
#pragma unroll
            for (int wv = 0; wv < kThreads / 64; ++wv) s += red[wv][hh][c];
            part[((int64_t)tile_id * n_q_heads + g * grp + h0 + hh) * D + c] = s;
        }
        __syncthreads();
    }
}

// one workgroup per (request, query head), one thread per channel: the request's tiles in order
template <int DTYPE>
__global__ void decode_attn_merge_kernel(const DecodeBatch bd, int n_q_heads, int d, const float *__restrict__ part,
                                         void *__restrict__ attn_out)
{
    const int b = blockIdx.x / n_q_heads, h = blockIdx.x % n_q_heads;
    const int c = threadIdx.x;
    if (c >= d) return;
    float s = 0.f;
    for (int t = bd.tile_begin[b]; t < bd.tile_begin[b + 1]; ++t) s += part[((int64_t)t * n_q_heads + h) * d + c];
    const int64_t oi = ((int64_t)(bd.req0 + b) * n_q_heads + h) * d + c;
    if (DTYPE == KVS_F32) ((float *)attn_out)[oi] = s;
    else ((uint16_t *)attn_out)[oi] = (uint16_t)f32_to_bf16_bits(s);
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

} // namespace

size_t decode_workspace_bytes(const kvs_shape *shape, int32_t batch, int64_t n_rows)
{
    size_t logits = align_up(sizeof(float) * (size_t)shape->n_q_heads * (size_t)n_rows, 256);
    size_t stats = align_up(sizeof(float2) * (size_t)batch * (size_t)shape->n_q_heads, 256);
    size_t score = align_up(sizeof(float) * (size_t)n_rows, 256);
    size_t partial = align_up(sizeof(float2) * ((size_t)n_rows / kTok + (size_t)batch + 1) * (size_t)shape->n_q_heads, 256);
    // per-tile shares of the optional attention output
    size_t attn = align_up(sizeof(float) * ((size_t)n_rows / kAttTok + (size_t)batch + 1) * (size_t)shape->n_q_heads * (size_t)shape->head_dim, 256);
    // rows of the top-k that are too long for one workgroup
    return logits + stats + score + partial + attn + align_up(select_workspace_bytes(batch, n_rows), 256);
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
    // The contexts must not share cache rows: logits, scores and the per-tile softmax partials are
    // indexed by cache row, so overlapping requests would overwrite each other's and overrun the
    // tile tables, which are sized for n_rows rows in all.  Batches whose offsets ascend (the usual
    // packing) are checked in one pass, any other order pairwise.
    {
        bool ascending = true;
        for (int32_t b = 1; b < batch && ascending; ++b) ascending = ctx_off[b] >= ctx_off[b - 1];
        int64_t end_so_far = 0;   // ascending offsets: end of the last non-empty context seen
        for (int32_t b = 0; b < batch; ++b) {
            if (ctx_len[b] == 0) continue;
            if (ascending) {
                if (ctx_off[b] < end_so_far)
                    return fail(KVS_EINVAL, "kvs_decode_check: request %d shares cache rows with an earlier one", b);
                end_so_far = ctx_off[b] + ctx_len[b];
            } else {
                for (int32_t a = 0; a < b; ++a)
                    if (ctx_len[a] > 0 && ctx_off[a] < ctx_off[b] + ctx_len[b] && ctx_off[b] < ctx_off[a] + ctx_len[a])
                        return fail(KVS_EINVAL, "kvs_decode_check: requests %d and %d share cache rows", a, b);
            }
        }
    }
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
    ws += align_up(sizeof(float2) * ((size_t)n_rows / kTok + (size_t)batch + 1) * (size_t)hq, 256);
    float *attn_part = (float *)ws;
    ws += align_up(sizeof(float) * ((size_t)n_rows / kAttTok + (size_t)batch + 1) * (size_t)hq * (size_t)d, 256);
    void *select_ws = ws;
    const int lph = (int)(d * elem_bytes(shape->dtype) / 16);
    // One context of a length the histogram-driven selection covers: the score kernel also leaves the keys and
    // their leading-bits histogram in the library's own device scratch (the one kvs_deviation_topk uses: calls on
    // one device that use it must not overlap), and two short launches replace the one-workgroup top-k.
    const bool from_hist = batch == 1 && k_req[0] > 0 && ctx_len[0] > kFusedMinTokens && ctx_len[0] <= kFusedMaxTokens;
    FusedScratch fs = {nullptr, nullptr, nullptr};
    if (from_hist) {
        const kvs_status fst = fused_scratch(&fs);
        if (fst != KVS_OK) return fst;
    }

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
        // every lane group keeps one kv head and the group size is one of the compiled ones: the
        // queries live in registers; every other shape reads them from LDS
        const bool regq = (kThreads / lph) % hk == 0 && (grp == 1 || grp == 2 || grp == 4 || grp == 7 || grp == 8);
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
        else if (regq) KVS_DEC_LAUNCH(DT, L, 8);                               \
        else KVS_DEC_LAUNCH(DT, L, 0);                                         \
    } while (0)
        // bf16 / head_dim 128: the matrix-core kernel, as long as 32-bit byte offsets reach the whole cache
        const bool mma = shape->dtype == KVS_BF16 && d == 128 && grp <= 32 && n_rows * (int64_t)hk * 256 < ((int64_t)1 << 32) &&
                         aligned16(q_new) && aligned16(k_cache);
        if (mma) {
            static DeviceOnce attr_once;
            st = once_per_device(attr_once, [] {
                const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&decode_logits_mfma_kernel),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, kMmaLds);
                return e == hipSuccess ? KVS_OK : fail(KVS_EHIP, "kvs_decode_check: hipFuncSetAttribute: %s", hipGetErrorString(e));
            });
            if (st != KVS_OK) return st;
            hipLaunchKernelGGL(decode_logits_mfma_kernel, dim3((unsigned)(KVS_DEC_PERSIST > 0 && tiles_tok > KVS_DEC_PERSIST ? KVS_DEC_PERSIST : tiles_tok)), block, kMmaLds, hs, bd_tok, hq, hk, n_rows,
                               (const uint16_t *)q_new, (const uint16_t *)k_cache, scale, logits, part_l, (int)tiles_tok);
        }
        else if (shape->dtype == KVS_BF16 && lph == 16) KVS_DEC_CASE(KVS_BF16, 16);
        else if (shape->dtype == KVS_BF16 && lph == 8) KVS_DEC_CASE(KVS_BF16, 8);
        else if (shape->dtype == KVS_F32 && lph == 16) KVS_DEC_CASE(KVS_F32, 16);
        else if (shape->dtype == KVS_F32 && lph == 32) KVS_DEC_CASE(KVS_F32, 32);
        else return fail(KVS_EUNSUPPORTED, "kvs_decode_check: head_dim %d", d);
#undef KVS_DEC_CASE
#undef KVS_DEC_LAUNCH
        if ((st = check_launch("kvs_decode_check(logits)")) != KVS_OK) return st;
        hipLaunchKernelGGL(decode_stats_kernel, dim3((unsigned)(nr * hq)), block, 0, hs, bd_tok, hq, part_l, stats);
        if ((st = check_launch("kvs_decode_check(stats)")) != KVS_OK) return st;
        const dim3 sgrid((unsigned)((tiles_tok + kThreads / 64 - 1) / (kThreads / 64)));
#define KVS_DEC_SCORE(G)                                                                                                          \
    do {                                                                                                                          \
        if (from_hist)                                                                                                            \
            hipLaunchKernelGGL((decode_score_kernel<G, true>), sgrid, block, 0, hs, bd_tok, (int)tiles_tok, hq, hk, n_rows, logits, \
                               stats, dev_v, reused, score, fs.keys, fs.hist);                                                    \
        else                                                                                                                      \
            hipLaunchKernelGGL((decode_score_kernel<G, false>), sgrid, block, 0, hs, bd_tok, (int)tiles_tok, hq, hk, n_rows, logits, \
                               stats, dev_v, reused, score, (uint32_t *)nullptr, (uint32_t *)nullptr);                            \
    } while (0)
        if (grp == 1) KVS_DEC_SCORE(1);
        else if (grp == 2) KVS_DEC_SCORE(2);
        else if (grp == 4) KVS_DEC_SCORE(4);
        else if (grp == 7) KVS_DEC_SCORE(7);
        else if (grp == 8) KVS_DEC_SCORE(8);
        else KVS_DEC_SCORE(0);
#undef KVS_DEC_SCORE
        if ((st = check_launch("kvs_decode_check(score)")) != KVS_OK) return st;
        if (attn_out) {
            DecodeBatch bd_att = bd_tok;   // the same requests in kAttTok-token tiles
            int64_t tiles_att = 0;
            for (int i = 0; i < kMaxReq; ++i) {
                bd_att.tile_begin[i] = (int32_t)tiles_att;
                tiles_att += ((int64_t)bd_att.ctx_len[i] + kAttTok - 1) / kAttTok;
            }
            bd_att.tile_begin[kMaxReq] = (int32_t)tiles_att;
            const dim3 agrid((unsigned)(tiles_att * hk));
#define KVS_DEC_ATTN(DT, L) hipLaunchKernelGGL((decode_attn_partial_kernel<DT, L>), agrid, block, 0, hs, bd_att, hq, hk, n_rows, logits, stats, (const uint4 *)v_cache, attn_part)
            if (shape->dtype == KVS_BF16 && lph == 16) KVS_DEC_ATTN(KVS_BF16, 16);
            else if (shape->dtype == KVS_BF16 && lph == 8) KVS_DEC_ATTN(KVS_BF16, 8);
            else if (shape->dtype == KVS_F32 && lph == 16) KVS_DEC_ATTN(KVS_F32, 16);
            else KVS_DEC_ATTN(KVS_F32, 32);
#undef KVS_DEC_ATTN
            if ((st = check_launch("kvs_decode_check(attn)")) != KVS_OK) return st;
            if (shape->dtype == KVS_BF16) hipLaunchKernelGGL(decode_attn_merge_kernel<KVS_BF16>, dim3((unsigned)(nr * hq)), dim3(128), 0, hs, bd_att, hq, d, attn_part, attn_out);
            else hipLaunchKernelGGL(decode_attn_merge_kernel<KVS_F32>, dim3((unsigned)(nr * hq)), dim3(128), 0, hs, bd_att, hq, d, attn_part, attn_out);
            if ((st = check_launch("kvs_decode_check(attn merge)")) != KVS_OK) return st;
        }
    }
    if (total_k == 0) return KVS_OK;
    if (from_hist) return launch_select_from_hist(fs, (int32_t)ctx_len[0], k_req[0], idx_out, hs);
    return launch_select(score, batch, ctx_off, ctx_len, k_req, idx_out, select_ws, select_workspace_bytes(batch, n_rows), hs);
}
