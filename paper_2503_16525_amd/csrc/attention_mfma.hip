// Partial-recompute attention on the gfx950 matrix cores (bf16 in, fp32 accumulate), head_dim 128.
// Computes Eq. (1) for the rows of the selected tokens only; each query attends causally, by its
// original position, over the blended cache.
//
// Work decomposition
//   * The G = n_q_heads / n_kv_heads query heads that share KV head g are flattened with the
//     selected tokens into rows r = t*G + hh (t = selected token, ascending position).  Any G
//     packs without padding (7 included): a row tile simply cuts the flattened list every
//     32*NWAVES rows.
//   * One workgroup = one KV head and one tile of 32*NWAVES rows; each wave owns 32 rows.  The
//     workgroup streams K/V tiles of 64 keys through LDS from key 0 up to the largest position
//     in its tile.  Only tiles that straddle a row's position need the causal compare; all
//     tiles below the wave's smallest position take the unmasked path.
//   * Workgroups are issued heaviest tile first, and KV head = blockIdx % n_kv_heads so that the
//     workgroups resident on one XCD walk the same head's K/V and share it in that XCD's L2.
//
// Per KV tile, per wave (v_mfma_f32_32x32x16_bf16, 64-lane wavefront):
//   S^T[key][q] = K[key][:] . Q[q][:]        A = K rows from LDS (16 B per lane), B = Q registers
//   online softmax down each lane's own column (a query's 64 keys sit in two lanes, l and l^32)
//   O^T[d][q]  += V^T[d][key] . P^T[key][q]  A = V^T rows from LDS, B = P straight from registers
// Computing the transposed products makes the S accumulator layout coincide with the B-operand
// layout of the second product, so P never leaves registers.  The K rows are fed to the first
// product in a permuted order (bits 2 and 3 of the row index swapped) so that the 8 P values a
// lane holds for one MFMA k-step belong to 8 consecutive keys, i.e. one 16-byte LDS read of V^T.
// V is transposed on its way into LDS: lanes sweep head_dim in 4-byte steps for 8 consecutive
// keys (coalesced 256 B per wave load), repack in registers, and write two 16-byte rows of V^T.
#include "attention.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

namespace kvs {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

#ifndef KVS_ATTN_NWAVES
#define KVS_ATTN_NWAVES 4
#endif
#ifndef KVS_ATTN_BIG_MIN_GRID
#define KVS_ATTN_BIG_MIN_GRID 256
#endif

constexpr int kAttnBigTileMinGrid = KVS_ATTN_BIG_MIN_GRID;
constexpr int D = 128;            // head_dim
constexpr int BN = 64;            // keys per LDS tile
constexpr int K_LD = D + 8;       // K tile row pitch in bf16 (272 B: 16-byte reads of 16 rows hit 16 bank groups)
constexpr int V_LD = BN + 8;      // V^T tile row pitch in bf16 (144 B)
constexpr int K_TILE = BN * K_LD; // bf16 elements
constexpr int V_TILE = D * V_LD;
constexpr int STAGE = K_TILE + V_TILE;

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// SPLIT: the key range of a row tile is cut into n_splits contiguous pieces handled by different
// workgroups (small launches would otherwise leave most of the chip idle while a few workgroups
// walk 32k keys each); every piece writes its unnormalised accumulators and (max, sum) to the
// workspace and attn_merge_kernel combines them.
template <int NWAVES, bool SPLIT>
__global__ __launch_bounds__(NWAVES * 64, 2) void attn_mfma_kernel(
    const AttnTiles td, int n_q_heads, int n_kv_heads, int total_tiles,
    const uint16_t *__restrict__ q_sel, const int32_t *__restrict__ sel_pos,
    const uint16_t *__restrict__ k_cache, const uint16_t *__restrict__ v_cache,
    float scale_log2, uint16_t *__restrict__ out, float *__restrict__ lse_out,
    int n_splits, float *__restrict__ part_o, float4 *__restrict__ part_ml)
{
    constexpr int NT = NWAVES * 64;
    constexpr int ROWS = NWAVES * 32;
    constexpr int K_PIECES = BN * (D / 8) / NT;    // 16-byte K pieces per thread per tile
    constexpr int V_ITEMS = (BN / 8) * (D / 2) / NT; // (key octet, channel pair) items per thread
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];   // 2 stages of (K tile, V^T tile)
    __shared__ int wg_max_pos[NWAVES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, ln = lane & 31;

    // ---- which (request, kv head, row tile) -----------------------------------------------------
    const int g = blockIdx.x % n_kv_heads;
    const int rest = (int)(blockIdx.x / n_kv_heads);
    const int split = SPLIT ? rest % n_splits : 0;
    const int tile_lin = total_tiles - 1 - (SPLIT ? rest / n_splits : rest);
    int b = 0;
    while (b + 1 < td.n_req && tile_lin >= td.tile_begin[b + 1]) ++b;
    const int tile = tile_lin - td.tile_begin[b];
    const int grp = n_q_heads / n_kv_heads;
    const int64_t sel0 = td.sel_lo[b];
    const int n_rows = td.n_sel[b] * grp;
    const int ctx_len = td.ctx_len[b];
    const int64_t ctx_off = td.ctx_off[b];

    // this lane's query row (both half-waves hold the same 32 queries)
    const int rq = tile * ROWS + wave * 32 + ln;
    const bool row_ok = rq < n_rows;
    const int rqc = row_ok ? rq : n_rows - 1;
    const int t_sel = rqc / grp, hh = rqc - t_sel * grp;
    const int64_t s_glob = sel0 + t_sel;
    int pos = sel_pos[s_glob];
    pos = min(max(pos, 0), ctx_len - 1);             // memory safety; the caller guarantees the range
    const int64_t q_row = (s_glob * n_q_heads + g * grp + hh) * (int64_t)D;

    // wave-wide smallest / largest position
    int pmin = pos, pmax = pos;
#pragma unroll
    for (int o = 1; o < 32; o <<= 1) {
        pmin = min(pmin, __shfl_xor(pmin, o));
        pmax = max(pmax, __shfl_xor(pmax, o));
    }
    if (lane == 0) wg_max_pos[wave] = pmax;

    // ---- Q as the B operand: Q[query ln][16*ks + 8*hf + j] ----------------------------------------
    bf16x8 qreg[D / 16];
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks)
        qreg[ks] = as_bf16x8(*reinterpret_cast<const u32x4_t *>(q_sel + q_row + 16 * ks + 8 * hf));

    __syncthreads();
    int wg_pmax = wg_max_pos[0];
#pragma unroll
    for (int w = 1; w < NWAVES; ++w) wg_pmax = max(wg_pmax, wg_max_pos[w]);
    const int n_kv_tiles = wg_pmax / BN + 1;
    // the KV tiles this workgroup walks: all of them, or its contiguous share
    const int t_chunk = SPLIT ? (n_kv_tiles + n_splits - 1) / n_splits : n_kv_tiles;
    const int t_lo = SPLIT ? min(n_kv_tiles, split * t_chunk) : 0;
    const int t_hi = SPLIT ? min(n_kv_tiles, t_lo + t_chunk) : n_kv_tiles;

    // ---- global -> register staging of one K/V tile -------------------------------------------------
    // Addresses are a wave-uniform tile base (scalar registers) plus a per-lane 32-bit byte offset
    // that never changes, so the loop carries no vector address arithmetic.  Only a tile that
    // reaches past the end of the context (the last one of a request) clamps its rows.
    const uint32_t row_bytes = (uint32_t)n_kv_heads * D * 2u;          // bytes between tokens
    const char *kbase = reinterpret_cast<const char *>(k_cache + (ctx_off * n_kv_heads + g) * (int64_t)D);
    const char *vbase = reinterpret_cast<const char *>(v_cache + (ctx_off * n_kv_heads + g) * (int64_t)D);
    u32x4_t kst[K_PIECES];
    uint32_t vst[V_ITEMS][8];
    const uint32_t k_lane_off = (uint32_t)(tid >> 4) * row_bytes + (uint32_t)(tid & 15) * 16u;
    const uint32_t v_lane_off = (uint32_t)lane * 4u;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);

    auto load_tile = [&](int kv0) {
        const char *kt = kbase + (int64_t)kv0 * row_bytes;
        const char *vt = vbase + (int64_t)kv0 * row_bytes;
        if (kv0 + BN <= ctx_len) {
#pragma unroll
            for (int i = 0; i < K_PIECES; ++i)
                kst[i] = *reinterpret_cast<const u32x4_t *>(kt + (size_t)(i * (NT / 16)) * row_bytes + k_lane_off);
#pragma unroll
            for (int it = 0; it < V_ITEMS; ++it) {
                const char *vo = vt + (size_t)(8 * (wave_u + NWAVES * it)) * row_bytes;
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    vst[it][j] = *reinterpret_cast<const uint32_t *>(vo + (size_t)j * row_bytes + v_lane_off);
            }
        } else {
#pragma unroll
            for (int i = 0; i < K_PIECES; ++i) {
                const int key = min(kv0 + i * (NT / 16) + (tid >> 4), ctx_len - 1);
                kst[i] = *reinterpret_cast<const u32x4_t *>(kbase + (int64_t)key * row_bytes + (tid & 15) * 16);
            }
#pragma unroll
            for (int it = 0; it < V_ITEMS; ++it)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int key = min(kv0 + 8 * (wave_u + NWAVES * it) + j, ctx_len - 1);
                    vst[it][j] = *reinterpret_cast<const uint32_t *>(vbase + (int64_t)key * row_bytes + v_lane_off);
                }
        }
    };
    auto store_tile = [&](int stage) {
        uint16_t *ks = lds + stage * STAGE;
        uint16_t *vs = ks + K_TILE;
#pragma unroll
        for (int i = 0; i < K_PIECES; ++i) {
            const int id = i * NT + tid;
            const int row = id >> 4, c16 = id & 15;
            *reinterpret_cast<u32x4_t *>(ks + row * K_LD + c16 * 8) = kst[i];
        }
#pragma unroll
        for (int it = 0; it < V_ITEMS; ++it) {
            const int ko = wave + NWAVES * it;
            u32x4_t lo, hi;   // channel 2*lane and 2*lane+1 of keys 8*ko .. 8*ko+7
            // v_perm_b32: bytes 0-3 come from the second operand, 4-7 from the first
            lo.x = __builtin_amdgcn_perm(vst[it][1], vst[it][0], 0x05040100u);
            lo.y = __builtin_amdgcn_perm(vst[it][3], vst[it][2], 0x05040100u);
            lo.z = __builtin_amdgcn_perm(vst[it][5], vst[it][4], 0x05040100u);
            lo.w = __builtin_amdgcn_perm(vst[it][7], vst[it][6], 0x05040100u);
            hi.x = __builtin_amdgcn_perm(vst[it][1], vst[it][0], 0x07060302u);
            hi.y = __builtin_amdgcn_perm(vst[it][3], vst[it][2], 0x07060302u);
            hi.z = __builtin_amdgcn_perm(vst[it][5], vst[it][4], 0x07060302u);
            hi.w = __builtin_amdgcn_perm(vst[it][7], vst[it][6], 0x07060302u);
            *reinterpret_cast<u32x4_t *>(vs + (2 * lane) * V_LD + 8 * ko) = lo;
            *reinterpret_cast<u32x4_t *>(vs + (2 * lane + 1) * V_LD + 8 * ko) = hi;
        }
    };

    // ---- running softmax state and output accumulators ---------------------------------------------
    floatx16 o_acc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
    // running max of scale*log2(e)*logit, shared by the two half-waves.  It starts at a huge
    // negative *finite* value so that a tile in which a row sees no key at all (possible when the
    // key range is split) gives exp2(-inf - m) = 0 and a rescale factor of 1 instead of a NaN
    float m_run = -1.0e30f;
    float l_run = 0.f;         // this half-wave's share of the running sum

    // K row fed to MFMA row ln: bits 2 and 3 swapped
    const int krow = (ln & ~12) | ((ln & 4) << 1) | ((ln & 8) >> 1);

    if (t_lo < t_hi) {
        load_tile(t_lo * BN);
        store_tile(t_lo & 1);
    }
    __syncthreads();

    for (int jt = t_lo; jt < t_hi; ++jt) {
        const int kv0 = jt * BN;
        const int stage = jt & 1;
        const bool more = jt + 1 < t_hi;
        if (more) load_tile(kv0 + BN);

        if (kv0 <= pmax) {                           // wave-uniform: this wave still has keys to see
            const uint16_t *ks = lds + stage * STAGE;
            const uint16_t *vs = ks + K_TILE;
            floatx16 s_acc[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s_acc[kb][r] = 0.f;
#pragma unroll
            for (int ksx = 0; ksx < D / 16; ++ksx) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const u32x4_t a = *reinterpret_cast<const u32x4_t *>(ks + (32 * kb + krow) * K_LD + 16 * ksx + 8 * hf);
                    s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), qreg[ksx], s_acc[kb], 0, 0, 0);
                }
            }
            // causal compare only where a key of this tile can exceed a position of this wave
            if (kv0 + BN - 1 > pmin) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = kv0 + 32 * kb + 16 * (r >> 3) + 8 * hf + (r & 7);
                        if (key > pos) s_acc[kb][r] = -INFINITY;
                    }
            }
            float mx = s_acc[0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s_acc[kb][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx * scale_log2);
            const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            float psum = 0.f;
            u32x4_t pop[2][2];                          // B operands of the second product: [kb][a]
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                float pv[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    pv[r] = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][r], scale_log2, -m_new));
                    psum += pv[r];
                }
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    pop[kb][a].x = pack2(pv[8 * a + 0], pv[8 * a + 1]);
                    pop[kb][a].y = pack2(pv[8 * a + 2], pv[8 * a + 3]);
                    pop[kb][a].z = pack2(pv[8 * a + 4], pv[8 * a + 5]);
                    pop[kb][a].w = pack2(pv[8 * a + 6], pv[8 * a + 7]);
                }
            }
            // rescale the running sum and the output accumulators only when some row's max moved
            // (wave-uniform test; after the first few tiles it rarely does)
            if (__builtin_amdgcn_ballot_w64(corr != 1.0f) != 0) {
                l_run *= corr;
#pragma unroll
                for (int db = 0; db < D / 32; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o_acc[db][r] *= corr;
            }
            l_run += psum;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    const int kstep = 2 * kb + a;
#pragma unroll
                    for (int db = 0; db < D / 32; ++db) {
                        const u32x4_t va = *reinterpret_cast<const u32x4_t *>(vs + (32 * db + ln) * V_LD + 16 * kstep + 8 * hf);
                        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va), as_bf16x8(pop[kb][a]), o_acc[db], 0, 0, 0);
                    }
                }
        }
        if (more) store_tile(stage ^ 1);
        __syncthreads();
    }

    // ---- epilogue: normalise, convert, store ----------------------------------------------------------
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (SPLIT) {
        if (row_ok) {
            const int64_t slot = (s_glob * n_q_heads + g * grp + hh) * (int64_t)n_splits + split;
            float *prow = part_o + slot * D;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int d0 = 32 * db + 8 * r4 + 4 * hf;
                    *reinterpret_cast<float4 *>(prow + d0) = make_float4(o_acc[db][4 * r4 + 0], o_acc[db][4 * r4 + 1],
                                                                         o_acc[db][4 * r4 + 2], o_acc[db][4 * r4 + 3]);
                }
            if (hf == 0) part_ml[slot] = make_float4(m_run, l_tot, l_tot, 0.f);
        }
        return;
    }
    const float inv = 1.0f / l_tot;
    if (row_ok) {
        uint16_t *orow = out + q_row;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int d0 = 32 * db + 8 * r4 + 4 * hf;
                uint2 w;
                w.x = pack2(o_acc[db][4 * r4 + 0] * inv, o_acc[db][4 * r4 + 1] * inv);
                w.y = pack2(o_acc[db][4 * r4 + 2] * inv, o_acc[db][4 * r4 + 3] * inv);
                *reinterpret_cast<uint2 *>(orow + d0) = w;
            }
        if (lse_out && hf == 0)
            lse_out[s_glob * n_q_heads + g * grp + hh] = (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    }
}


// combines the split pieces of every row: out = sum_s w_s O_s / sum_s w_s l_s with
// w_s = 2^(m_s - max m); pieces that saw no key carry l = 0 and drop out.  32 lanes per row, four
// channels per lane, all pieces' loads issued before they are used.
__global__ __launch_bounds__(256) void attn_merge_kernel(int64_t n_rows, int n_splits,
                                                         const float *__restrict__ part_o,
                                                         const float4 *__restrict__ part_ml,
                                                         uint16_t *__restrict__ out, float *__restrict__ lse_out)
{
    const int64_t row = (int64_t)blockIdx.x * 8 + threadIdx.x / 32;
    const int c = (threadIdx.x % 32) * 4;
    if (row >= n_rows) return;
    const float4 *ml = part_ml + row * n_splits;
    const float *po = part_o + row * n_splits * D + c;
    float4 v[kAttnSplitMax];
    float4 p[kAttnSplitMax];
#pragma unroll
    for (int s = 0; s < kAttnSplitMax; ++s)
        if (s < n_splits) p[s] = ml[s];
#pragma unroll
    for (int s = 0; s < kAttnSplitMax; ++s)
        if (s < n_splits && p[s].y > 0.f) v[s] = *reinterpret_cast<const float4 *>(po + s * D);
    float m = -1.0e30f;
#pragma unroll
    for (int s = 0; s < kAttnSplitMax; ++s)
        if (s < n_splits && p[s].y > 0.f) m = fmaxf(m, p[s].x);
    float l = 0.f, l_exact = 0.f;
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int s = 0; s < kAttnSplitMax; ++s)
        if (s < n_splits && p[s].y > 0.f) {
            const float w = __builtin_amdgcn_exp2f(p[s].x - m);
            l += w * p[s].y;
            l_exact += w * p[s].z;
            o.x += w * v[s].x;
            o.y += w * v[s].y;
            o.z += w * v[s].z;
            o.w += w * v[s].w;
        }
    const float inv = 1.0f / l;
    uint2 w2;
    w2.x = f32_to_bf16_bits(o.x * inv) | (f32_to_bf16_bits(o.y * inv) << 16);
    w2.y = f32_to_bf16_bits(o.z * inv) | (f32_to_bf16_bits(o.w * inv) << 16);
    *reinterpret_cast<uint2 *>(out + row * D + c) = w2;
    if (lse_out && c == 0) lse_out[row] = (m + __builtin_amdgcn_logf(l_exact)) * 0.6931471805599453f;
}

constexpr size_t kPartBytesPerSlot = kAttnPartBytesPerSlot;
constexpr int kSplitMaxWgs = 1024;        // splits are chosen so that the grid stays near this
constexpr int kSplitBelowWgs = kAttnSplitBelowWgs;
constexpr int kSplitMax = kAttnSplitMax;

template <int NWAVES>
kvs_status launch_mfma_variant(const kvs_shape *shape, const AttnBatch &bd, const void *q_sel, const int32_t *sel_pos,
                               const void *k_cache, const void *v_cache, float scale, void *out, float *lse_out,
                               void *workspace, size_t workspace_bytes, hipStream_t st)
{
    constexpr int ROWS = NWAVES * 32;
    AttnTiles td;
    const int64_t tiles = build_attn_tiles(shape, bd, ROWS, td);
    if (tiles < 0) return fail(KVS_EINVAL, "kvs_partial_attention: too many row tiles");
    if (tiles == 0) return KVS_OK;
    const size_t lds_bytes = 2 * STAGE * sizeof(uint16_t);
    static DeviceOnce attr_once;
    const kvs_status ast = once_per_device(attr_once, [] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_mfma_kernel<NWAVES, false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_mfma_kernel<NWAVES, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        return e == hipSuccess ? KVS_OK : fail(KVS_EHIP, "kvs_partial_attention: hipFuncSetAttribute: %s", hipGetErrorString(e));
    });
    if (ast != KVS_OK) return ast;
    const float scale_log2 = scale * 1.4426950408889634f;
    // split the key range when the launch is too small to fill the chip, the contexts are long
    // enough for every piece to have work, and the caller's workspace can hold the pieces
    const int64_t wgs = tiles * shape->n_kv_heads;
    int64_t max_ctx = 0;
    for (int i = 0; i < bd.n_req; ++i) max_ctx = bd.ctx_len[i] > max_ctx ? bd.ctx_len[i] : max_ctx;
    const int64_t n_rows_total = (bd.cu_sel[bd.n_req] - bd.cu_sel[0]) * shape->n_q_heads;
    int n_splits = 1;
    if (wgs < kSplitBelowWgs && workspace) {
        int64_t s = (kSplitMaxWgs + wgs - 1) / wgs;
        if (s > kSplitMax) s = kSplitMax;
        const int64_t by_len = max_ctx / (8 * BN);                      // at least 8 KV tiles per piece
        if (s > by_len) s = by_len;
        const int64_t by_ws = (int64_t)(workspace_bytes / (kPartBytesPerSlot * (size_t)(n_rows_total > 0 ? n_rows_total : 1)));
        if (s > by_ws) s = by_ws;
        if (s >= 2) n_splits = (int)s;
    }
    if (n_splits == 1) {
        hipLaunchKernelGGL((attn_mfma_kernel<NWAVES, false>), dim3((unsigned)wgs), dim3(NWAVES * 64), lds_bytes, st, td,
                           shape->n_q_heads, shape->n_kv_heads, (int)tiles, (const uint16_t *)q_sel, sel_pos,
                           (const uint16_t *)k_cache, (const uint16_t *)v_cache, scale_log2, (uint16_t *)out, lse_out,
                           1, (float *)nullptr, (float4 *)nullptr);
        return check_launch("kvs_partial_attention(mfma)");
    }
    // pieces are indexed by the row's position in the whole call's output, so offset the tables by
    // the first row of this launch
    const int64_t row0 = bd.cu_sel[0] * shape->n_q_heads;
    float *part_o = (float *)workspace - row0 * n_splits * D;
    float4 *part_ml = (float4 *)((char *)workspace + (size_t)n_rows_total * n_splits * D * sizeof(float)) - row0 * n_splits;
    hipLaunchKernelGGL((attn_mfma_kernel<NWAVES, true>), dim3((unsigned)(wgs * n_splits)), dim3(NWAVES * 64), lds_bytes, st, td,
                       shape->n_q_heads, shape->n_kv_heads, (int)tiles, (const uint16_t *)q_sel, sel_pos,
                       (const uint16_t *)k_cache, (const uint16_t *)v_cache, scale_log2, (uint16_t *)out, lse_out,
                       n_splits, part_o, part_ml);
    kvs_status stt = check_launch("kvs_partial_attention(mfma split)");
    if (stt != KVS_OK) return stt;
    return launch_attention_merge(n_rows_total, n_splits, (const float *)workspace,
                                  (const float4 *)((char *)workspace + (size_t)n_rows_total * n_splits * D * sizeof(float)),
                                  (uint16_t *)out + row0 * D, lse_out ? lse_out + row0 : nullptr, st);
}

} // namespace

kvs_status launch_attention_merge(int64_t n_rows, int n_splits, const float *part_o, const float4 *part_ml,
                                  uint16_t *out, float *lse_out, hipStream_t st)
{
    if (n_rows <= 0) return KVS_OK;
    hipLaunchKernelGGL(attn_merge_kernel, dim3((unsigned)((n_rows + 7) / 8)), dim3(256), 0, st, n_rows, n_splits,
                       part_o, part_ml, out, lse_out);
    return check_launch("kvs_partial_attention(merge)");
}

int64_t build_attn_tiles(const kvs_shape *shape, const AttnBatch &bd, int rows_per_tile, AttnTiles &td)
{
    const int grp = shape->n_q_heads / shape->n_kv_heads;
    // requests by context length, ascending (insertion sort: at most kAttnMaxReq entries, usually
    // already in order); ties keep the caller's order
    int order[kAttnMaxReq];
    for (int i = 0; i < bd.n_req; ++i) {
        int j = i;
        while (j > 0 && bd.ctx_len[order[j - 1]] > bd.ctx_len[i]) { order[j] = order[j - 1]; --j; }
        order[j] = i;
    }
    int64_t tiles = 0;
    for (int e = 0; e < kAttnMaxReq; ++e) {
        const bool live = e < bd.n_req;
        const int i = live ? order[e] : 0;
        td.ctx_off[e] = live ? bd.ctx_off[i] : 0;
        td.ctx_len[e] = live ? (int32_t)bd.ctx_len[i] : 0;
        td.sel_lo[e] = live ? bd.cu_sel[i] : 0;
        td.n_sel[e] = live ? (int32_t)(bd.cu_sel[i + 1] - bd.cu_sel[i]) : 0;
        td.tile_begin[e] = (int32_t)tiles;
        if (live) tiles += ((int64_t)td.n_sel[e] * grp + rows_per_tile - 1) / rows_per_tile;
        if (tiles * shape->n_kv_heads > 0x7fffffffLL) return -1;
    }
    td.tile_begin[kAttnMaxReq] = (int32_t)tiles;
    td.n_req = bd.n_req;
    return tiles;
}

bool attention_mfma_supports(const kvs_shape *shape)
{
    return shape->dtype == KVS_BF16 && shape->head_dim == D;
}

kvs_status launch_attention_mfma(const kvs_shape *shape, const AttnBatch &bd, int64_t n_sel,
                                 const void *q_sel, const int32_t *sel_pos, const void *k_cache,
                                 const void *v_cache, float scale, void *out, float *lse_out,
                                 void *workspace, size_t workspace_bytes, hipStream_t st)
{
    if (!attention_mfma_supports(shape)) return fail(KVS_EUNSUPPORTED, "kvs_partial_attention: matrix-core path needs bf16, head_dim 128");
    if (!(scale > 0.f) || !isfinite(scale)) return fail(KVS_EUNSUPPORTED, "kvs_partial_attention: matrix-core path needs a positive finite scale");
    // enough 256-row tiles to give every CU work: the 64-rows-per-wave kernel; otherwise the
    // finer-grained one, which fills the chip better.  A build with -DKVS_ATTN_FORCE=1 (small) or 2
    // (large) pins the choice: the test suite builds such a library beside the shipped one to reach
    // the large-launch kernel at sizes the oracle can follow.  The shipped library has no switch.
#ifndef KVS_ATTN_FORCE
#define KVS_ATTN_FORCE 0
#endif
    constexpr int forced = KVS_ATTN_FORCE;
    const int grp = shape->n_q_heads / shape->n_kv_heads;
    int64_t big_tiles = 0, rows = 0;
    // the large kernel addresses a request's keys with 32-bit byte offsets from its first token
    bool fits32 = true;
    for (int i = 0; i < bd.n_req; ++i) {
        big_tiles += ((bd.cu_sel[i + 1] - bd.cu_sel[i]) * grp + 255) / 256;
        rows += (bd.cu_sel[i + 1] - bd.cu_sel[i]) * grp;
        fits32 = fits32 && bd.ctx_len[i] * (int64_t)shape->n_kv_heads * D * 2 < (int64_t)1 << 32;
    }
    // with fewer 256-row tiles than compute units the large kernel still wins if the caller's
    // workspace lets it cut the key ranges and its tiles are not mostly padding
    AttnSplitPlan plan2 = {1, 0, 0, 0, 0};
    if (workspace && fits32) plan2 = attention_mfma2_plan(shape, bd, workspace_bytes);
    const int splits2 = plan2.n_splits;
    const bool fills = big_tiles * shape->n_kv_heads >= kAttnBigTileMinGrid;
    const bool dense_tiles = rows * 10 >= big_tiles * 256 * 6;
    // (below ~50 such tiles the per-workgroup start-up of the large kernel costs more than it gains)
    const bool big = fits32 && (forced ? forced == 2 : fills || (splits2 >= 2 && dense_tiles && big_tiles * shape->n_kv_heads >= 48));
    if (big) {
        if (fills && !forced && plan2.chunk == 0) plan2 = {1, 0, 0, 0, 0};   // fills the chip and stays cached: whole key ranges
        return launch_attention_mfma2(shape, bd, q_sel, sel_pos, k_cache, v_cache, scale, out, lse_out, workspace, plan2, st);
    }
    return launch_mfma_variant<KVS_ATTN_NWAVES>(shape, bd, q_sel, sel_pos, k_cache, v_cache, scale, out, lse_out,
                                                workspace, workspace_bytes, st);
}

size_t attention_workspace_bytes(const kvs_shape *shape, int32_t batch, int64_t n_rows_total, int64_t n_sel_total)
{
    const int64_t rows = n_sel_total * shape->n_q_heads;
    int64_t slots = rows * kSplitMax;
    // Launches that fill the chip keep whole key ranges unless their K and V outgrow the last-level
    // cache (then every row may have up to kSplitMax pieces).  Otherwise pieces are only used below
    // kSplitBelowWgs workgroups: at most kSplitMaxWgs workgroup-pieces of 32*KVS_ATTN_NWAVES rows
    // each (128-row kernel) or fewer than kAttnSplitBelowWgs tiles of 256 rows with up to kSplitMax
    // pieces each (256-row kernel).
    // (a batch is sized for the capped case: with several requests the rows say nothing about the
    // longest one, and a launch whose workspace is too small for pieces keeps whole key ranges)
    const int64_t kv_bytes = n_rows_total * shape->n_kv_heads * (int64_t)D * 2 * 2;
    if (batch > 1 || kv_bytes <= kAttnRangeMajorBytes) {
        const int64_t cap = (int64_t)(kSplitMaxWgs + kSplitBelowWgs) * 256 + (int64_t)batch * 256 * kSplitMax;
        if (slots > cap) slots = cap;
    }
    return (size_t)slots * kPartBytesPerSlot + kAttnPlanBytes + 256;
}

} // namespace kvs
