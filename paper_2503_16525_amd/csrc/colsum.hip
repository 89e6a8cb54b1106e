// kvs_attn_colsum: the attention column mass of a whole prefill (Alg. 1 steps 1-2),
//     alpha[g, i] = sum over the query heads h of KV head g and over the rows j >= i of A_h[j, i],
//     A_h = causal row softmax of scale * Q_h K_g^T,
// in two sweeps over the score matrix, neither of which stores it:
//   sweep 1 (per query row): the log-sum-exp of the row, kept in a scratch array;
//   sweep 2 (per key):       the sum over the rows of exp(score - row's log-sum-exp).
//
// Both sweeps are the same kernel.  A workgroup owns 256 "fixed" rows of one KV head (sweep 1:
// query rows, flattened (token, head-in-group) like the attention kernels; sweep 2: keys), held
// in registers as the B operand of v_mfma_f32_32x32x16_bf16, 64 per wave; the other side streams
// past in tiles of 32 rows that go from global memory straight into an LDS ring (buffer loads
// with the LDS flag) and are read as the A operand, each read feeding two MFMAs.  In the result
// tile a lane's column is one fixed row, so the running sum of a fixed row is one scalar per lane
// (two half-waves, added at the end) and the loop has no cross-lane traffic: per score one fma,
// one exp2 and one add.  State is small (about 128 registers, 33 KiB of LDS), so several
// workgroups share a compute unit and the hardware overlaps one wave's MFMAs with another's
// vector work.
//
// Sweep 1 uses a fixed exponent reference per row, taken from the row's first key tile (plus a
// shift that centres the fp32 exponent range); if a sum
// ends above 2^100 the workgroup finds the exact row maxima in a score-only sweep and repeats.
// Sweep 2 needs none: exp(score - lse) <= 1.  No atomics: the result is identical from run to run.
#include "kvs_internal.h"

#include <math.h>

namespace kvs {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int D = 128;                  // head_dim
constexpr int TS = 32;                  // streamed rows per tile
constexpr int NB = 2;                   // 32-row blocks of fixed rows per wave
constexpr int NWAVES = 4;
constexpr int NT = NWAVES * 64;
constexpr int FIXED = NWAVES * NB * 32; // fixed rows per workgroup
constexpr int ROW_B = D * 2;            // bytes of one row of one head
constexpr int TILE_B = TS * ROW_B;
constexpr int SLOT_B = TILE_B + 256;    // a tile and the 32 log-sum-exps of its rows (sweep 2)
constexpr int RING = 4;                 // slots; tiles are requested RING - 1 steps ahead
constexpr int LDS_BYTES = RING * SLOT_B;
// base-2 offset of sweep 1's fixed reference above the first tile's maximum: the row sums are then
// taken around 2^-60, where fp32 is as precise as around 1, and only overflow for a logit 160 above
constexpr float kRefShift = 60.0f;

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8, v); }

// row of the 32x32 result tile that element r of a lane in half-wave hf holds
__device__ __forceinline__ int tile_row(int r, int hf) { return 8 * (r >> 2) + 4 * hf + (r & 3); }

// `in_flight` = staging instructions of younger tiles that may still be outstanding
#define KVS_CS_BARRIER_(in_flight) asm volatile("s_waitcnt vmcnt(" #in_flight ")\n\ts_barrier" ::: "memory")
#define KVS_CS_BARRIER(in_flight) KVS_CS_BARRIER_(in_flight)

// SWEEP 1: fixed = query rows, streamed = keys, writes lse2[g][row] (base-2, scale included).
// SWEEP 2: fixed = keys, streamed = query rows, reads lse2, writes alpha[g][key].
// Rows of a KV head's queries are flattened as row = token * grp + head-in-group.
template <int SWEEP>
__global__ __launch_bounds__(NT, 2) void colsum_kernel(int n, int n_q_heads, int n_kv_heads,
                                                       const uint16_t *__restrict__ q,
                                                       const uint16_t *__restrict__ k, float scale_log2,
                                                       float *__restrict__ lse2, float *__restrict__ alpha)
{
    extern __shared__ __attribute__((aligned(16))) char lds_b[];
    __shared__ int redo_flag;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hf = lane >> 5, ln = lane & 31;
    const int grp = n_q_heads / n_kv_heads;
    // x / grp for x < 2^24 without a division in the loops (grp 1 has no 32-bit multiplier)
    const uint32_t grp_magic = 0xffffffffu / (uint32_t)grp + 1u;
    auto div_grp = [&](uint32_t x) -> uint32_t { return grp == 1 ? x : __umulhi(x, grp_magic); };
    const int g = blockIdx.x % n_kv_heads;
    const int blk = blockIdx.x / n_kv_heads;
    const int n_qrows = n * grp;
    const int n_fixed = SWEEP == 1 ? n_qrows : n;
    const int n_stream = SWEEP == 1 ? n : n_qrows;
    const int n_blocks = (n_fixed + FIXED - 1) / FIXED;
    // heaviest first: the last query rows see the most keys, the first keys are seen by the most rows
    const int fb = (SWEEP == 1 ? n_blocks - 1 - blk : blk) * FIXED;

    // ---- fixed rows: operands and positions ------------------------------------------------------
    bf16x8 bfix[NB][D / 16];
    int fpos[NB];          // token position of the lane's fixed row (query token / key index)
    int frow[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        frow[nb] = fb + wave * (NB * 32) + nb * 32 + ln;
        const int fr = min(frow[nb], n_fixed - 1);
        const uint16_t *src;
        if (SWEEP == 1) {
            const int tok = (int)div_grp((uint32_t)fr), hh = fr - tok * grp;
            fpos[nb] = tok;
            src = q + ((int64_t)tok * n_q_heads + g * grp + hh) * D;
        } else {
            fpos[nb] = fr;
            src = k + ((int64_t)fr * n_kv_heads + g) * D;
        }
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            bfix[nb][ks] = as_bf16x8(*reinterpret_cast<const u32x4_t *>(src + 16 * ks + 8 * hf));
    }
    int pmin = min(fpos[0], fpos[1]), pmax = max(fpos[0], fpos[1]);
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        pmin = min(pmin, __shfl_xor(pmin, o));
        pmax = max(pmax, __shfl_xor(pmax, o));
    }

    // ---- streamed tiles ---------------------------------------------------------------------------
    // sweep 1: key tiles 0 .. (last token of the workgroup) / 32; sweep 2: query-row tiles from the
    // workgroup's first key on
    const int last_fixed = min(fb + FIXED, n_fixed) - 1;
    const int t_begin = SWEEP == 1 ? 0 : (int)(((int64_t)fb * grp) / TS);
    const int t_end = SWEEP == 1 ? (int)div_grp((uint32_t)last_fixed) / TS + 1 : (n_stream + TS - 1) / TS;
    const int n_tiles = t_end - t_begin;
    // Step k of a sweep takes tile t_begin + k in sweep 1 and tile t_end - 1 - k in sweep 2: every
    // workgroup of a KV head then starts at the same end of the streamed tensor (key 0 / the last
    // query row) whatever its own range, so the workgroups that run together read the same tiles
    // at the same time and share them through L2.  (Sweep 2 run forwards, each workgroup from its
    // own first key, fetched 13 GB from HBM per call at 32k instead of well under 1 GB.)
    auto tile_of = [&](int k) { k = min(k, n_tiles - 1); return SWEEP == 1 ? t_begin + k : t_end - 1 - k; };

    auto make_rsrc = [&](const void *base, uint32_t bytes) -> u32x4_t {
        const uint64_t a = reinterpret_cast<uint64_t>(base);
        u32x4_t r = {(uint32_t)a, (uint32_t)(a >> 32) & 0xffffu, bytes, 0x00020000u};
        r.x = __builtin_amdgcn_readfirstlane(r.x);
        r.y = __builtin_amdgcn_readfirstlane(r.y);
        r.z = __builtin_amdgcn_readfirstlane(r.z);
        return r;
    };
    // the streamed tensor seen from this KV head's first row (byte offsets below fit 32 bits: the
    // host checks the tensor size)
    const uint32_t k_row_bytes = (uint32_t)n_kv_heads * ROW_B, q_row_bytes = (uint32_t)n_q_heads * ROW_B;
    const u32x4_t srs = SWEEP == 1 ? make_rsrc(k + (int64_t)g * D, (uint32_t)n * k_row_bytes - (uint32_t)g * ROW_B)
                                   : make_rsrc(q + (int64_t)g * grp * D, (uint32_t)n * q_row_bytes - (uint32_t)(g * grp) * ROW_B);
    const u32x4_t lrs = make_rsrc(lse2 + (int64_t)g * n_qrows, (uint32_t)n_qrows * 4u);
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds_b);
    // One staging instruction moves 64 x 16 bytes to 1 KiB of consecutive LDS: four rows.  A wave
    // stages rows 4w .. 4w+3 of each half of the tile.  The 16-byte piece p of row r sits at
    // position p ^ (r & 15), which makes the operand reads below conflict-free; the load realises
    // it by letting lane (row, position) fetch piece position ^ (row & 15).
    const int st_row = 4 * wave + (lane >> 4);
    const uint32_t st_piece = (uint32_t)((lane & 15) ^ st_row) * 16u;
    auto stage_16 = [&](uint32_t lds_dst, uint32_t voff) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                     :: "s"(lds_dst), "v"(voff), "s"(srs));
    };
    auto stage_4 = [&](uint32_t lds_dst, uint32_t voff) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                     :: "s"(lds_dst), "v"(voff), "s"(lrs));
    };
    // Any step index is accepted and clamped to the sweep's last step, rows past the tensor to its
    // last row: the sweep requests tiles past its end (into slots nothing reads) so that every step
    // issues the same number of loads and the waits can count them.
    // Offsets of the lane's two rows inside tile 0, with the swizzled piece: a tile wholly inside the
    // tensor then only adds its own offset (sweep 2: when the group size divides 32, so that every
    // tile starts at a token boundary; otherwise the row index is split per tile).
    uint32_t st_off[2];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const uint32_t r = (uint32_t)(16 * half + st_row);
        if (SWEEP == 1) {
            st_off[half] = r * k_row_bytes + st_piece;
        } else {
            const uint32_t tok = div_grp(r), hh = r - tok * (uint32_t)grp;
            st_off[half] = tok * q_row_bytes + hh * ROW_B + st_piece;
        }
    }
    const bool even_tiles = SWEEP == 1 || TS % grp == 0;
    const uint32_t tile_bytes = SWEEP == 1 ? TS * k_row_bytes : (uint32_t)(TS / grp) * q_row_bytes;
    auto stage_tile = [&](int k) {                  // step k's tile into slot k % RING
        const uint32_t slot = lds_base + (uint32_t)((k & (RING - 1)) * SLOT_B);
        const int t = tile_of(k);
        const bool inside = even_tiles && (t + 1) * TS <= n_stream;      // uniform
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            uint32_t off;
            if (inside) {
                off = st_off[half] + (uint32_t)t * tile_bytes;
            } else {
                const int sr = min(t * TS + 16 * half + st_row, n_stream - 1);
                if (SWEEP == 1) {
                    off = (uint32_t)sr * k_row_bytes + st_piece;
                } else {
                    const uint32_t tok = div_grp((uint32_t)sr), hh = (uint32_t)sr - tok * (uint32_t)grp;
                    off = tok * q_row_bytes + hh * ROW_B + st_piece;
                }
            }
            stage_16(__builtin_amdgcn_readfirstlane(slot + (uint32_t)(16 * half + 4 * wave) * ROW_B), off);
        }
        if (SWEEP == 2 && wave == 0) {
            if (lane < TS) stage_4(__builtin_amdgcn_readfirstlane(slot + TILE_B), (uint32_t)min(t * TS + lane, n_stream - 1) * 4u);
        }
    };
    // the lane reads piece 2*ks + hf of row ln, at position (2*ks + hf) ^ (ln & 15)
    const uint32_t a_read_off = (uint32_t)(ln * ROW_B + ((hf ^ (ln & 15)) * 16));
    auto read_a = [&](uint32_t slot_off, int ks) -> u32x4_t {
        return *reinterpret_cast<const u32x4_t *>(lds_b + ((a_read_off ^ (uint32_t)(32 * ks)) + slot_off));
    };

    const floatx16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    auto scores = [&](int k, floatx16 (&s)[NB]) {
        const uint32_t slot_off = (uint32_t)((k & (RING - 1)) * SLOT_B);
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            const u32x4_t a = read_a(slot_off, ks);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), bfix[nb][ks], ks == 0 ? zero : s[nb], 0, 0, 0);
        }
    };
    // causal mask where the tile can hold a (key, query) pair with key > query for this wave, and
    // streamed rows past the tensor; s -> -inf there
    auto mask_tile = [&](int t, floatx16 (&s)[NB]) {
        const int r0 = t * TS;
        if (SWEEP == 1) {
            if (r0 + TS - 1 > pmin) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (r0 + tile_row(r, hf) > fpos[nb]) s[nb][r] = -INFINITY;
            }
        } else {
            const int tok0 = (int)div_grp((uint32_t)r0);
            if (tok0 < pmax || r0 + TS > n_stream) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int sr = r0 + tile_row(r, hf);
                    const int tok = (int)div_grp((uint32_t)sr);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        if (tok < fpos[nb] || sr >= n_stream) s[nb][r] = -INFINITY;
                }
            }
        }
    };
    // wave 0 issues one more load per tile in sweep 2 (the log-sum-exps)
    auto step_barrier = [&]() {
        if (SWEEP == 2 && wave == 0) KVS_CS_BARRIER(6);
        else KVS_CS_BARRIER(4);
    };
    // One sweep over the streamed tiles; f(k, t, s) consumes the masked scores of step k = tile t.
    // At the top of step k the loads of steps k .. k+2 have been sent; the barrier makes step k's
    // tile visible to every wave and tells that every wave is done with step k-1, whose slot step
    // k+3 then takes.
    auto sweep = [&](auto f) {
#pragma unroll
        for (int i = 0; i < RING - 1; ++i) stage_tile(i);
        for (int k = 0; k < n_tiles; ++k) {
            step_barrier();
            stage_tile(k + RING - 1);
            const int t = tile_of(k);
            floatx16 s[NB];
            scores(k, s);
            mask_tile(t, s);
            f(k, t, s);
        }
        // nothing may still be on its way into LDS when the ring is reused or the workgroup ends
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    };

    float acc[NB];
    if (SWEEP == 1) {
        float ref[NB] = {0.f, 0.f};
        for (int pass = 0; pass < 2; ++pass) {
            if (pass == 1) {
                // exact row maxima
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) ref[nb] = -INFINITY;
                sweep([&](int, int, floatx16 (&s)[NB]) {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) ref[nb] = fmaxf(ref[nb], s[nb][r]);
                });
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) ref[nb] = fmaxf(ref[nb], __shfl_xor(ref[nb], 32)) * scale_log2;
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) acc[nb] = 0.f;
            sweep([&](int k, int, floatx16 (&s)[NB]) {
                if (pass == 0 && k == 0) {
                    // the reference: the largest score of the row's first tile (key 0 is never masked)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        float mx = s[nb][0];
#pragma unroll
                        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[nb][r]);
                        ref[nb] = fmaxf(mx, __shfl_xor(mx, 32)) * scale_log2 + kRefShift;
                    }
                }
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        acc[nb] += __builtin_amdgcn_exp2f(fmaf(s[nb][r], scale_log2, -ref[nb]));
            });
            bool bad = false;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                acc[nb] += __shfl_xor(acc[nb], 32);
                bad |= !(acc[nb] < 1.2676506e30f);          // 2^100; also true for inf and nan
            }
            if (pass == 1) break;
            if (tid == 0) redo_flag = 0;
            __syncthreads();
            if (bad) redo_flag = 1;
            __syncthreads();
            if (redo_flag == 0) break;
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
            if (hf == 0 && frow[nb] < n_fixed) lse2[(int64_t)g * n_qrows + frow[nb]] = ref[nb] + __builtin_amdgcn_logf(acc[nb]);
    } else {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[nb] = 0.f;
        sweep([&](int k, int, floatx16 (&s)[NB]) {
            const char *lp = lds_b + (k & (RING - 1)) * SLOT_B + TILE_B + 16 * hf;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float4 l4 = *reinterpret_cast<const float4 *>(lp + 32 * i);   // rows 8i + 4hf .. +3
                const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[nb] += __builtin_amdgcn_exp2f(fmaf(s[nb][4 * i + c], scale_log2, -lv[c]));
            }
        });
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            acc[nb] += __shfl_xor(acc[nb], 32);
            if (hf == 0 && frow[nb] < n_fixed) alpha[(int64_t)g * n + frow[nb]] = acc[nb];
        }
    }
}

template <int SWEEP>
kvs_status launch_sweep(const kvs_shape *shape, int64_t n, const void *q, const void *k, float scale_log2,
                        float *lse2, float *alpha, hipStream_t st)
{
    static DeviceOnce attr_once;
    const kvs_status ast = once_per_device(attr_once, [] {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&colsum_kernel<SWEEP>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        return e == hipSuccess ? KVS_OK : fail(KVS_EHIP, "kvs_attn_colsum: hipFuncSetAttribute: %s", hipGetErrorString(e));
    });
    if (ast != KVS_OK) return ast;
    const int grp = shape->n_q_heads / shape->n_kv_heads;
    const int64_t n_fixed = SWEEP == 1 ? n * grp : n;
    const int64_t blocks = (n_fixed + FIXED - 1) / FIXED;
    hipLaunchKernelGGL(colsum_kernel<SWEEP>, dim3((unsigned)(blocks * shape->n_kv_heads)), dim3(NT), LDS_BYTES, st,
                       (int)n, shape->n_q_heads, shape->n_kv_heads, (const uint16_t *)q, (const uint16_t *)k, scale_log2,
                       lse2, alpha);
    return check_launch(SWEEP == 1 ? "kvs_attn_colsum(row sums)" : "kvs_attn_colsum(column sums)");
}

} // namespace

size_t colsum_workspace_bytes(const kvs_shape *shape, int64_t n_tokens)
{
    return (size_t)n_tokens * shape->n_q_heads * sizeof(float) + 256;
}

} // namespace kvs

extern "C" kvs_status kvs_attn_colsum(const kvs_shape *shape, int64_t n_tokens, const void *q, const void *k,
                                      float scale, float *alpha, void *workspace, size_t workspace_bytes,
                                      void *stream)
{
    using namespace kvs;
    kvs_status st = check_shape(shape);
    if (st != KVS_OK) return st;
    if (n_tokens < 0) return fail(KVS_EINVAL, "kvs_attn_colsum: n_tokens < 0");
    if (n_tokens == 0) return KVS_OK;
    if (!isfinite(scale)) return fail(KVS_EINVAL, "kvs_attn_colsum: scale is not finite");
    if (!q || !k || !alpha) return fail(KVS_EINVAL, "kvs_attn_colsum: NULL tensor pointer");
    if (!aligned16(q) || !aligned16(k)) return fail(KVS_EINVAL, "kvs_attn_colsum: Q/K pointers must be 16-byte aligned");
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return fail(KVS_EINVAL, "kvs_attn_colsum: workspace must be given, 256-byte aligned");
    if (workspace_bytes < colsum_workspace_bytes(shape, n_tokens))
        return fail(KVS_EWORKSPACE, "kvs_attn_colsum: workspace of %zu bytes, %zu needed", workspace_bytes, colsum_workspace_bytes(shape, n_tokens));
    // the matrix-core kernel: bf16, head_dim 128, a positive scale (it folds the scale into an exp2
    // argument after taking maxima), rows addressed with 32-bit byte offsets and divided by the group
    // size with a 24-bit trick.  Everything else takes the plain vector kernels.
    const bool mfma = shape->dtype == KVS_BF16 && shape->head_dim == D && scale > 0.f;
    if (!mfma) return launch_colsum_valu(shape, n_tokens, q, k, scale, (float *)workspace, alpha, (hipStream_t)stream);
    if (n_tokens * shape->n_q_heads * (int64_t)ROW_B >= ((int64_t)1 << 32) || n_tokens * (shape->n_q_heads / shape->n_kv_heads) >= (1 << 24))
        return fail(KVS_EUNSUPPORTED, "kvs_attn_colsum: %lld tokens x %d heads exceed the 4 GiB the kernel addresses", (long long)n_tokens, shape->n_q_heads);
    float *lse2 = (float *)workspace;
    const float scale_log2 = scale * 1.4426950408889634f;
    hipStream_t hs = (hipStream_t)stream;
    st = launch_sweep<1>(shape, n_tokens, q, k, scale_log2, lse2, alpha, hs);
    if (st != KVS_OK) return st;
    return launch_sweep<2>(shape, n_tokens, q, k, scale_log2, lse2, alpha, hs);
}
