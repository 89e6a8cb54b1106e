// Partial-recompute attention on the gfx950 matrix cores, large-launch variant: 64 query rows per
// wave, one wave per SIMD, software-pipelined over K/V tiles of 32 keys.
//
// Why this shape.  Feeding every v_mfma_f32_32x32x16_bf16 with a fresh 16-byte-per-lane operand
// from LDS saturates the LDS read pipe (measured: the MFMA rate drops to ~75 % with nothing else
// going on).  Here each K row block / V^T row block read from LDS is used by two MFMAs (two
// blocks of 32 queries), which halves the LDS traffic per flop.  Two query blocks per wave need
// the whole register file (output accumulators 128, Q operands 64, two score tiles 64, ...), so
// one wave per SIMD is resident and the overlap of matrix and vector work has to come from within
// the wave: the score product of tile j+1 is issued before the softmax of tile j, whose vector
// instructions then run in the shadow of those MFMAs; the PV product of tile j follows.  The
// softmax uses a per-row exponent reference that is fixed for the whole sweep (taken from the
// row's first tile, with an exact-maximum fallback sweep if that ever overflows), so the output
// accumulators are only ever touched by MFMAs and stay in the accumulation registers.
//
// Everything else follows the 32-rows-per-wave kernel: rows are flattened (selected token,
// head-in-group), transposed products S^T = K Q^T and O^T += V^T P^T so that P stays in registers
// as the B operand, K rows fed in a bit-swapped order so that a lane's 8 P values per k-step are 8
// consecutive keys, V transposed on its way into LDS, exp2 with the scale folded in, causal compare
// only on tiles that can straddle a row position of the wave, heaviest row tiles first, KV head =
// blockIdx % n_kv_heads.
//
// LDS ring of three stages (K tile, V^T tile).  In iteration j the wave reads K of tile j+1 and
// V^T of tile j and, at the bottom, writes tile j+2 into the stage that held tile j-1; one barrier
// per iteration.
#include "attention.h"

#include <math.h>

namespace kvs {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int D = 128;             // head_dim
constexpr int BN = 32;             // keys per tile
constexpr int NWAVES = 4;
constexpr int NB = 2;              // 32-row query blocks per wave
constexpr int NT = NWAVES * 64;
constexpr int WROWS = 32 * NB;
constexpr int ROWS = NWAVES * WROWS;   // 256 rows per workgroup
constexpr int K_LD = D + 8;        // K tile row pitch in bf16 (272 B)
constexpr int V_LD = BN + 8;       // V^T tile row pitch in bf16 (80 B)
constexpr int K_TILE = BN * K_LD;
constexpr int V_TILE = D * V_LD;
constexpr int STAGE = K_TILE + V_TILE;
constexpr int NSTAGE = 3;
constexpr int K_PIECES = BN * (D / 8) / NT;   // 2
static_assert(K_PIECES == 2 && (BN / 8) == NWAVES, "tile staging assumes 256 lanes and 32 keys");

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// Sum of the eight bf16 values of a packed P operand, exactly as the matrix core will see them.
// The softmax normaliser is built from these rounded weights, not from the fp32 ones: numerator
// and denominator then carry the same rounding, so a row dominated by a single key still returns
// that key's V exactly (with a fixed exponent reference the dominant weight is not 1.0 and its
// bf16 rounding error, up to 2^-9, would otherwise pass straight into the output).
__device__ __forceinline__ float rounded_sum(const u32x4_t w)
{
    return ((bf16_lo(w.x) + bf16_hi(w.x)) + (bf16_lo(w.y) + bf16_hi(w.y))) +
           ((bf16_lo(w.z) + bf16_hi(w.z)) + (bf16_lo(w.w) + bf16_hi(w.w)));
}

// WANT_LSE: additionally keep the unrounded sum of weights, from which the log-sum-exp is reported
template <bool WANT_LSE>
__global__ __launch_bounds__(NT, 1) void attn_mfma2_kernel(
    const AttnTiles td, int n_q_heads, int n_kv_heads, int total_tiles,
    const uint16_t *__restrict__ q_sel, const int32_t *__restrict__ sel_pos,
    const uint16_t *__restrict__ k_cache, const uint16_t *__restrict__ v_cache,
    float scale_log2, uint16_t *__restrict__ out, float *__restrict__ lse_out)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];   // NSTAGE x (K tile, V^T tile)
    __shared__ int wg_max_pos[NWAVES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, ln = lane & 31;

    // ---- which (request, kv head, row tile) -----------------------------------------------------
    const int g = blockIdx.x % n_kv_heads;
    const int tile_lin = total_tiles - 1 - (int)(blockIdx.x / n_kv_heads);
    int b = 0;
    while (b + 1 < td.n_req && tile_lin >= td.tile_begin[b + 1]) ++b;
    const int tile = tile_lin - td.tile_begin[b];
    const int grp = n_q_heads / n_kv_heads;
    const int64_t sel0 = td.cu_sel[b];
    const int n_rows = (int)(td.cu_sel[b + 1] - sel0) * grp;
    const int ctx_len = td.ctx_len[b];
    const int64_t ctx_off = td.ctx_off[b];

    // this lane's query rows, one per 32-row block (both half-waves hold the same queries)
    bool row_ok[NB];
    int pos[NB];
    int64_t row_idx[NB];
    int pmin = 0x7fffffff, pmax = 0;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int rq = tile * ROWS + wave * WROWS + nb * 32 + ln;
        row_ok[nb] = rq < n_rows;
        const int rqc = row_ok[nb] ? rq : n_rows - 1;
        const int t_sel = rqc / grp, hh = rqc - t_sel * grp;
        const int64_t s_glob = sel0 + t_sel;
        int p = sel_pos[s_glob];
        p = min(max(p, 0), ctx_len - 1);             // memory safety; the caller guarantees the range
        pos[nb] = p;
        row_idx[nb] = s_glob * n_q_heads + g * grp + hh;
        pmin = min(pmin, p);
        pmax = max(pmax, p);
    }
#pragma unroll
    for (int o = 1; o < 32; o <<= 1) {
        pmin = min(pmin, __shfl_xor(pmin, o));
        pmax = max(pmax, __shfl_xor(pmax, o));
    }
    if (lane == 0) wg_max_pos[wave] = pmax;

    // ---- Q as the B operand: Q[query ln][16*ks + 8*hf + j] ----------------------------------------
    bf16x8 qreg[NB][D / 16];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            qreg[nb][ks] = as_bf16x8(*reinterpret_cast<const u32x4_t *>(q_sel + row_idx[nb] * D + 16 * ks + 8 * hf));

    // Q is only ever an MFMA operand: park it in the accumulation half of the register file so the
    // vector half is left to the softmax and the tile staging
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) asm volatile("" : "+a"(qreg[nb][ks]));

    __syncthreads();
    int wg_pmax = wg_max_pos[0];
#pragma unroll
    for (int w = 1; w < NWAVES; ++w) wg_pmax = max(wg_pmax, wg_max_pos[w]);
    const int n_kv_tiles = wg_pmax / BN + 1;

    // ---- global -> register -> LDS staging of one K/V tile ------------------------------------------
    const uint32_t row_bytes = (uint32_t)n_kv_heads * D * 2u;          // bytes between tokens
    const char *kbase = reinterpret_cast<const char *>(k_cache + (ctx_off * n_kv_heads + g) * (int64_t)D);
    const char *vbase = reinterpret_cast<const char *>(v_cache + (ctx_off * n_kv_heads + g) * (int64_t)D);
    struct Staged { u32x4_t k[K_PIECES]; uint32_t v[8]; };   // one tile on its way from HBM to LDS
    const uint32_t k_lane_off = (uint32_t)(tid >> 4) * row_bytes + (uint32_t)(tid & 15) * 16u;
    const uint32_t v_lane_off = (uint32_t)lane * 4u;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);

    // tile jt wholly inside the context: uniform tile base + constant per-lane offsets
    auto load_tile_inside = [&](int jt, Staged &st) {
        const char *kt = kbase + (int64_t)jt * BN * row_bytes;
        const char *vt = vbase + ((int64_t)jt * BN + 8 * wave_u) * row_bytes;
#pragma unroll
        for (int i = 0; i < K_PIECES; ++i)
            st.k[i] = *reinterpret_cast<const u32x4_t *>(kt + (size_t)(i * (NT / 16)) * row_bytes + k_lane_off);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            st.v[j] = *reinterpret_cast<const uint32_t *>(vt + (size_t)j * row_bytes + v_lane_off);
    };
    auto load_tile = [&](int jt, Staged &st) {      // any tile: rows past the context are clamped
        const int kv0 = jt * BN;
        if (kv0 + BN <= ctx_len) {
            load_tile_inside(jt, st);
        } else {
#pragma unroll
            for (int i = 0; i < K_PIECES; ++i) {
                const int key = min(kv0 + i * (NT / 16) + (tid >> 4), ctx_len - 1);
                st.k[i] = *reinterpret_cast<const u32x4_t *>(kbase + (int64_t)key * row_bytes + (tid & 15) * 16);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int key = min(kv0 + 8 * wave_u + j, ctx_len - 1);
                st.v[j] = *reinterpret_cast<const uint32_t *>(vbase + (int64_t)key * row_bytes + v_lane_off);
            }
        }
    };
    auto store_tile = [&](int jt, const Staged &st) {
        uint16_t *ks = lds + (jt % NSTAGE) * STAGE;
        uint16_t *vs = ks + K_TILE;
#pragma unroll
        for (int i = 0; i < K_PIECES; ++i) {
            const int id = i * NT + tid;
            *reinterpret_cast<u32x4_t *>(ks + (id >> 4) * K_LD + (id & 15) * 8) = st.k[i];
        }
        u32x4_t lo, hi;   // channel 2*lane and 2*lane+1 of keys 8*wave .. 8*wave+7
        // v_perm_b32: bytes 0-3 come from the second operand, 4-7 from the first
        lo.x = __builtin_amdgcn_perm(st.v[1], st.v[0], 0x05040100u);
        lo.y = __builtin_amdgcn_perm(st.v[3], st.v[2], 0x05040100u);
        lo.z = __builtin_amdgcn_perm(st.v[5], st.v[4], 0x05040100u);
        lo.w = __builtin_amdgcn_perm(st.v[7], st.v[6], 0x05040100u);
        hi.x = __builtin_amdgcn_perm(st.v[1], st.v[0], 0x07060302u);
        hi.y = __builtin_amdgcn_perm(st.v[3], st.v[2], 0x07060302u);
        hi.z = __builtin_amdgcn_perm(st.v[5], st.v[4], 0x07060302u);
        hi.w = __builtin_amdgcn_perm(st.v[7], st.v[6], 0x07060302u);
        *reinterpret_cast<u32x4_t *>(vs + (2 * lane) * V_LD + 8 * wave) = lo;
        *reinterpret_cast<u32x4_t *>(vs + (2 * lane + 1) * V_LD + 8 * wave) = hi;
    };

    // ---- the three pieces of one tile's work ----------------------------------------------------------
    // K row fed to MFMA row ln: bits 2 and 3 swapped, so that accumulator entry r of a lane is key
    // 16*(r>>3) + 8*hf + (r&7) of the tile
    const int krow = (ln & ~12) | ((ln & 4) << 1) | ((ln & 8) >> 1);
    const uint32_t k_read_off = (uint32_t)(krow * K_LD + 8 * hf);      // + 16*ks
    const uint32_t v_read_off = (uint32_t)(ln * V_LD + 8 * hf);        // + 32*db*V_LD + 16*kstep

    auto qk = [&](int jt, floatx16 (&s)[NB]) {
        const uint16_t *ks = lds + (jt % NSTAGE) * STAGE;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[nb][r] = 0.f;
#pragma unroll
        for (int ksx = 0; ksx < D / 16; ++ksx) {
            const u32x4_t a = *reinterpret_cast<const u32x4_t *>(ks + k_read_off + 16 * ksx);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), qreg[nb][ksx], s[nb], 0, 0, 0);
        }
    };

    // causal compare where a key of tile jt can exceed a row position of this wave (wave-uniform test)
    auto mask_tile = [&](int jt, floatx16 (&s)[NB]) {
        const int kv0 = jt * BN;
        if (kv0 + BN - 1 > pmin) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kv0 + 16 * (r >> 3) + 8 * hf + (r & 7);
                    if (key > pos[nb]) s[nb][r] = -INFINITY;
                }
        }
    };
    // max over the tile's keys of scale*log2(e)*logit, per query (combines the two half-waves)
    auto row_max = [&](const floatx16 &s) -> float {
        float mx = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
        return fmaxf(mx, __shfl_xor(mx, 32)) * scale_log2;
    };

    floatx16 o_acc[D / 32][NB];
    float m_ref[NB], l_run[NB];   // softmax exponent reference (shared by the two half-waves) and this
                                  // half-wave's share of the running sum of (bf16-rounded) weights
    float l_exact[NB];            // same sum over the unrounded weights (WANT_LSE only)
    // P = exp2(scale*log2e*S - m_ref) -> bf16 B operands.  The reference is fixed for the whole
    // pass, so the output accumulators are touched by MFMAs only and can stay in the accumulation
    // registers; see the comment at the pass loop for why that is safe.
    auto softmax = [&](int jt, floatx16 (&s)[NB], u32x4_t (&pop)[NB][2]) {
        mask_tile(jt, s);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            float pv[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) pv[r] = __builtin_amdgcn_exp2f(fmaf(s[nb][r], scale_log2, -m_ref[nb]));
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                pop[nb][a].x = pack2(pv[8 * a + 0], pv[8 * a + 1]);
                pop[nb][a].y = pack2(pv[8 * a + 2], pv[8 * a + 3]);
                pop[nb][a].z = pack2(pv[8 * a + 4], pv[8 * a + 5]);
                pop[nb][a].w = pack2(pv[8 * a + 6], pv[8 * a + 7]);
            }
            l_run[nb] += rounded_sum(pop[nb][0]) + rounded_sum(pop[nb][1]);
            if (WANT_LSE) {
                float e = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) e += pv[r];
                l_exact[nb] += e;
            }
        }
    };
    auto pv_product = [&](int jt, const u32x4_t (&pop)[NB][2]) {
        const uint16_t *vs = lds + (jt % NSTAGE) * STAGE + K_TILE;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                const u32x4_t va = *reinterpret_cast<const u32x4_t *>(vs + v_read_off + 32 * db * V_LD + 16 * a);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    o_acc[db][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va), as_bf16x8(pop[nb][a]), o_acc[db][nb], 0, 0, 0);
            }
    };

    // One tile of the fast sweep: no masking, no tail handling, one straight-line block.  On entry
    // tiles jt and jt+1 are in the LDS ring and `held` carries tile jt+2; the global loads of tile
    // jt+3 go out first (they have this whole step and the next to land), then all LDS operands of
    // the step (K of tile jt+1, V^T of tile jt), the score MFMAs of tile jt+1 ahead of the softmax of
    // tile jt so that the vector work runs in their shadow, and the PV MFMAs of tile jt.
    auto fast_step = [&](int jt, floatx16 (&s_in)[NB], floatx16 (&s_out)[NB], const Staged &held, Staged &next) {
        load_tile_inside(jt + 3, next);
        const uint16_t *ks = lds + ((jt + 1) % NSTAGE) * STAGE;
        const uint16_t *vs = lds + (jt % NSTAGE) * STAGE + K_TILE;
        u32x4_t ka[D / 16], va[2][D / 32];
#pragma unroll
        for (int ksx = 0; ksx < D / 16; ++ksx) ka[ksx] = *reinterpret_cast<const u32x4_t *>(ks + k_read_off + 16 * ksx);
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
                va[a][db] = *reinterpret_cast<const u32x4_t *>(vs + v_read_off + 32 * db * V_LD + 16 * a);
        const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
            s_out[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ka[0]), qreg[nb][0], zero, 0, 0, 0);
#pragma unroll
        for (int ksx = 1; ksx < D / 16; ++ksx)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                s_out[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ka[ksx]), qreg[nb][ksx], s_out[nb], 0, 0, 0);
        u32x4_t pop[NB][2];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            float pv[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) pv[r] = __builtin_amdgcn_exp2f(fmaf(s_in[nb][r], scale_log2, -m_ref[nb]));
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                pop[nb][a].x = pack2(pv[8 * a + 0], pv[8 * a + 1]);
                pop[nb][a].y = pack2(pv[8 * a + 2], pv[8 * a + 3]);
                pop[nb][a].z = pack2(pv[8 * a + 4], pv[8 * a + 5]);
                pop[nb][a].w = pack2(pv[8 * a + 6], pv[8 * a + 7]);
            }
            l_run[nb] += rounded_sum(pop[nb][0]) + rounded_sum(pop[nb][1]);
            if (WANT_LSE) {
                float e = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) e += pv[r];
                l_exact[nb] += e;
            }
        }
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    o_acc[db][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va[a][db]), as_bf16x8(pop[nb][a]), o_acc[db][nb], 0, 0, 0);
        store_tile(jt + 2, held);
        __syncthreads();
    };

    // ---- passes -------------------------------------------------------------------------------------------
    // Pass 0 takes each row's exponent reference from its first tile (every row sees key 0) and
    // never moves it: softmax(x) is invariant to the reference as long as nothing overflows, and
    // fp32 / bf16 leave 2^127 of headroom.  If a row's sum ends above 2^100 (or inf / nan) some later
    // logit was more than ~2^6 above the first tile's max; then the workgroup computes the exact
    // row maxima in a score-only sweep and repeats the pass with those (pass 1), which cannot
    // overflow.  Real attention logits do not do that, so pass 1 is a correctness net.
    __shared__ int redo_flag;
    float l_tot[NB];
    for (int pass = 0; pass < 2; ++pass) {
        if (pass == 1) {
            // exact row maxima: one tile at a time through stage 0
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) m_ref[nb] = -INFINITY;
            for (int jt = 0; jt < n_kv_tiles; ++jt) {
                Staged st;
                load_tile(jt, st);
                store_tile(jt, st);
                __syncthreads();
                floatx16 s[NB];
                qk(jt, s);
                mask_tile(jt, s);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) m_ref[nb] = fmaxf(m_ref[nb], row_max(s[nb]));
                __syncthreads();
            }
        }
        // tiles 0 and 1 into the ring, tile 2 on its way, scores of tile 0
        Staged held, next;
        load_tile(0, held);
        store_tile(0, held);
        if (n_kv_tiles > 1) { load_tile(1, held); store_tile(1, held); }
        if (n_kv_tiles > 2) load_tile(2, held);
        __syncthreads();
        floatx16 s_cur[NB], s_nxt[NB];
        qk(0, s_cur);
        if (pass == 0) {
            mask_tile(0, s_cur);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) m_ref[nb] = row_max(s_cur[nb]);
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) { l_run[nb] = 0.f; l_exact[nb] = 0.f; }
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[db][nb][r] = 0.f;

        int jt = 0;
        // Fast sweep, two tiles per trip so the two score buffers swap roles without copies.  It
        // covers the tiles that need no causal compare for any row of this wave and whose look-ahead
        // tiles lie wholly inside the context; each wave leaves it at its own point and finishes in
        // the general loop below (both loops stage the same tile and hit one barrier per tile, so
        // the waves of a workgroup may sit in different loops).
        const int j_unmasked = (pmin + 1) / BN;                       // tiles 0 .. j_unmasked-1: every key <= pmin
        const int j_lookahead = min(n_kv_tiles, ctx_len / BN);        // tiles that exist and need no row clamp
        for (; jt + 1 < j_unmasked && jt + 4 < j_lookahead; jt += 2) {
            fast_step(jt, s_cur, s_nxt, held, next);
            fast_step(jt + 1, s_nxt, s_cur, next, held);
        }
        // general loop; invariant at the top: `held` carries tile jt+2 if that tile exists
        for (; jt < n_kv_tiles; ++jt) {
            if (jt + 3 < n_kv_tiles) load_tile(jt + 3, next);
            // scores of the next tile first (past the last tile the stage holds stale data and the
            // result is discarded)
            qk(jt + 1, s_nxt);
            u32x4_t pop[NB][2];
            softmax(jt, s_cur, pop);
            pv_product(jt, pop);
            if (jt + 2 < n_kv_tiles) store_tile(jt + 2, held);
            __syncthreads();
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) s_cur[nb] = s_nxt[nb];
            held = next;
        }

        bool bad = false;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            l_tot[nb] = l_run[nb] + __shfl_xor(l_run[nb], 32);
            bad |= !(l_tot[nb] < 1.2676506e30f);          // 2^100; also true for inf and nan
        }
        if (pass == 1) break;
        if (tid == 0) redo_flag = 0;
        __syncthreads();
        if (bad) redo_flag = 1;
        __syncthreads();
        if (redo_flag == 0) break;
    }

    // ---- epilogue: normalise, convert, store ----------------------------------------------------------
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const float inv = 1.0f / l_tot[nb];
        const float l_exact_tot = WANT_LSE ? l_exact[nb] + __shfl_xor(l_exact[nb], 32) : 0.f;
        if (row_ok[nb]) {
            uint16_t *orow = out + row_idx[nb] * D;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int d0 = 32 * db + 8 * r4 + 4 * hf;
                    uint2 w;
                    w.x = pack2(o_acc[db][nb][4 * r4 + 0] * inv, o_acc[db][nb][4 * r4 + 1] * inv);
                    w.y = pack2(o_acc[db][nb][4 * r4 + 2] * inv, o_acc[db][nb][4 * r4 + 3] * inv);
                    *reinterpret_cast<uint2 *>(orow + d0) = w;
                }
            if (WANT_LSE && hf == 0)
                lse_out[row_idx[nb]] = (m_ref[nb] + __builtin_amdgcn_logf(l_exact_tot)) * 0.6931471805599453f;
        }
    }
}

} // namespace

kvs_status launch_attention_mfma2(const kvs_shape *shape, const AttnBatch &bd, const void *q_sel,
                                  const int32_t *sel_pos, const void *k_cache, const void *v_cache,
                                  float scale, void *out, float *lse_out, hipStream_t st)
{
    AttnTiles td;
    const int64_t tiles = build_attn_tiles(shape, bd, ROWS, td);
    if (tiles < 0) return fail(KVS_EINVAL, "kvs_partial_attention: too many row tiles");
    if (tiles == 0) return KVS_OK;
    const size_t lds_bytes = NSTAGE * STAGE * sizeof(uint16_t);
    static bool attr_set = false;   // idempotent; a race only repeats the same call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_mfma2_kernel<false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_mfma2_kernel<true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return fail(KVS_EHIP, "kvs_partial_attention: hipFuncSetAttribute: %s", hipGetErrorString(e));
        attr_set = true;
    }
    const float scale_log2 = scale * 1.4426950408889634f;
    const dim3 grid((unsigned)(tiles * shape->n_kv_heads)), block(NT);
    if (lse_out)
        hipLaunchKernelGGL(attn_mfma2_kernel<true>, grid, block, lds_bytes, st, td, shape->n_q_heads, shape->n_kv_heads,
                           (int)tiles, (const uint16_t *)q_sel, sel_pos, (const uint16_t *)k_cache,
                           (const uint16_t *)v_cache, scale_log2, (uint16_t *)out, lse_out);
    else
        hipLaunchKernelGGL(attn_mfma2_kernel<false>, grid, block, lds_bytes, st, td, shape->n_q_heads, shape->n_kv_heads,
                           (int)tiles, (const uint16_t *)q_sel, sel_pos, (const uint16_t *)k_cache,
                           (const uint16_t *)v_cache, scale_log2, (uint16_t *)out, lse_out);
    return check_launch("kvs_partial_attention(mfma2)");
}

} // namespace kvs
