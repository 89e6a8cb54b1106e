// kvs_project_qkv: a later layer's Q, K and V of the selected tokens (App. D.1: the tokens picked in an
// early layer are the ones recomputed in the layers after it).  Recomputing a token's Q/K/V in a layer is
// that layer's projection of its hidden state; the models the paper evaluates turn Q and K by rotary
// position factors, which are applied here from a caller-supplied table while the results are still in
// registers.  One launch: gather of the selected hidden rows, the bf16 matrix product on the matrix
// cores, the rotation, the split into the Q / K / V tensors.
//
// Shape of the product: out[token, feature] = sum_c x[rows[token], c] * w[feature, c].  Both operands
// are contiguous along c, the contraction index, which is what the matrix core wants from both sides
// (8 consecutive c per lane): neither needs a transposing read.
//
// Tiling.  A workgroup owns 256 features x 256 tokens; its four waves 128 x 128 each (one wave per
// SIMD, the 16 accumulator tiles of 32 x 32 fill the accumulation registers), so every 16-byte
// operand fetched from LDS feeds four MFMAs.  The contraction runs in steps of 32; a step's two
// tiles (256 rows x 64 bytes each) are staged from global memory straight into LDS by buffer loads
// with the LDS flag -- the gather costs nothing, every lane supplies the address of its own row --
// into a ring of five stages, two to four steps ahead of their use, one barrier per step.  Rows are 64
// bytes in LDS; the 16-byte pieces of a row are permuted per row (row_swizzle) so that the lanes an operand
// read serves together never share a bank (the plain layout and a swizzle by (r >> 1) & 3 both measured
// one conflict cycle per active LDS cycle).
//
// The features are the MFMA's rows and the tokens its columns: a lane then ends up with four
// consecutive features of one token per accumulator quad, so the rotation pairs (c, c + 64) sit in
// the same lane (feature blocks fb and fb + 2 of the wave's head).  The rotary table rows come in and
// the results go out through LDS, as whole rows.
//
// Launch order.  Workgroup b runs on XCD b % 8.  The grid of tiles (feature tiles x token tiles) is cut
// into eight blocks, fx along the features and 8 / fx along the tokens, one block per XCD: what an XCD
// pulls through its L2 is then its block's rows of weights plus its block's hidden rows, and the cut is
// chosen for the smallest block first (the launch is as long as the fullest XCD) and the smallest sum of
// the two after that.
#include "kvs_internal.h"

#include <type_traits>

namespace kvs {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int PD = 128;                 // head_dim
constexpr int PBM = 256;                // tokens per workgroup tile
constexpr int PBN = 256;                // features per workgroup tile (two heads)
constexpr int PBK = 32;                 // contraction step
constexpr int PSTAGES = 5;              // ring slots of 32 KiB: 5 fill the 160 KiB of a compute unit
constexpr int PNT = 256;
constexpr int PROW_B = PBK * 2;         // bytes of a tile row in LDS
constexpr int PTILE_B = 256 * PROW_B;   // one operand tile: 16 KiB
constexpr int PSTAGE_B = 2 * PTILE_B;   // weights, then tokens
constexpr int PLDS_BYTES = PSTAGES * PSTAGE_B;
constexpr int PXCDS = 8;

// position of the 16-byte piece p of tile row r inside the row's 64 bytes: p ^ row_swizzle(r).  Rows are 64
// bytes apart, so rows r, r+4, r+8, r+12 meet in the same quarter of a 256-byte bank line and rows r, r+2,
// r+4, r+6 in the same half of a 128-byte one: the two bits below are a one-to-one image of (r3, r2) and of
// (r2, r1) alike, so lanes reading the same piece of neighbouring rows never share a bank either way.
__device__ __forceinline__ int row_swizzle(int r) { return ((r >> 2) & 1) | ((((r >> 3) ^ (r >> 1)) & 1) << 1); }

__device__ __forceinline__ bf16x8 as_frag(u32x4_t v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

__global__ __launch_bounds__(PNT, 1) void project_qkv_kernel(
    int n_q_heads, int n_kv_heads, int hidden, const uint16_t *__restrict__ x, int64_t n_tokens,
    const int32_t *__restrict__ x_rows, const int32_t *__restrict__ sel_pos, int n_sel,
    const uint16_t *__restrict__ w, const float *__restrict__ rope, int rope_positions,
    uint16_t *__restrict__ q_out, uint16_t *__restrict__ k_out, uint16_t *__restrict__ v_out,
    int tiles_m, int tiles_n, int xcd_fx, int block_n, int block_m)
{
    extern __shared__ __attribute__((aligned(16))) char plds[];
    const int tid = threadIdx.x, lane = tid & 63, ln = lane & 31, hf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wf = wave & 1, wt = wave >> 1;      // which 128 features / 128 tokens of the tile
    // the XCD's block of the tile grid, walked with the feature tile running fastest
    const int xcd = (int)(blockIdx.x % PXCDS), in_block = (int)(blockIdx.x / PXCDS);
    const int tile_n = (xcd % xcd_fx) * block_n + in_block % block_n, tile_m = (xcd / xcd_fx) * block_m + in_block / block_n;
    if (tile_n >= tiles_n || tile_m >= tiles_m) return;      // uniform: blocks at the edges of the grid are not full
    const int m0 = tile_m * PBM, n0 = tile_n * PBN;
    const int nk = hidden / PBK;

    // ---- staging: one instruction moves 64 x 16 bytes = 16 tile rows; a wave stages rows
    // 64 w .. 64 w + 63 of the weight tile and of the token tile, 8 instructions per step
    const uint32_t row_bytes = (uint32_t)hidden * 2u;
    const int st_row = lane >> 2, st_pos = lane & 3;
    uint32_t voff_w[4], voff_x[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = 64 * wave + 16 * i + st_row;                   // row of the tile
        const uint32_t piece = (uint32_t)(st_pos ^ row_swizzle(r)) * 16u;
        voff_w[i] = (uint32_t)(n0 + r) * row_bytes + piece;
        const int t = min(m0 + r, n_sel - 1);                         // rows past the end repeat the last token (never stored)
        int64_t xr = x_rows ? (int64_t)x_rows[t] : (int64_t)t;
        xr = min(max(xr, (int64_t)0), n_tokens - 1);                  // memory safety; the caller guarantees the range
        voff_x[i] = (uint32_t)xr * row_bytes + piece;
    }
    const int n_features = (n_q_heads + 2 * n_kv_heads) * PD;
    auto make_rsrc = [&](const uint16_t *base, uint64_t bytes) -> u32x4_t {
        const uint64_t a = reinterpret_cast<uint64_t>(base);
        u32x4_t r = {(uint32_t)a, (uint32_t)(a >> 32) & 0xffffu, (uint32_t)bytes, 0x00020000u};
        r.x = __builtin_amdgcn_readfirstlane(r.x);
        r.y = __builtin_amdgcn_readfirstlane(r.y);
        r.z = __builtin_amdgcn_readfirstlane(r.z);
        return r;
    };
    const u32x4_t wrs = make_rsrc(w, (uint64_t)n_features * row_bytes);
    const u32x4_t xrs = make_rsrc(x, (uint64_t)n_tokens * row_bytes);
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)plds);
    // the offsets above came through ordinary loads: none may be outstanding when the counted waits begin
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    auto stage_1k = [&](const u32x4_t &rs, uint32_t lds_dst, uint32_t voff, uint32_t soff) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                     :: "s"(lds_dst), "v"(voff), "s"(rs), "s"(soff));
    };
    // Contraction steps 2t and 2t+1 are the two halves of the same 128-byte lines of global memory and are
    // requested as a pair, a row group's first half right before its second.  Load k of a pair (0..15): row
    // group k / 4; weights for k % 4 < 2, tokens otherwise; first step of the pair for even k.  Steps
    // past the end repeat the last one (their slots are never read).
    auto stage_one = [&](int first_step, int slot_a, int slot_b, int k) {
        const int i = k >> 2, second = k & 1, tokens = (k >> 1) & 1;
        const int ks = min(first_step + second, nk - 1);
        const uint32_t soff = __builtin_amdgcn_readfirstlane((uint32_t)ks * (uint32_t)(PBK * 2));
        const uint32_t dst = lds_base + (uint32_t)((second ? slot_b : slot_a) * PSTAGE_B) + (uint32_t)(64 * wave + 16 * i) * PROW_B
                             + (uint32_t)(tokens ? PTILE_B : 0);
        stage_1k(tokens ? xrs : wrs, __builtin_amdgcn_readfirstlane(dst), tokens ? voff_x[i] : voff_w[i], soff);
    };

    // ---- operand reads: lane (ln, hf) reads piece 2 ks + hf of row (block base + ln)
    const uint32_t rd_off = (uint32_t)(ln * PROW_B + ((hf ^ row_swizzle(ln)) * 16));
    auto read_frag = [&](uint32_t tile_off, int block, int ks) -> u32x4_t {      // tile_off: byte offset of the operand tile
        return *reinterpret_cast<const u32x4_t *>(plds + tile_off + (uint32_t)(block * 32 * PROW_B) + (rd_off ^ (uint32_t)(32 * ks)));
    };

    floatx16 acc[4][4];     // [feature block][token block]
#pragma unroll
    for (int fb = 0; fb < 4; ++fb)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[fb][tb][r] = 0.f;

    // Software pipeline.  Step j multiplies with the first half of its operands (read from LDS during step
    // j-1) while it fetches the second half, passes the step's one barrier, fetches the first half of
    // step j+1 and multiplies with the second half: the matrix pipe has work on both sides of the barrier.
    // Everything is issued in order, so what must overlap is interleaved in program order and pinned there
    // with scheduling fences: per 4 MFMAs two LDS fetches and one global -> LDS load.  (LDS takes one 16-byte
    // fetch per ~9 clocks from the four waves together and the texture path one 1 KiB load per ~23: issued in
    // bursts they hold up the MFMAs behind them -- fetches in a block cost 1760 clocks per step against 1024 of
    // matrix work, a step's loads in a block another 40 %.)
    //
    // Slots and waits.  The slot of step s is read from the barrier of step s-1 to the barrier of step s.
    // The pair (e+4, e+5), e even, takes the slots of steps e-1 and e and goes out in four quarters
    // after the barrier of step e: second half of e, both halves of e+1, first half of e+2; it is needed at
    // the barriers of e+3 (first step) and e+4 (second), a full step after its last load.  So at an even
    // step's barrier the youngest pair (16 loads) is complete behind the one needed, and at an odd step's
    // barrier 8 loads of the next pair plus the last load of the needed pair (which belongs to its second
    // step) may be in flight.  Each wave waits for its own loads and LDS fetches, the barrier covers the
    // others'.
    static_assert(PSTAGES == 5, "the waits below are counted for five slots");
#pragma unroll
    for (int k = 0; k < 16; ++k) stage_one(0, 0, 1, k);
#pragma unroll
    for (int k = 0; k < 12; ++k) stage_one(2, 2, 3, k);                 // (its last quarter goes out in step 0, as in every even step)
    asm volatile("s_waitcnt vmcnt(13)\n\ts_barrier" ::: "memory");      // step 0 has landed
    u32x4_t a0[4], b0[4];
    {
        const uint32_t w_tile = (uint32_t)(wf * 128 * PROW_B), x_tile = (uint32_t)(PTILE_B + wt * 128 * PROW_B);
#pragma unroll
        for (int i = 0; i < 4; ++i) { a0[i] = read_frag(w_tile, i, 0); b0[i] = read_frag(x_tile, i, 0); }
    }
    // one half of a step: 16 MFMAs with (a_use, b_use); the fetches of (a_get, b_get) from the given tiles, ks;
    // loads quarter*4 .. quarter*4+3 of the pair that starts at `pair_step`
    auto half = [&](const u32x4_t (&a_use)[4], const u32x4_t (&b_use)[4], u32x4_t (&a_get)[4], u32x4_t (&b_get)[4],
                    uint32_t w_from, uint32_t x_from, int ks, int pair_step, int slot_a, int slot_b, int quarter) {
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            const int fb = g >> 1, tb0 = 2 * (g & 1);
            acc[fb][tb0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(a_use[fb]), as_frag(b_use[tb0]), acc[fb][tb0], 0, 0, 0);
            acc[fb][tb0 + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(a_use[fb]), as_frag(b_use[tb0 + 1]), acc[fb][tb0 + 1], 0, 0, 0);
            if (g < 4) b_get[g] = read_frag(x_from, g, ks);      // the token operands first: the next half's first MFMAs
            else a_get[g - 4] = read_frag(w_from, g - 4, ks);    // need all four of them and one weight operand
            if (g & 1) stage_one(pair_step, slot_a, slot_b, 4 * quarter + (g >> 1));
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto wrap = [](int s) { return s >= PSTAGES ? s - PSTAGES : s; };
    int slot = 0;           // ring slot of step e
    for (int e = 0; e < nk; e += 2) {      // nk is even
        const int s1 = wrap(slot + 1), s2 = wrap(slot + 2), s3 = wrap(slot + 3), s4 = wrap(slot + 4);
        auto w_of = [&](int sl) { return (uint32_t)(sl * PSTAGE_B) + (uint32_t)(wf * 128 * PROW_B); };
        auto x_of = [&](int sl) { return (uint32_t)(sl * PSTAGE_B) + (uint32_t)(PTILE_B + wt * 128 * PROW_B); };
        u32x4_t a1[4], b1[4];
        // even step e: pair (e+2, e+3) sits in slots s2, s3; pair (e+4, e+5) goes to slots s4 and `slot`
        half(a0, b0, a1, b1, w_of(slot), x_of(slot), 1, e + 2, s2, s3, 3);
        asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        half(a1, b1, a0, b0, w_of(s1), x_of(s1), 0, e + 4, s4, slot, 0);
        // odd step e+1
        half(a0, b0, a1, b1, w_of(s1), x_of(s1), 1, e + 4, s4, slot, 1);
        asm volatile("s_waitcnt vmcnt(9) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        half(a1, b1, a0, b0, w_of(s2), x_of(s2), 0, e + 4, s4, slot, 2);
        slot = s2;
    }
    // nothing may still be on its way into LDS when the workgroup ends
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- epilogue: rotate, convert, store -----------------------------------------------------------
    // entry r of acc[fb][tb]: feature 32 fb + 8 (r >> 2) + 4 hf + (r & 3) of the wave's head, token 32 tb + ln.
    // A lane's results are 8-byte pieces of 128 different rows and the rotary factors it needs are 32-byte
    // pieces of its tokens' table rows: written and read that way, a tile spent as long in its epilogue as
    // in 50 contraction steps.  Both go through LDS instead (the ring is free now): the table rows of the
    // tile's 256 tokens come in as whole rows, the results leave as whole rows.
    const int head = n0 / PD + wf;
    uint16_t *dst;
    int heads_of_dst, h_local;
    if (head < n_q_heads) { dst = q_out; heads_of_dst = n_q_heads; h_local = head; }
    else if (head < n_q_heads + n_kv_heads) { dst = k_out; heads_of_dst = n_kv_heads; h_local = head - n_q_heads; }
    else { dst = v_out; heads_of_dst = n_kv_heads; h_local = head - n_q_heads - n_kv_heads; }
    const bool turned = rope != nullptr && head < n_q_heads + n_kv_heads;
    const bool tile_turned = rope != nullptr && n0 / PD < n_q_heads + n_kv_heads;      // uniform over the workgroup
    __syncthreads();                                   // every wave is done with the ring
    if (tile_turned) {
        // table rows of tokens 64 w .. 64 w + 63 of the tile, two rows (2 x 512 bytes) per instruction, straight
        // into LDS; the 16-byte piece p of token T's row sits at position p ^ (T & 31), so that the 32 lanes of
        // a half-wave, which hold 32 consecutive tokens and want the same piece, read 32 different columns
        const int t_mine = min(m0 + 64 * wave + lane, n_sel - 1);
        int p_mine = sel_pos[t_mine];
        p_mine = min(max(p_mine, 0), rope_positions - 1);          // memory safety; the caller guarantees the range
        const uint64_t ra = reinterpret_cast<uint64_t>(rope);
        u32x4_t rrs = {(uint32_t)ra, (uint32_t)(ra >> 32) & 0xffffu, (uint32_t)rope_positions * (uint32_t)(PD * 4), 0x00020000u};
        rrs.x = __builtin_amdgcn_readfirstlane(rrs.x);
        rrs.y = __builtin_amdgcn_readfirstlane(rrs.y);
        rrs.z = __builtin_amdgcn_readfirstlane(rrs.z);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll 4
        for (int i = 0; i < 32; ++i) {
            const int tok = 2 * i + hf;                             // token of the wave's 64 this lane fetches a piece of
            const int p = __shfl(p_mine, tok);
            const uint32_t voff = (uint32_t)p * (uint32_t)(PD * 4) + (uint32_t)((ln ^ (tok & 31)) * 16);
            stage_1k(rrs, __builtin_amdgcn_readfirstlane(lds_base + (uint32_t)((64 * wave + 2 * i) * (PD * 4))), voff, 0u);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (turned) {
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) {
                const int T = 128 * wt + 32 * tb + ln;              // token of the tile; T & 31 == ln
                const char *row = plds + T * (PD * 4);
#pragma unroll
                for (int fb = 0; fb < 2; ++fb)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const int piece = (32 * fb + 8 * r4 + 4 * hf) / 2;      // (cos, sin) of channels c0, c0+1; the next piece: c0+2, c0+3
                        const float4 cs01 = *reinterpret_cast<const float4 *>(row + ((piece ^ ln) * 16));
                        const float4 cs23 = *reinterpret_cast<const float4 *>(row + (((piece + 1) ^ ln) * 16));
                        const float cs[4] = {cs01.x, cs01.z, cs23.x, cs23.z}, sn[4] = {cs01.y, cs01.w, cs23.y, cs23.w};
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float y1 = acc[fb][tb][4 * r4 + i], y2 = acc[fb + 2][tb][4 * r4 + i];
                            acc[fb][tb][4 * r4 + i] = y1 * cs[i] - y2 * sn[i];
                            acc[fb + 2][tb][4 * r4 + i] = y2 * cs[i] + y1 * sn[i];
                        }
                    }
            }
        }
        __syncthreads();                               // the table rows have been read: LDS is free again
    }
    // results -> this wave's LDS region [128 tokens][264 bytes] (the 8 bytes of padding spread a half-wave's
    // 32 rows over all banks) -> whole rows of 256 bytes to global memory, four rows per store instruction
    constexpr int OROW_B = PD * 2 + 8;
    char *region = plds + wave * (128 * OROW_B);
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
        for (int fb = 0; fb < 4; ++fb)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int c0 = 32 * fb + 8 * r4 + 4 * hf;
                *reinterpret_cast<uint2 *>(region + (32 * tb + ln) * OROW_B + 2 * c0) =
                    make_uint2(pack_bf16x2(acc[fb][tb][4 * r4 + 0], acc[fb][tb][4 * r4 + 1]), pack_bf16x2(acc[fb][tb][4 * r4 + 2], acc[fb][tb][4 * r4 + 3]));
            }
    // (same wave wrote and reads: LDS handles a wave's requests in order, no barrier)
    const int sub = lane >> 4, chunk = lane & 15;
#pragma unroll 4
    for (int i = 0; i < 32; ++i) {
        const int tok = 4 * i + sub;
        const int t = m0 + 128 * wt + tok;
        const uint2 lo = *reinterpret_cast<const uint2 *>(region + tok * OROW_B + 16 * chunk);
        const uint2 hi = *reinterpret_cast<const uint2 *>(region + tok * OROW_B + 16 * chunk + 8);
        if (t < n_sel)
            *reinterpret_cast<uint4 *>(dst + ((int64_t)t * heads_of_dst + h_local) * PD + 8 * chunk) = make_uint4(lo.x, lo.y, hi.x, hi.y);
    }
}

} // namespace
} // namespace kvs

extern "C" kvs_status kvs_project_qkv(const kvs_shape *shape, int32_t hidden, const void *x, int64_t n_tokens,
                                      const int32_t *x_rows, const int32_t *sel_pos, int64_t n_sel,
                                      const void *w_qkv, const float *rope, int64_t rope_positions,
                                      void *q_out, void *k_out, void *v_out, void *stream)
{
    using namespace kvs;
    kvs_status st = check_shape(shape);
    if (st != KVS_OK) return st;
    if (n_tokens < 0 || n_sel < 0) return fail(KVS_EINVAL, "kvs_project_qkv: negative size");
    if (shape->dtype != KVS_BF16 || shape->head_dim != PD)
        return fail(KVS_EUNSUPPORTED, "kvs_project_qkv: bf16 with head_dim 128 is built");
    if ((shape->n_q_heads + 2 * shape->n_kv_heads) % 2 != 0)
        return fail(KVS_EUNSUPPORTED, "kvs_project_qkv: an odd number of heads in all (a workgroup takes two)");
    if (hidden < 2 * PBK || hidden % (2 * PBK) != 0) return fail(KVS_EUNSUPPORTED, "kvs_project_qkv: hidden size %d (multiples of %d)", hidden, 2 * PBK);
    if (n_sel == 0) return KVS_OK;
    if (n_tokens == 0) return fail(KVS_EINVAL, "kvs_project_qkv: tokens selected from an empty x");
    if (!x_rows && n_sel > n_tokens) return fail(KVS_EINVAL, "kvs_project_qkv: n_sel %lld exceeds the rows of x", (long long)n_sel);
    if (!x || !w_qkv || !q_out || !k_out || !v_out) return fail(KVS_EINVAL, "kvs_project_qkv: NULL tensor pointer");
    if (rope && (!sel_pos || rope_positions <= 0)) return fail(KVS_EINVAL, "kvs_project_qkv: a rotary table needs sel_pos and its own length");
    if (!aligned16(x) || !aligned16(w_qkv) || !aligned16(q_out) || !aligned16(k_out) || !aligned16(v_out) || (rope && !aligned16(rope)))
        return fail(KVS_EINVAL, "kvs_project_qkv: tensors must be 16-byte aligned");
    const int64_t features = (int64_t)(shape->n_q_heads + 2 * shape->n_kv_heads) * PD;
    // rows are addressed with 32-bit byte offsets
    if (n_tokens * hidden * 2 >= ((int64_t)1 << 32) || features * hidden * 2 >= ((int64_t)1 << 32))
        return fail(KVS_EUNSUPPORTED, "kvs_project_qkv: x or w of 4 GiB or more");
    if (n_sel > 0x7fffffff) return fail(KVS_EUNSUPPORTED, "kvs_project_qkv: too many tokens");
    if (rope && rope_positions * (int64_t)(PD * 4) >= ((int64_t)1 << 32)) return fail(KVS_EUNSUPPORTED, "kvs_project_qkv: rotary table of 4 GiB or more");
    static DeviceOnce attr_once;
    st = once_per_device(attr_once, [] {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&project_qkv_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, PLDS_BYTES);
        return e == hipSuccess ? KVS_OK : fail(KVS_EHIP, "kvs_project_qkv: hipFuncSetAttribute: %s", hipGetErrorString(e));
    });
    if (st != KVS_OK) return st;
    const int64_t tiles_m = (n_sel + PBM - 1) / PBM, tiles_n = features / PBN;
    int fx = PXCDS;
    int64_t block_n = 0, block_m = 0;
    for (int f = PXCDS; f >= 1; f >>= 1) {
        const int64_t bn = (tiles_n + f - 1) / f, bm = (tiles_m + PXCDS / f - 1) / (PXCDS / f);
        if (block_n == 0 || bn * bm < block_n * block_m || (bn * bm == block_n * block_m && bn + bm < block_n + block_m)) {
            fx = f; block_n = bn; block_m = bm;
        }
    }
    const int64_t per_xcd = block_n * block_m;
    if (per_xcd * PXCDS > 0x7fffffff) return fail(KVS_EUNSUPPORTED, "kvs_project_qkv: too many tiles");
    hipLaunchKernelGGL(project_qkv_kernel, dim3((unsigned)(per_xcd * PXCDS)), dim3(PNT), PLDS_BYTES, (hipStream_t)stream,
                       shape->n_q_heads, shape->n_kv_heads, (int)hidden, (const uint16_t *)x, n_tokens, x_rows, sel_pos, (int)n_sel,
                       (const uint16_t *)w_qkv, rope, (int)rope_positions, (uint16_t *)q_out, (uint16_t *)k_out, (uint16_t *)v_out,
                       (int)tiles_m, (int)tiles_n, fx, (int)block_n, (int)block_m);
    return check_launch("kvs_project_qkv");
}
