// Partial-recompute attention on the gfx950 matrix cores, large-launch variant: 64 query rows per
// wave, one wave per SIMD, software-pipelined over K/V tiles of 32 keys.
//
// Why this shape.  Feeding every v_mfma_f32_32x32x16_bf16 with a fresh 16-byte-per-lane operand
// from LDS saturates the LDS read pipe (measured: the MFMA rate drops to ~75 % with nothing else
// going on).  Here each K / V operand read from LDS is used by two MFMAs (two blocks of 32
// queries), which halves the LDS traffic per flop.  Two query blocks per wave need the whole
// register file (output accumulators 128, Q operands 64, two score tiles 64, ...), so one wave per
// SIMD is resident and the overlap of matrix, vector and memory work has to come from within the
// wave.  The softmax uses a per-row exponent reference that is fixed for the whole sweep (taken
// from the row's first tile, with an exact-maximum fallback sweep if that ever overflows), so the
// output accumulators are only ever touched by MFMAs and stay in the accumulation registers.
//
// As in the 32-rows-per-wave kernel, rows are flattened (selected token, head-in-group), the
// products are transposed (S^T = K Q^T, O^T += V^T P^T) so that P stays in registers as the B
// operand, K rows are fed in a bit-swapped order so that a lane's 8 P values per k-step are 8
// consecutive keys, exp2 carries the scale, the heaviest row tiles come first and the KV head is
// blockIdx % n_kv_heads.  Unlike there, V stays row-major in LDS and the V^T operand is produced
// by the transposing LDS read, so K and V are staged by the same plain 16-byte copies.
//
// Software pipeline.  Step j issues, for one wave, three independent strands:
//   * the score MFMAs of tile j+1        (K tile j+1 from LDS, Q from registers),
//   * the PV MFMAs of tile j-1           (V tile j-1 from LDS, P of tile j-1 from registers),
//   * the softmax of tile j              (vector instructions only),
// so every MFMA of the step has vector work that can run beside it.  Tiles that need the causal
// compare go through the same pipeline with two more vector instructions per score.
//
// Staging.  K and V tiles go from global memory straight into LDS (buffer loads with the LDS
// flag): no staging registers, no LDS store instructions, nothing passing through the vector
// register file.  Measured on a replica of the step, register staging (4 loads + 4 LDS stores per
// wave and step) cost 28 % on top of the step without any staging; the direct loads cost nothing
// measurable.  LDS holds a K ring of four tiles and a V ring of eight, unpadded and XOR-swizzled
// per 16-byte piece.  The loads of tile j+4 go out in the second half of step j, one instruction
// per slice; the one barrier per step sits in the middle of the step and is also where each wave
// waits for its own loads of tile j+2.  The rings are deep enough that a slot is refilled only
// after every wave has passed a barrier since its last reader, so no wave waits at a step boundary
// and the LDS operands of a step's first MFMAs are fetched at the end of the step before.
#include "attention.h"


#include <math.h>
#include <type_traits>

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
constexpr int ROW_B = D * 2;            // bytes of one K or V row of one head
constexpr int TILE_B = BN * ROW_B;      // a K or V tile in LDS: 32 rows of 256 B, 16-byte pieces XOR-swizzled
// Tiles are requested AHEAD steps before their softmax; the barrier of a step lets the
// 4 * (AHEAD - 3) staging instructions of the younger tiles stay in flight.
#ifndef KVS_ATTN_SHARE_MAX_X2
#define KVS_ATTN_SHARE_MAX_X2 7      // launches run per-unit shares up to this many half-tiles per unit (7 = 3.5 tiles)
#endif
#ifndef KVS_ATTN_AHEAD
#define KVS_ATTN_AHEAD 4
#define KVS_ATTN_IN_FLIGHT 4
#endif
constexpr int AHEAD = KVS_ATTN_AHEAD;
static_assert(KVS_ATTN_IN_FLIGHT == 4 * (AHEAD - 3), "staging instructions per tile and wave: 4");
constexpr int K_RING = AHEAD <= 4 ? 4 : 8;   // tiles, >= AHEAD; see the slot argument at stage_part
constexpr int V_RING = 8;                    // >= AHEAD + 2
static_assert(K_RING >= AHEAD && V_RING >= AHEAD + 2, "ring depth");
constexpr int LDS_BYTES = (K_RING + V_RING) * TILE_B;
constexpr float kRefShift = 60.0f;      // base-2 offset of the fixed softmax reference above the first tile's maximum
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
__device__ __forceinline__ float add_rounded_pair(uint32_t w, float acc)   // acc + lo(w) + hi(w), one instruction
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, 0x3f803f80u), acc, false);
}


// An unsplit launch with shares (share_units > 0) starts one workgroup per compute unit and KV
// head; every workgroup packs the head's row tiles onto the head's units by itself, from the
// tiles' actual reach in the context, and runs its own unit's share (see plan_shares).
constexpr int kAttnShareMaxTiles = 512;
constexpr int kAttnShareMaxUnits = 64;     // one lane of a wavefront per unit
constexpr float kAttnTileOverhead = 8.0f;  // key-tile steps a tile costs before its first

// Packs the row tiles of one KV head onto `units` compute units and returns the share of unit
// `unit` (heaviest tile first) in LDS; every workgroup of the launch computes the same packing.
//
// Why: within an XCD the dispatcher deals workgroup n of a launch to shader engine n % 4 (8 compute
// units each), strictly in order: a workgroup whose engine is full holds back everything behind
// it, also workgroups whose engine has room.  With one workgroup per tile, heaviest first, and
// tile weights that grow up the context, the first two rounds pair up to equal sums on every unit
// and whatever is left lands on top: 72 tiles per head finish 11 % above the mean load of the
// head's 32 units (measured, and reproduced by a model of those rules; no list order is robustly
// better under them).  The units of an XCD run at the same pace (+-0.5 % measured), so a fixed
// share per unit loses nothing against a queue.
//
// How: weight of a tile = key tiles up to its last row's position (read from sel_pos: exact) plus
// a fixed cost; tiles ranked by weight; first fit decreasing under a capacity, one lane per unit
// (a ballot finds the first unit with room); the four waves try four capacities at a time, from
// 0.5 % above the mean load upwards, and the smallest that works is taken.
__device__ __forceinline__ void plan_shares(const AttnTiles &td, int grp, int total_tiles, const int32_t *__restrict__ sel_pos,
                                            int units, int unit, char *scratch, uint16_t *my_tiles, int *n_my_tiles)
{
    constexpr int MAXT = kAttnShareMaxTiles;
    float *w = reinterpret_cast<float *>(scratch);                       // [MAXT] weight of tile t
    float *sw = w + MAXT;                                                // [MAXT] weights in falling order
    uint16_t *st = reinterpret_cast<uint16_t *>(sw + MAXT);              // [MAXT] the tiles in that order
    uint16_t *found = st + MAXT;                                         // [NWAVES][MAXT] ranks that fall to `unit`, per trial
    int *n_found = reinterpret_cast<int *>(found + NWAVES * MAXT);       // [NWAVES], -1: the capacity did not work
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int t = tid; t < total_tiles; t += NT) {
        int b = 0;
        while (b + 1 < td.n_req && t >= td.tile_begin[b + 1]) ++b;
        const int tile = t - td.tile_begin[b];
        const int n_rows = td.n_sel[b] * grp;
        const int last_row = (tile + 1) * ROWS - ((td.tile_begin[b + 1] - td.tile_begin[b]) * ROWS - n_rows) - 1;   // tiles end-aligned
        int p = sel_pos[td.sel_lo[b] + last_row / grp];
        p = min(max(p, 0), td.ctx_len[b] - 1);
        w[t] = (float)(p / BN + 1) + kAttnTileOverhead;
    }
    __syncthreads();
    float sum = 0.f, biggest = 0.f;
    for (int t = 0; t < total_tiles; ++t) { sum += w[t]; biggest = fmaxf(biggest, w[t]); }   // same order in every thread
    for (int t = tid; t < total_tiles; t += NT) {
        const float wt = w[t];
        int rank = 0;
        for (int j = 0; j < total_tiles; ++j) rank += (w[j] > wt || (w[j] == wt && j > t)) ? 1 : 0;
        sw[rank] = wt;
        st[rank] = (uint16_t)t;
    }
    __syncthreads();
    const float mean = fmaxf(sum / (float)units, biggest);
    // the sorted weights, rank 64 k + lane in register k of the lane (read back with a lane broadcast:
    // an LDS round trip per tile would dominate the loop)
    float mine_w[MAXT / 64];
#pragma unroll
    for (int k = 0; k < MAXT / 64; ++k) mine_w[k] = 64 * k + lane < total_tiles ? sw[64 * k + lane] : 0.f;
    // first fit decreasing under `cap`: lane l is unit l, a ballot finds the first unit with room;
    // the ranks that fall to `unit` go to found[wave]
    auto pack = [&](float cap) {
        float load = lane < units ? 0.f : 3.0e38f;
        int n = 0;
        bool ok = true;
#pragma unroll
        for (int k = 0; k < MAXT / 64; ++k) {
            const int n_here = min(64, total_tiles - 64 * k);          // uniform
            for (int l = 0; l < n_here; ++l) {
                const float wt = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine_w[k]), l));
                const unsigned long long room = __ballot(load + wt <= cap);
                ok = ok && room != 0;
                const int first = room ? __ffsll((long long)room) - 1 : 0;
                if (lane == first) load += wt;
                if (first == unit) { if (lane == 0) found[wave * MAXT + n] = (uint16_t)(64 * k + l); ++n; }
            }
        }
        if (lane == 0) n_found[wave] = ok ? n : -1;
    };
    // The four waves try four capacities at once, the smallest that works is taken; the ladder goes
    // on until twice the mean load, which always works (a tile that finds no room under it would
    // mean every unit already carries more than the mean).  Tile sets that one wave of equal
    // weights spread evenly need the first round only; very uneven ones (a few tiles per unit and
    // reaches bunched together) can need 10-20 %.
    static_assert(NWAVES == 4, "one capacity per wave");
    const float ladder[3][NWAVES] = {{1.005f, 1.015f, 1.03f, 1.06f}, {1.09f, 1.13f, 1.18f, 1.25f}, {1.35f, 1.5f, 1.7f, 2.0f}};
    int pick = -1;
    for (int round = 0; round < 3 && pick < 0; ++round) {      // uniform over the workgroup
        if (round > 0) __syncthreads();                           // n_found of the round before has been read
        pack(mean * ladder[round][wave]);
        __syncthreads();
#pragma unroll
        for (int v = NWAVES - 1; v >= 0; --v) pick = n_found[v] >= 0 ? v : pick;
    }
    if (pick < 0) {
        // not reachable by the argument above; if rounding ever defeats it, deal the ranks round robin
        // (every tile still runs exactly once)
        int n = 0;
        for (int i = unit; i < total_tiles; i += units, ++n)
            if (tid == 0) my_tiles[n] = st[i];
        if (tid == 0) *n_my_tiles = n;
    } else {
        const int n = n_found[pick];
        for (int i = tid; i < n; i += NT) my_tiles[i] = st[found[pick * MAXT + i]];
        if (tid == 0) *n_my_tiles = n;
    }
    __syncthreads();
}

// WANT_LSE: additionally keep the unrounded sum of weights, from which the log-sum-exp is reported.
// SPLIT: the key range is cut into pieces handled by different workgroups (launches with few row
// tiles over long contexts would otherwise leave most of the chip idle); at most n_splits slots
// per row tile, the sizes and the order of the pieces come from what attn_plan_kernel leaves in
// device memory.  Every piece writes its unnormalised accumulators and (reference, sums) to the
// workspace and the merge kernel combines them.  The pieces are absolute key ranges, the same for
// every row tile, and the list runs through them range by range: the workgroups that are resident
// together read the same stretch of K and V, which then stays in L2.
template <bool WANT_LSE, bool SPLIT>
__global__ __launch_bounds__(NT, 1) void attn_mfma2_kernel(
    const AttnTiles td, int n_q_heads, int n_kv_heads, int total_tiles,
    const uint16_t *__restrict__ q_sel, const int32_t *__restrict__ sel_pos,
    const uint16_t *__restrict__ k_cache, const uint16_t *__restrict__ v_cache,
    float scale_log2, uint16_t *__restrict__ out, float *__restrict__ lse_out,
    int n_splits, const int4 *__restrict__ split_plan, const uint16_t *__restrict__ piece_list,
    float *__restrict__ part_o, float4 *__restrict__ part_ml, int share_units)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];   // K ring, then V^T ring
    __shared__ int wg_max_pos[NWAVES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, ln = lane & 31;
    // ---- which (request, kv head, row tile) -----------------------------------------------------
    const int g = blockIdx.x % n_kv_heads;
    const int wg = (int)(blockIdx.x / n_kv_heads);
    // With shares the workgroup is one compute unit's part of KV head g and works through its
    // tiles; otherwise it has the one tile (or piece) its index names.
    const bool listed = !SPLIT && share_units > 0;
    __shared__ uint16_t my_tiles[kAttnShareMaxTiles];
    __shared__ int n_my_tiles;
    if (listed) plan_shares(td, n_q_heads / n_kv_heads, total_tiles, sel_pos, share_units, wg,
                            reinterpret_cast<char *>(lds), my_tiles, &n_my_tiles);
    const int it_begin = listed ? 0 : wg, it_end = listed ? n_my_tiles : wg + 1;
    for (int it = it_begin; it < it_end; ++it) {
    if (it != it_begin) __syncthreads();   // every wave has left the previous tile: rings and tables are free
    const int rest = it;
    // split launches walk the list of pieces the plan kernel wrote: the pieces that have keys first,
    // from the top of the context down, then the empty ones (which only mark their slot)
    const int piece = SPLIT ? piece_list[rest] : rest;
    const int split = SPLIT ? piece / total_tiles : 0;
    const int tile_lin = SPLIT ? total_tiles - 1 - piece % total_tiles
                               : (listed ? (int)my_tiles[rest] : total_tiles - 1 - rest);
    int b = 0;
    while (b + 1 < td.n_req && tile_lin >= td.tile_begin[b + 1]) ++b;
    const int tile = tile_lin - td.tile_begin[b];
    const int grp = n_q_heads / n_kv_heads;
    const int64_t sel0 = td.sel_lo[b];
    const int n_rows = td.n_sel[b] * grp;
    // Row tiles are aligned to the end of the request's rows: the one partly filled tile is then the
    // first, whose rows sit lowest in the context and see the fewest keys, so the padding lanes of
    // the launch idle through the shortest sweep instead of the longest.
    const int row0 = tile * ROWS - ((td.tile_begin[b + 1] - td.tile_begin[b]) * ROWS - n_rows);
    const int ctx_len = td.ctx_len[b];
    const int64_t ctx_off = td.ctx_off[b];

    // the plan: (pieces per row tile in use, key tiles per large piece, per small piece, small pieces)
    int4 plan = make_int4(1, 0, 0, 0);
    if (SPLIT) {
        plan = *split_plan;
        if (split >= plan.x) {   // a piece slot the plan does not use: mark it empty for the merge
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int rq = row0 + wave * WROWS + nb * 32 + ln;
                const int t_sel = rq / grp, hh = rq - t_sel * grp;
                if (rq >= 0 && hf == 0)
                    part_ml[((sel0 + t_sel) * n_q_heads + g * grp + hh) * (int64_t)n_splits + split] = make_float4(-1.0e30f, 0.f, 0.f, 0.f);
            }
            return;
        }
    }

    // this lane's query rows, one per 32-row block (both half-waves hold the same queries)
    bool row_ok[NB];
    int pos[NB];
    int64_t row_idx[NB];
    int pmin = 0x7fffffff, pmax = 0;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int rq = row0 + wave * WROWS + nb * 32 + ln;
        row_ok[nb] = rq >= 0;
        const int rqc = max(rq, 0);
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
    // this workgroup's share of the key tiles: [t_lo, t_hi)
    int t_lo = 0, t_hi = n_kv_tiles;
    if (SPLIT) {
        // piece 0 is the top of the context; counted from the bottom, the first plan.w pieces are
        // plan.z key tiles long and the others plan.y
        const int j = plan.x - 1 - split;
        const int lo = j < plan.w ? j * plan.z : plan.w * plan.z + (j - plan.w) * plan.y;
        t_lo = min(n_kv_tiles, lo);
        t_hi = min(n_kv_tiles, lo + (j < plan.w ? plan.z : plan.y));
    }
    if (SPLIT && t_lo >= t_hi) {   // nothing of this tile in this key range: mark the piece empty
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
            if (row_ok[nb] && hf == 0) part_ml[row_idx[nb] * (int64_t)n_splits + split] = make_float4(-1.0e30f, 0.f, 0.f, 0.f);
        return;
    }

    // ---- global -> LDS staging of one K/V tile ---------------------------------------------------------
    // Buffer loads that write straight into LDS: no registers, no LDS store instructions, and the
    // data does not pass through the vector register file.  One instruction moves 64 x 16 bytes to
    // 1 KiB of consecutive LDS (lane l -> bytes 16 l), i.e. four 256-byte rows; a wave stages rows
    // 4w .. 4w+3 of each half of the tile, K and V, four instructions per tile.  A tile in LDS is 32
    // rows of 256 B without padding; the 16-byte piece p of row r sits at position p ^ f(r), which
    // the load realises by letting lane (row, position) fetch piece position ^ f(row).  f is chosen
    // per tile kind so that the operand reads below are free of bank conflicts:
    //   K: f(r) = r & 15           (8 lanes read 8 different rows at the same piece index),
    //   V: f(r) = 2 (r & 7)        (a transposing read covers 4 consecutive rows x 2 pieces).
    // Every address is kept inside the request's rows by construction (tiles wholly inside the
    // context, or per-row clamping); the buffer's record count is a second guard only.
    const uint32_t row_bytes = (uint32_t)n_kv_heads * D * 2u;          // bytes between tokens
    const uint32_t head_bytes = ((uint32_t)ctx_len - 1u) * row_bytes + D * 2u;   // this head's span of the request
    // buffer resource: base address, 48 bits; stride 0; size in bytes; dword 3 as for untyped access
    auto make_rsrc = [&](const uint16_t *base) -> u32x4_t {
        const uint64_t a = reinterpret_cast<uint64_t>(base);
        u32x4_t r = {(uint32_t)a, (uint32_t)(a >> 32) & 0xffffu, head_bytes, 0x00020000u};
        r.x = __builtin_amdgcn_readfirstlane(r.x);
        r.y = __builtin_amdgcn_readfirstlane(r.y);
        r.z = __builtin_amdgcn_readfirstlane(r.z);
        return r;
    };
    const u32x4_t krs = make_rsrc(k_cache + (ctx_off * n_kv_heads + g) * (int64_t)D);
    const u32x4_t vrs = make_rsrc(v_cache + (ctx_off * n_kv_heads + g) * (int64_t)D);
    char *const lds_b = reinterpret_cast<char *>(lds);
    // byte offset of the dynamic LDS array inside the workgroup's allocation (what M0 has to carry)
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds_b);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int st_row = 4 * wave_u + (lane >> 4);       // row inside a 16-row half of the tile, 0..15
    const int st_pos = lane & 15;                      // piece position inside the row
    const uint32_t st_k_piece = (uint32_t)(st_pos ^ st_row) * 16u;
    const uint32_t st_v_piece = (uint32_t)(st_pos ^ (2 * (st_row & 7))) * 16u;
    const uint32_t st_k_voff = (uint32_t)(lane >> 4) * row_bytes + st_k_piece;
    const uint32_t st_v_voff = (uint32_t)(lane >> 4) * row_bytes + st_v_piece;
    // Slots.  Tile t goes to K slot t % K_RING and V slot t % V_RING.  stage_part(t, .) is issued in
    // the second half of step t-AHEAD, after that step's barrier.  The K slot held tile t-K_RING, last
    // read in step t-K_RING-1, the V slot tile t-V_RING, last read in step t-V_RING+1 (the general
    // loop: t-V_RING): with K_RING >= AHEAD and V_RING >= AHEAD+2 every wave has passed a barrier
    // since.  The tile must have landed by the barrier of step t-2 (its K is first read at the end of
    // step t-2): each wave waits for its own parts there, allowing only the instructions of tiles
    // t+1 .. t+AHEAD-3 to be still in flight.
    // The instruction is written out by hand: issued through the compiler's builtin it makes the
    // compiler wait for all outstanding loads before every later LDS read it cannot prove disjoint,
    // which would serialise the sweep on global-memory latency.  Here the waiting is done once per
    // step, at the barrier (KVS_ATTN_BARRIER).  M0 holds the LDS destination of lane 0; the nop covers
    // the wait state an M0 write needs before such a load.
    auto stage_1k = [&](const u32x4_t &rs, uint32_t lds_dst, uint32_t voff, uint32_t soff) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                     :: "s"(lds_dst), "v"(voff), "s"(rs), "s"(soff));
    };
    auto stage_part = [&](int t, int part) {           // part 0,1: K rows 0-15 / 16-31; 2,3: V likewise
        const int q = part & 1;
        const uint32_t soff = __builtin_amdgcn_readfirstlane(((uint32_t)t * BN + (uint32_t)(16 * q + 4 * wave_u)) * row_bytes);
        const uint32_t dst = lds_base + (uint32_t)(16 * q + 4 * wave_u) * ROW_B;
        if (part < 2)
            stage_1k(krs, __builtin_amdgcn_readfirstlane(dst + (uint32_t)((t & (K_RING - 1)) * TILE_B)), st_k_voff, soff);
        else
            stage_1k(vrs, __builtin_amdgcn_readfirstlane(dst + (uint32_t)((K_RING + (t & (V_RING - 1))) * TILE_B)), st_v_voff, soff);
    };
    auto stage_tile_inside = [&](int t) {              // tile wholly inside the context
#pragma unroll
        for (int part = 0; part < 4; ++part) stage_part(t, part);
    };
    auto stage_tile = [&](int t) {                     // any tile: rows past the context are clamped
        if ((t + 1) * BN <= ctx_len) {
            stage_tile_inside(t);
        } else {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int key = min(t * BN + 16 * q + st_row, ctx_len - 1);
                const uint32_t dst = lds_base + (uint32_t)(16 * q + 4 * wave_u) * ROW_B;
                stage_1k(krs, __builtin_amdgcn_readfirstlane(dst + (uint32_t)((t & (K_RING - 1)) * TILE_B)),
                         (uint32_t)key * row_bytes + st_k_piece, 0u);
                stage_1k(vrs, __builtin_amdgcn_readfirstlane(dst + (uint32_t)((K_RING + (t & (V_RING - 1))) * TILE_B)),
                         (uint32_t)key * row_bytes + st_v_piece, 0u);
            }
        }
    };
    // Barriers of the sweep.  The staged data arrives asynchronously (the vector-memory counter
    // tracks it, oldest first); nothing else of the workgroup's LDS traffic needs ordering here: a
    // slot is only overwritten long after its last reader (above).  `in_flight` = staging
    // instructions of younger tiles that may still be outstanding.
#define KVS_ATTN_BARRIER_(in_flight) asm volatile("s_waitcnt vmcnt(" #in_flight ")\n\ts_barrier" ::: "memory")
#define KVS_ATTN_BARRIER(in_flight) KVS_ATTN_BARRIER_(in_flight)

    // ---- the three pieces of one tile's work ----------------------------------------------------------
    // K row fed to MFMA row ln: bits 2 and 3 swapped, so that accumulator entry r of a lane is key
    // 16*(r>>3) + 8*hf + (r&7) of the tile.  The lane reads piece 2*ks + hf of that row, which sits
    // at position (2*ks + hf) ^ (row & 15): byte offset = lane constant ^ 32*ks.
    const int krow = (ln & ~12) | ((ln & 4) << 1) | ((ln & 8) >> 1);
    const uint32_t k_read_off = (uint32_t)(krow * ROW_B + ((hf ^ (krow & 15)) * 16));
    // V stays row-major [key][channel] in LDS; the A operand of the PV product (channel = MFMA row,
    // 8 consecutive keys per lane) comes out of two transposing LDS reads.  In each group of 16
    // lanes, lane s points at 8 bytes (4 channels) and lane i receives, as element j, element i%4 of
    // the lane i/4 + 4j: with lane s on key k0 + s/4, channels d0 + 4*(s%4) .. +3, lane i ends up
    // with channel d0 + i of keys k0 .. k0+3.  Groups 0/1 are channels 0-15 / 16-31 of the block,
    // groups 2/3 the same for the half-wave's second set of 8 keys.  The 8 bytes are half (s & 1) of
    // piece 4*db + 2*(group & 1) + (s % 4) / 2 of their row: byte offset = lane constant ^ 64*db.
    const int tr_s = lane & 15, tr_g = lane >> 4;
    const int tr_key = 8 * (tr_g >> 1) + (tr_s >> 2);                  // keys 0-3 of the lane's 8; +4 for keys 4-7
    const int tr_c = 2 * (tr_g & 1) + ((tr_s & 3) >> 1);
    const uint32_t v_read_lo = (uint32_t)(tr_key * ROW_B + ((tr_c ^ (2 * (tr_key & 7))) * 16) + 8 * (tr_s & 1));
    const uint32_t v_read_hi = (uint32_t)((tr_key + 4) * ROW_B + ((tr_c ^ (2 * ((tr_key + 4) & 7))) * 16) + 8 * (tr_s & 1));
    auto read_k = [&](uint32_t slot_off, int ks) -> u32x4_t {          // slot_off: byte offset of the K tile in LDS
        return *reinterpret_cast<const u32x4_t *>(lds_b + ((k_read_off ^ (uint32_t)(32 * ks)) + slot_off));
    };
    auto read_vt = [&](uint32_t slot_off, int kstep, int db) -> u32x4_t {
        typedef short v4i16 __attribute__((ext_vector_type(4)));
        typedef __attribute__((address_space(3))) v4i16 lds_v4i16;
        const uint32_t base = slot_off + (uint32_t)(16 * kstep * ROW_B);
        const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16 *)(lds_b + ((v_read_lo ^ (uint32_t)(64 * db)) + base)));
        const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16 *)(lds_b + ((v_read_hi ^ (uint32_t)(64 * db)) + base)));
        const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
        u32x4_t r = {l2.x, l2.y, h2.x, h2.y};
        return r;
    };
    auto k_slot = [&](int t) -> uint32_t { return (uint32_t)((t & (K_RING - 1)) * TILE_B); };
    auto v_slot = [&](int t) -> uint32_t { return (uint32_t)((K_RING + (t & (V_RING - 1))) * TILE_B); };
    const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    auto qk = [&](int jt, floatx16 (&s)[NB]) {
        const uint32_t ks = k_slot(jt);
#pragma unroll
        for (int ksx = 0; ksx < D / 16; ++ksx) {
            const u32x4_t a = read_k(ks, ksx);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), qreg[nb][ksx], ksx == 0 ? zero : s[nb], 0, 0, 0);
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
    // Four scores r0..r0+3 of query block nb -> two packed bf16 pairs of the P operand, and their
    // contribution to the running sums.  P = exp2(scale*log2e*S - m_ref); the reference is fixed for
    // the whole pass, so the output accumulators are touched by MFMAs only and can stay in the
    // accumulation registers; see the comment at the pass loop for why that is safe.
    auto softmax4 = [&](const floatx16 &s, int nb, int r0, u32x4_t (&pop)[2]) {
        const float e0 = __builtin_amdgcn_exp2f(fmaf(s[r0 + 0], scale_log2, -m_ref[nb]));
        const float e1 = __builtin_amdgcn_exp2f(fmaf(s[r0 + 1], scale_log2, -m_ref[nb]));
        const float e2 = __builtin_amdgcn_exp2f(fmaf(s[r0 + 2], scale_log2, -m_ref[nb]));
        const float e3 = __builtin_amdgcn_exp2f(fmaf(s[r0 + 3], scale_log2, -m_ref[nb]));
        const uint32_t w0 = pack2(e0, e1), w1 = pack2(e2, e3);
        pop[r0 >> 3][(r0 & 7) >> 1] = w0;
        pop[r0 >> 3][((r0 & 7) >> 1) + 1] = w1;
        l_run[nb] = add_rounded_pair(w1, add_rounded_pair(w0, l_run[nb]));
        if (WANT_LSE) l_exact[nb] += (e0 + e1) + (e2 + e3);
    };
    auto softmax = [&](int jt, floatx16 (&s)[NB], u32x4_t (&pop)[NB][2]) {
        mask_tile(jt, s);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r0 = 0; r0 < 16; r0 += 4) softmax4(s[nb], nb, r0, pop[nb]);
    };
    auto pv_product = [&](int jt, const u32x4_t (&pop)[NB][2]) {
        const uint32_t vs = v_slot(jt);
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                const u32x4_t va = read_vt(vs, a, db);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    o_acc[db][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va), as_bf16x8(pop[nb][a]), o_acc[db][nb], 0, 0, 0);
            }
    };

    // One step of the pipelined sweep (tile jt+AHEAD lies wholly inside the context; `masked` says whether
    // tile jt needs the causal compare for this wave): scores of tile jt+1, softmax of tile jt, PV of
    // tile jt-1, written as eight slices of four MFMAs and four scores each, LDS operands fetched one
    // slice ahead (ka / va enter with slice 0's operands and leave with those of the next step).
    // On entry tiles jt-1 .. jt+1 are in the LDS rings and tiles jt+2 .. jt+AHEAD-1 on their way, s_in holds
    // the scores of tile jt and p_in the weights of tile jt-1.  The barrier in mid-step makes tile
    // jt+2 visible; the second half sends out the loads of tile jt+AHEAD, one instruction per slice.
    int key_lim[NB];   // a key of the tile is visible to the lane's query nb iff its (half-wave-relative) index <= this
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) key_lim[nb] = pos[nb] - 8 * hf;
    auto fast_step = [&](auto masked, int jt, const floatx16 (&s_in)[NB], floatx16 (&s_out)[NB],
                         const u32x4_t (&p_in)[NB][2], u32x4_t (&p_out)[NB][2],
                         u32x4_t &ka, u32x4_t &va) {
        constexpr bool MASKED = decltype(masked)::value;
        const uint32_t ks = k_slot(jt + 1), vs = v_slot(jt - 1), ks_next = k_slot(jt + 2), vs_next = v_slot(jt);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // source order of the slice: next slice's LDS operands, then one MFMA at a time, each
            // followed by vector work that can run beside it.  The compiler's scheduler is left free
            // to reorder within the step: pinning this order with scheduling barriers measured 4-6 %
            // slower than its own choice.
            u32x4_t ka_n, va_n;
            if (i < 7) {
                ka_n = read_k(ks, i + 1);
                va_n = read_vt(vs, (i + 1) >> 2, (i + 1) & 3);
            } else {
                ka_n = read_k(ks_next, 0);
                va_n = read_vt(vs_next, 0, 0);
            }
            const int nbs = i >> 2, r0 = 4 * (i & 3), a = i >> 2, db = i & 3;
            s_out[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ka), qreg[0][i], i == 0 ? zero : s_out[0], 0, 0, 0);
            float x0 = fmaf(s_in[nbs][r0 + 0], scale_log2, -m_ref[nbs]);
            float x1 = fmaf(s_in[nbs][r0 + 1], scale_log2, -m_ref[nbs]);
            float x2 = fmaf(s_in[nbs][r0 + 2], scale_log2, -m_ref[nbs]);
            float x3 = fmaf(s_in[nbs][r0 + 3], scale_log2, -m_ref[nbs]);
            if (MASKED) {   // entry r of the lane is key jt*BN + 16*(r>>3) + 8*hf + (r&7)
                const int k0 = jt * BN + 16 * (r0 >> 3) + (r0 & 7);
                x0 = k0 + 0 > key_lim[nbs] ? -INFINITY : x0;
                x1 = k0 + 1 > key_lim[nbs] ? -INFINITY : x1;
                x2 = k0 + 2 > key_lim[nbs] ? -INFINITY : x2;
                x3 = k0 + 3 > key_lim[nbs] ? -INFINITY : x3;
            }
            s_out[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ka), qreg[1][i], i == 0 ? zero : s_out[1], 0, 0, 0);
            const float e0 = __builtin_amdgcn_exp2f(x0);
            const float e1 = __builtin_amdgcn_exp2f(x1);
            const float e2 = __builtin_amdgcn_exp2f(x2);
            const float e3 = __builtin_amdgcn_exp2f(x3);
            o_acc[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va), as_bf16x8(p_in[0][a]), o_acc[db][0], 0, 0, 0);
            const uint32_t w0 = pack2(e0, e1), w1 = pack2(e2, e3);
            p_out[nbs][r0 >> 3][(r0 & 7) >> 1] = w0;
            p_out[nbs][r0 >> 3][((r0 & 7) >> 1) + 1] = w1;
            l_run[nbs] = add_rounded_pair(w1, add_rounded_pair(w0, l_run[nbs]));
            if (WANT_LSE) l_exact[nbs] += (e0 + e1) + (e2 + e3);
            o_acc[db][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va), as_bf16x8(p_in[1][a]), o_acc[db][1], 0, 0, 0);
            ka = ka_n;
            va = va_n;
            if (i == 3) KVS_ATTN_BARRIER(KVS_ATTN_IN_FLIGHT);   // tile jt+2 has landed; younger ones may be in flight
            if (i >= 4) stage_part(jt + AHEAD, i - 4);
        }
    };

    // ---- passes -------------------------------------------------------------------------------------------
    // Pass 0 takes each row's exponent reference from its first tile (every row sees key 0) and
    // never moves it: softmax(x) is invariant to the reference as long as nothing overflows or
    // underflows.  The reference is the first tile's largest logit plus kRefShift (in base-2 units),
    // so weights are computed around 2^-60 instead of around 1: fp32 and bf16 share an 8-bit exponent,
    // nothing loses precision down there, and the sum only passes 2^100 if a later logit lies more
    // than 160 (111 in natural units) above the first tile's maximum, while a key has to be 2^-66
    // of the row's largest weight before it is flushed to zero.  (Unshifted, a logit ~2^6 above
    // the first tile's maximum already overflowed, which heavy-tailed keys do reach: half the
    // workgroups of a 131k-token launch repeated the pass.)  If a row's sum does end above 2^100 (or
    // inf / nan) the workgroup computes the exact row maxima in a score-only sweep and repeats the
    // pass with those (pass 1), which cannot overflow: a correctness net.
    __shared__ int redo_flag;
    float l_tot[NB];
    for (int pass = 0; pass < 2; ++pass) {
        if (pass == 1) {
            // exact row maxima: a score-only sweep with three tiles on their way.  Tile jt+3 goes to
            // the K slot of tile jt-1, which every wave has finished reading when it passes the
            // barrier of step jt; tiles past the end are requested too (rows clamped, never
            // read), so the count of younger loads in flight at a barrier is always two tiles' worth.
            static_assert(K_RING >= 4, "the score-only sweep keeps three tiles in flight beside the one in use");
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) m_ref[nb] = -INFINITY;
            for (int k = 0; k < 3; ++k) stage_tile(t_lo + k);
            for (int jt = t_lo; jt < t_hi; ++jt) {
                KVS_ATTN_BARRIER(8);
                stage_tile(jt + 3);
                floatx16 s[NB];
                qk(jt, s);
                mask_tile(jt, s);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) m_ref[nb] = fmaxf(m_ref[nb], row_max(s[nb]));
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();   // every wave is done with the ring before the sweep refills it
        }
        // Invariant at the top of step j, in either loop: the loads of tiles j .. j+AHEAD-1 have been sent
        // (where those tiles exist; the pipelined loop also sends tiles past the piece, which nothing
        // reads), tiles j and j+1 are visible to every wave, and the barrier of step j makes tile j+2
        // visible.  The loads of tile j+AHEAD go out after that barrier.
#pragma unroll
        for (int k = 0; k < AHEAD; ++k)
            if (t_lo + k < t_hi) stage_tile(t_lo + k);
        KVS_ATTN_BARRIER(0);
        floatx16 s_cur[NB], s_nxt[NB];
        qk(t_lo, s_cur);
        if (pass == 0) {
            mask_tile(t_lo, s_cur);
            // a row whose keys all lie before this piece sees nothing here: a finite reference keeps
            // its weights at exp2(-inf) = 0 instead of NaN (the merge drops pieces with zero sum)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) m_ref[nb] = fmaxf(row_max(s_cur[nb]), -1.0e30f) + kRefShift;
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) { l_run[nb] = 0.f; l_exact[nb] = 0.f; }
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) o_acc[db][nb] = zero;

        int jt = t_lo;
        // Pipelined sweep over the tiles whose look-ahead tiles lie wholly inside the context.  Each
        // wave leaves it at its own point and finishes in the general loop below: both send the same
        // tile's loads in the same step and hit one barrier per step, so the waves of a workgroup
        // may sit in different loops.
        const int j_unmasked = (pmin + 1) / BN;     // tiles 0 .. j_unmasked-1: every key <= pmin
        const int j_inside = ctx_len / BN;          // tiles 0 .. j_inside-1 need no row clamp
        if (t_lo + 3 <= t_hi && t_lo + AHEAD + 3 <= j_inside) {
            // the first step has no earlier tile to multiply: scores of the second tile, softmax of the first
            u32x4_t p_a[NB][2], p_b[NB][2];
            qk(t_lo + 1, s_nxt);
            softmax(t_lo, s_cur, p_a);
            KVS_ATTN_BARRIER(KVS_ATTN_IN_FLIGHT);
            stage_tile_inside(t_lo + AHEAD);
            // K of the third tile, V of the first
            u32x4_t ka = read_k(k_slot(t_lo + 2), 0);
            u32x4_t va = read_vt(v_slot(t_lo), 0, 0);
            // two steps per trip so that the score and weight buffers swap roles without copies
            for (jt = t_lo + 1; jt + 1 < min(j_unmasked, t_hi) && jt + AHEAD + 1 < j_inside; jt += 2) {
                fast_step(std::false_type{}, jt, s_nxt, s_cur, p_a, p_b, ka, va);
                fast_step(std::false_type{}, jt + 1, s_cur, s_nxt, p_b, p_a, ka, va);
            }
            // the tiles around the wave's own positions, same pipeline with the causal compare
            for (; jt + 1 < t_hi && jt + AHEAD + 1 < j_inside; jt += 2) {
                fast_step(std::true_type{}, jt, s_nxt, s_cur, p_a, p_b, ka, va);
                fast_step(std::true_type{}, jt + 1, s_cur, s_nxt, p_b, p_a, ka, va);
            }
            pv_product(jt - 1, p_a);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) s_cur[nb] = s_nxt[nb];
        }
        // general loop; s_cur = scores of tile jt
        for (; jt < t_hi; ++jt) {
            // scores of the next tile first (past the last tile the slot holds stale data and the
            // result is discarded)
            qk(jt + 1, s_nxt);
            u32x4_t pop[NB][2];
            softmax(jt, s_cur, pop);
            pv_product(jt, pop);
            KVS_ATTN_BARRIER(0);
            if (jt + AHEAD < t_hi) stage_tile(jt + AHEAD);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) s_cur[nb] = s_nxt[nb];
        }
        // nothing may still be on its way into LDS when the rings are reused or the workgroup ends
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

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
        if (SPLIT) {
            if (row_ok[nb]) {
                const int64_t slot = row_idx[nb] * (int64_t)n_splits + split;
                float *prow = part_o + slot * D;
#pragma unroll
                for (int db = 0; db < D / 32; ++db)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const int d0 = 32 * db + 8 * r4 + 4 * hf;
                        *reinterpret_cast<float4 *>(prow + d0) = make_float4(o_acc[db][nb][4 * r4 + 0], o_acc[db][nb][4 * r4 + 1],
                                                                             o_acc[db][nb][4 * r4 + 2], o_acc[db][nb][4 * r4 + 3]);
                    }
                if (hf == 0) part_ml[slot] = make_float4(m_ref[nb], l_tot[nb], WANT_LSE ? l_exact_tot : l_tot[nb], 0.f);
            }
            continue;
        }
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
    }   // tiles of this workgroup
}

} // namespace

namespace {

// Plans a split launch on the device, where the positions are: the size of the large pieces and
// the order in which the workgroups take the pieces.
//
// Size.  The large pieces run in rounds of one per compute unit, each round as long as the chunk,
// and a piece costs about piece_overhead key tiles on top of its own: so for 1, 2, ... rounds the
// best chunk is the smallest one whose pieces just fit, and the round count with the shortest
// predicted time wins (fewer, longer rounds win ties through the overhead).  round_fill < 1 leaves
// head-room.  Thread i tries chunk c_min + i * step over the lengths of all row tiles (taken from
// each tile's last row, i.e. exact for positions in ascending order; any other order costs speed
// only: the attention kernel finds its own key range).
//
// Order.  piece id = split * total_tiles + (row tiles from the last one down).  A workgroup that
// finds its piece empty still holds a compute unit for a few microseconds, and the dispatcher
// hands out workgroups strictly in order, so empty pieces in between starve the pieces behind
// them: the list names the pieces with keys first and all empty slots after them.
constexpr int PLAN_NT = 256;
constexpr int PLAN_MAX_TILES = kAttnPlanMaxTiles;
constexpr int PLAN_MAX_ROUNDS = 4;
__global__ __launch_bounds__(PLAN_NT) void attn_plan_kernel(
    const AttnTiles td, int grp, int n_kv_heads, int total_tiles, const int32_t *__restrict__ sel_pos,
    int s_max, int ctx_tiles, int small_chunk, int n_small, float round_fill, float piece_overhead,
    int forced_chunk, int4 *__restrict__ plan, uint16_t *__restrict__ piece_list)
{
    __shared__ int len[PLAN_MAX_TILES];       // key tiles of each row tile
    __shared__ int first_fit[PLAN_MAX_ROUNDS];
    __shared__ int4 chosen;
    __shared__ int wave_total[PLAN_NT / 64];
    const int tid = threadIdx.x;
    const int bottom = n_small * small_chunk;
    for (int t = tid; t < total_tiles; t += PLAN_NT) {
        int b = 0;
        while (b + 1 < td.n_req && t >= td.tile_begin[b + 1]) ++b;
        const int tile = t - td.tile_begin[b];
        const int n_rows = td.n_sel[b] * grp;
        const int last_row = (tile + 1) * ROWS - ((td.tile_begin[b + 1] - td.tile_begin[b]) * ROWS - n_rows) - 1;   // tiles end-aligned
        int p = sel_pos[td.sel_lo[b] + last_row / grp];
        p = min(max(p, 0), td.ctx_len[b] - 1);
        len[t] = p / BN + 1;
    }
    if (tid < PLAN_MAX_ROUNDS) first_fit[tid] = 0x7fffffff;
    __syncthreads();
    const int c_min = max(1, (ctx_tiles - bottom + (s_max - n_small) - 1) / (s_max - n_small));
    const int c_max = max(c_min, ctx_tiles - bottom);
    const int step = (c_max - c_min + PLAN_NT - 1) / PLAN_NT;
    const int c = c_min + tid * step;
    const bool tries = forced_chunk <= 0 && c <= c_max && (step > 0 || tid == 0);   // a fixed chunk needs no search
    int pieces = 0x7fffffff;
    if (tries) {
        const float rc = 1.0f / (float)c;
        pieces = 0;
        for (int t = 0; t < total_tiles; ++t) pieces += (int)ceilf((float)max(0, len[t] - bottom) * rc - 1.0e-4f);
        pieces *= n_kv_heads;
    }
    // the piece count falls as the chunk grows, so per round count the first thread that fits is
    // the answer: one LDS atomic per wave instead of one per thread
    for (int r = 0; r < PLAN_MAX_ROUNDS; ++r) {
        const bool fits = tries && (float)pieces <= round_fill * (float)(kAttnSplitCus * (r + 1));
        const unsigned long long m = __ballot(fits);
        if (m != 0 && (tid & 63) == __ffsll((long long)m) - 1) atomicMin(&first_fit[r], c);
    }
    __syncthreads();
    if (tid == 0) {
        int best_c = c_max;                 // one large piece per row tile always "fits"
        float best_t = 3.0e38f;
        for (int r = 0; r < PLAN_MAX_ROUNDS; ++r) {
            if (first_fit[r] == 0x7fffffff) continue;
            const float time = (float)(r + 1) * ((float)first_fit[r] + piece_overhead);
            if (time < best_t) { best_t = time; best_c = first_fit[r]; }
        }
        if (forced_chunk > 0) best_c = min(max(forced_chunk, c_min), c_max);
        chosen = make_int4(n_small + (ctx_tiles - bottom + best_c - 1) / best_c, best_c, small_chunk, n_small);
        *plan = chosen;
    }
    __syncthreads();
    // the list: a stable partition of the piece ids into those with keys and the rest
    const int4 pl = chosen;
    const int n_ids = s_max * total_tiles;
    const int per = (n_ids + PLAN_NT - 1) / PLAN_NT;
    const int e0 = min(n_ids, tid * per), e1 = min(n_ids, e0 + per);
    auto has_keys = [&](int e) {
        const int split = e / total_tiles, tile_lin = total_tiles - 1 - e % total_tiles;
        if (split >= pl.x) return false;
        const int j = pl.x - 1 - split;
        const int lo = j < pl.w ? j * pl.z : pl.w * pl.z + (j - pl.w) * pl.y;
        return len[tile_lin] > lo;
    };
    int mine = 0;
    for (int e = e0; e < e1; ++e) mine += has_keys(e) ? 1 : 0;
    // exclusive prefix sum over the threads: within each wave by shuffles, across the waves through LDS
    const int lane = tid & 63, wave = tid >> 6;
    int incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o);
        if (lane >= o) incl += v;
    }
    if (lane == 63) wave_total[wave] = incl;
    __syncthreads();
    int before = incl - mine, total = 0;
#pragma unroll
    for (int w = 0; w < PLAN_NT / 64; ++w) {
        before += w < wave ? wave_total[w] : 0;
        total += wave_total[w];
    }
    int full = before, empty = total + (e0 - before);
    for (int e = e0; e < e1; ++e) {
        if (has_keys(e)) piece_list[full++] = (uint16_t)e;
        else piece_list[empty++] = (uint16_t)e;
    }
}

template <bool WANT_LSE, bool SPLIT>
kvs_status launch_one(const dim3 grid, size_t lds_bytes, hipStream_t st, const AttnTiles &td, const kvs_shape *shape,
                      int tiles, const void *q_sel, const int32_t *sel_pos, const void *k_cache, const void *v_cache,
                      float scale_log2, void *out, float *lse_out, int n_splits, const int4 *split_plan,
                      const uint16_t *piece_list, float *part_o, float4 *part_ml, int share_units)
{
    static DeviceOnce attr_once;
    const kvs_status ast = once_per_device(attr_once, [lds_bytes] {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_mfma2_kernel<WANT_LSE, SPLIT>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        return e == hipSuccess ? KVS_OK : fail(KVS_EHIP, "kvs_partial_attention: hipFuncSetAttribute: %s", hipGetErrorString(e));
    });
    if (ast != KVS_OK) return ast;
    hipLaunchKernelGGL((attn_mfma2_kernel<WANT_LSE, SPLIT>), grid, dim3(NT), lds_bytes, st, td, shape->n_q_heads,
                       shape->n_kv_heads, tiles, (const uint16_t *)q_sel, sel_pos, (const uint16_t *)k_cache,
                       (const uint16_t *)v_cache, scale_log2, (uint16_t *)out, lse_out, n_splits, split_plan, piece_list,
                       part_o, part_ml, share_units);
    return check_launch("kvs_partial_attention(mfma2)");
}

// units per KV head for a launch that runs shares (0: one workgroup per tile).  Few tiles per unit
// is where the dispatcher does badly; from ~3.5 per unit on its one-by-one hand-out evens out as
// well as fixed shares do (3 % above the mean load at 4.5 per unit).
int share_units_for(const kvs_shape *shape, int64_t tiles)
{
#ifdef KVS_ATTN_NO_ORDER
    return 0;
#endif
    // one workgroup per compute unit only works out if the device has the units the shares are made for
    static std::atomic<int> cus_of[kMaxDevices];   // 0: not asked yet; the query is idempotent
    const int dev = current_device();
    if (dev < 0 || dev >= kMaxDevices) return 0;
    int device_cus = cus_of[dev].load(std::memory_order_relaxed);
    if (device_cus == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = -1;
        cus_of[dev].store(n, std::memory_order_relaxed);
        device_cus = n;
    }
    if (device_cus != kAttnSplitCus) return 0;
    const int units = kAttnSplitCus / shape->n_kv_heads;
    if (units < 1 || units > kAttnShareMaxUnits || tiles > kAttnShareMaxTiles) return 0;
    if (tiles <= units || 2 * tiles > KVS_ATTN_SHARE_MAX_X2 * units) return 0;
    return units;
}
} // namespace

AttnSplitPlan attention_mfma2_plan(const kvs_shape *shape, const AttnBatch &bd, size_t workspace_bytes)
{
    const AttnSplitPlan whole = {1, 0, 0, 0, 0};
    const int grp = shape->n_q_heads / shape->n_kv_heads;
    int64_t tiles = 0, max_ctx = 0, kv_bytes = 0;
    for (int i = 0; i < bd.n_req; ++i) {
        tiles += ((bd.cu_sel[i + 1] - bd.cu_sel[i]) * grp + ROWS - 1) / ROWS;
        max_ctx = bd.ctx_len[i] > max_ctx ? bd.ctx_len[i] : max_ctx;
        // (what has to stay cached is one request's K and V: requests do not share keys)
        if (bd.cu_sel[i + 1] > bd.cu_sel[i]) {
            const int64_t b = bd.ctx_len[i] * (int64_t)shape->n_kv_heads * ROW_B * 2;
            kv_bytes = b > kv_bytes ? b : kv_bytes;
        }
    }
    const int64_t wgs = tiles * shape->n_kv_heads;
    if (wgs <= 0 || tiles > kAttnPlanMaxTiles) return whole;
    const bool small_launch = wgs < kAttnSplitBelowWgs;
    const bool range_major = !small_launch && kv_bytes > kAttnRangeMajorBytes;
    if (!small_launch && !range_major) return whole;
    const int64_t ctx_tiles = (max_ctx + BN - 1) / BN;
    const int64_t n_rows_total = (bd.cu_sel[bd.n_req] - bd.cu_sel[0]) * shape->n_q_heads;
    int64_t s_max = kAttnSplitMax;
    const int64_t by_len = ctx_tiles / 16;                           // at least 16 key tiles per piece
    if (s_max > by_len) s_max = by_len;
    if (workspace_bytes < kAttnPlanBytes) return whole;
    const int64_t by_ws = (int64_t)((workspace_bytes - kAttnPlanBytes) / (kAttnPartBytesPerSlot * (size_t)(n_rows_total > 0 ? n_rows_total : 1)));
    if (s_max > by_ws) s_max = by_ws;
    if (s_max < 2) return whole;
    if (range_major) {
        // as small a piece as the slots allow, down to the one whose K and V fit an L2
        int64_t chunk = (ctx_tiles + s_max - 1) / s_max;
        if (chunk < kAttnRangeChunk) chunk = kAttnRangeChunk;
        const int64_t n = (ctx_tiles + chunk - 1) / chunk;
        if (n < 2) return whole;
        return AttnSplitPlan{(int)n, (int)ctx_tiles, 0, 0, (int)chunk};
    }
    // Small pieces at the bottom of the context (every row tile has them, and they start last)
    // fill the gaps the large ones leave; they pay off once the large pieces can be several times
    // their size.
    const bool taper = s_max >= 6 && ctx_tiles >= 8 * kAttnSmallChunk;
    return AttnSplitPlan{(int)s_max, (int)ctx_tiles, kAttnSmallChunk, taper ? kAttnSmallPieces : 0, 0};
}

kvs_status launch_attention_mfma2(const kvs_shape *shape, const AttnBatch &bd, const void *q_sel,
                                  const int32_t *sel_pos, const void *k_cache, const void *v_cache,
                                  float scale, void *out, float *lse_out, void *workspace,
                                  const AttnSplitPlan &plan, hipStream_t st)
{
    AttnTiles td;
    const int64_t tiles = build_attn_tiles(shape, bd, ROWS, td);
    if (tiles < 0) return fail(KVS_EINVAL, "kvs_partial_attention: too many row tiles");
    if (tiles == 0) return KVS_OK;
    const size_t lds_bytes = LDS_BYTES;
    const float scale_log2 = scale * 1.4426950408889634f;
    const int n_splits = plan.n_splits;
    if (n_splits <= 1 || !workspace) {
        const int share_units = share_units_for(shape, tiles);
        const dim3 grid((unsigned)((share_units > 0 ? share_units : tiles) * shape->n_kv_heads));
        return lse_out ? launch_one<true, false>(grid, lds_bytes, st, td, shape, (int)tiles, q_sel, sel_pos, k_cache, v_cache,
                                                 scale_log2, out, lse_out, 1, nullptr, nullptr, nullptr, nullptr, share_units)
                       : launch_one<false, false>(grid, lds_bytes, st, td, shape, (int)tiles, q_sel, sel_pos, k_cache, v_cache,
                                                  scale_log2, out, lse_out, 1, nullptr, nullptr, nullptr, nullptr, share_units);
    }
    if (tiles > PLAN_MAX_TILES) return fail(KVS_EINVAL, "kvs_partial_attention: split launch with %lld row tiles", (long long)tiles);
    // workspace: the pieces' accumulators, their (reference, sums) records, the plan, the piece list.  Pieces are
    // indexed by the row's position in the whole call's output, so offset the tables by the first
    // row of this launch.
    const int64_t n_rows_total = (bd.cu_sel[bd.n_req] - bd.cu_sel[0]) * shape->n_q_heads;
    const int64_t row0 = bd.cu_sel[0] * shape->n_q_heads;
    float *part_o = (float *)workspace - row0 * n_splits * D;
    float4 *ml_base = (float4 *)((char *)workspace + (size_t)n_rows_total * n_splits * D * sizeof(float));
    float4 *part_ml = ml_base - row0 * n_splits;
    int4 *split_plan = (int4 *)(ml_base + n_rows_total * n_splits);
    uint16_t *piece_list = (uint16_t *)(split_plan + 1);
    float round_fill = kAttnRoundFill, piece_overhead = kAttnPieceOverhead;
    int forced_chunk = plan.chunk, small_chunk = plan.small_chunk, n_small = plan.n_small;
    hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(PLAN_NT), 0, st, td, shape->n_q_heads / shape->n_kv_heads,
                       shape->n_kv_heads, (int)tiles, sel_pos, n_splits, plan.ctx_tiles, small_chunk, n_small, round_fill,
                       piece_overhead, forced_chunk, split_plan, piece_list);
    kvs_status stt = check_launch("kvs_partial_attention(plan)");
    if (stt != KVS_OK) return stt;
    const dim3 grid((unsigned)(tiles * shape->n_kv_heads * n_splits));
    stt = lse_out ? launch_one<true, true>(grid, lds_bytes, st, td, shape, (int)tiles, q_sel, sel_pos, k_cache, v_cache,
                                           scale_log2, out, lse_out, n_splits, split_plan, piece_list, part_o, part_ml, 0)
                  : launch_one<false, true>(grid, lds_bytes, st, td, shape, (int)tiles, q_sel, sel_pos, k_cache, v_cache,
                                            scale_log2, out, lse_out, n_splits, split_plan, piece_list, part_o, part_ml, 0);
    if (stt != KVS_OK) return stt;
    return launch_attention_merge(n_rows_total, n_splits, (const float *)workspace, ml_base,
                                  (uint16_t *)out + row0 * D, lse_out ? lse_out + row0 : nullptr, st);
}

} // namespace kvs

