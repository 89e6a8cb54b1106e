// Internal declarations shared by the attention translation units (not part of the ABI).
#pragma once

#include "kvs_internal.h"

namespace kvs {

constexpr int kAttnMaxReq = 64; // requests described per launch (passed by value as a kernel argument)

// Host-side request table, copied into the kernel's argument block: no device allocation, no
// asynchronous host-to-device copy whose source would have to outlive the call.
struct AttnBatch {
    int64_t ctx_off[kAttnMaxReq];     // first cache row of request b
    int64_t ctx_len[kAttnMaxReq];     // context rows of request b
    int64_t cu_sel[kAttnMaxReq + 1];  // selected tokens of request b: [cu_sel[b], cu_sel[b+1]) (global numbering)
    int64_t sel_begin;                // first selected token covered by this launch (= cu_sel[0])
    int32_t n_req;
};

// Per-launch table for the matrix-core kernels: request geometry plus the first row tile of each
// request in the launch's grid (row tiles never span requests).
// The entries are the launch's requests ordered by context length, longest last: the kernels take
// row tiles from the end of the table, so the workgroups with the longest sweeps start first and
// the short ones fill the end of the launch.
struct AttnTiles {
    int64_t ctx_off[kAttnMaxReq];
    int64_t sel_lo[kAttnMaxReq];      // first selected token of the entry's request (global numbering)
    int32_t n_sel[kAttnMaxReq];       // and how many
    int32_t ctx_len[kAttnMaxReq];
    int32_t tile_begin[kAttnMaxReq + 1];
    int32_t n_req;
};

// fills `td` for row tiles of `rows_per_tile` flattened (token, head-in-group) rows; returns the
// number of row tiles, or -1 if the grid would overflow
int64_t build_attn_tiles(const kvs_shape *shape, const AttnBatch &bd, int rows_per_tile, AttnTiles &td);

// Key-range splitting (both matrix-core kernels): a piece stores its unnormalised fp32 accumulators
// and (exponent reference, sum of the weights as the matrix core saw them, sum of the unrounded
// weights, unused) per row; slot = row * n_splits + piece.
constexpr size_t kAttnPartBytesPerSlot = 128 * sizeof(float) + 4 * sizeof(float);
constexpr int kAttnSplitMax = 16;
constexpr int kAttnSplitCus = 256;         // compute units a round of pieces is spread over
constexpr int kAttnSplitBelowWgs = 384;    // launches with fewer workgroups than this get split
constexpr int kAttnSmallChunk = 32;        // key tiles per small piece at the bottom of the context
constexpr int kAttnSmallPieces = 2;        // how many of them
constexpr double kAttnPieceOverhead = 30.0;   // start-up, write-out and merge share of a piece, in key tiles
constexpr double kAttnRoundFill = 0.92;       // pieces per round / compute units the plan aims for
// out = sum_s w_s O_s / sum_s w_s l_s with w_s = 2^(m_s - max m); pieces with l = 0 drop out;
// the log-sum-exp comes from the unrounded sums
kvs_status launch_attention_merge(int64_t n_rows, int n_splits, const float *part_o, const float4 *part_ml,
                                  uint16_t *out, float *lse_out, hipStream_t st);

// What the host fixes for a split launch of the 256-row kernel: piece slots per row tile (1: no
// cutting, nothing else is read), the longest context in key tiles, and the small pieces at the
// bottom of the context (n_small of small_chunk key tiles).  Two cases cut the key range:
//   * launches too small to fill the chip: the size of the large pieces is chosen on the device,
//     from the positions, so that the pieces just fill whole rounds of the compute units;
//   * launches whose K and V no longer fit the last-level cache (kAttnRangeMajorBytes; the 131k
//     context): chunk > 0 fixes the piece size so that one key range of one KV head fits an L2.
//     Workgroups of a KV head that start at different times otherwise sweep K/V at different
//     places and every one of them streams from HBM on its own (measured: 16 % of the matrix
//     peak at 131k against 45 % at 32k, where K and V stay cached).
// Pieces are started from the top of the context down, range by range.
struct AttnSplitPlan {
    int n_splits;
    int ctx_tiles;
    int small_chunk;
    int n_small;
    int chunk;          // 0: chosen on the device
};
constexpr int64_t kAttnRangeMajorBytes = (int64_t)192 << 20;   // K + V of a launch above which key ranges are walked in step
constexpr int kAttnRangeChunk = 256;       // key tiles per piece then: 8192 keys = 4 MiB of K and V per KV head
constexpr int kAttnPlanMaxTiles = 2048;    // row tiles a planned launch may have
// the device-side plan and the list of piece ids (16 bits each, kAttnSplitMax per row tile), after
// the pieces in the workspace
constexpr size_t kAttnPlanBytes = 16 + 2 * (size_t)kAttnSplitMax * kAttnPlanMaxTiles;
static_assert(kAttnSplitMax * kAttnPlanMaxTiles <= 65536, "piece ids are 16 bits");
// 64 query rows per wave (two MFMAs per LDS operand), one wave per SIMD, 256-row tiles.  The plan
// comes from attention_mfma2_plan, which needs the workspace size.
AttnSplitPlan attention_mfma2_plan(const kvs_shape *shape, const AttnBatch &bd, size_t workspace_bytes);
kvs_status launch_attention_mfma2(const kvs_shape *shape, const AttnBatch &bd, const void *q_sel,
                                  const int32_t *sel_pos, const void *k_cache, const void *v_cache,
                                  float scale, void *out, float *lse_out, void *workspace,
                                  const AttnSplitPlan &plan, hipStream_t st);

kvs_status launch_attention_valu(const kvs_shape *shape, const AttnBatch &bd, int64_t n_sel,
                                 const void *q_sel, const int32_t *sel_pos, const void *k_cache,
                                 const void *v_cache, float scale, void *out, float *lse_out,
                                 hipStream_t st);

// bf16, head_dim 128 matrix-core path; returns KVS_EUNSUPPORTED for shapes it does not cover
kvs_status launch_attention_mfma(const kvs_shape *shape, const AttnBatch &bd, int64_t n_sel,
                                 const void *q_sel, const int32_t *sel_pos, const void *k_cache,
                                 const void *v_cache, float scale, void *out, float *lse_out,
                                 void *workspace, size_t workspace_bytes, hipStream_t st);
// workspace that lets small launches split their key range (0 bytes still works, unsplit)
size_t attention_workspace_bytes(const kvs_shape *shape, int32_t batch, int64_t n_rows_total, int64_t n_sel_total);
bool attention_mfma_supports(const kvs_shape *shape);

} // namespace kvs
