// kvs_select_topk: exact top-k of each row of a ragged fp32 score matrix (Alg. 1 step 4),
// order (score descending, index ascending), indices emitted in ascending order.
//
// One workgroup of 1024 lanes owns a row.  Scores are mapped to order-preserving unsigned keys
// and kept in registers (rows up to 32768 entries) or re-read from L2 (longer rows).  A 4-pass
// MSB-first radix select over an LDS histogram finds the key T of the k-th entry; the answer is
// then { key > T } plus the first (k - #{key > T}) entries with key == T in index order.  That
// set is written by an order-preserving compaction: wave ballots give per-(tile, wave) counts,
// one wave scans them, and every selected lane computes its output slot in closed form
//     slot = #greater before it + min(#equal before it, quota of equals).
// Integer counting only: the result is exact and identical from run to run.
#include "kvs_internal.h"

#include <new>

namespace kvs {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;   // 16
constexpr int kChunkTiles = 32;                  // tiles (of 1024 entries) per compaction round, streaming path
constexpr int kMaxRowsPerLaunch = 64;

struct SelectRows {
    int64_t begin[kMaxRowsPerLaunch];    // first score of the row
    int64_t out_off[kMaxRowsPerLaunch];  // where the row's indices go in idx_out
    int32_t len[kMaxRowsPerLaunch];
    int32_t k[kMaxRowsPerLaunch];
};

// monotone map fp32 -> uint32 (larger score <=> larger key); -0 is first folded onto +0
__device__ __forceinline__ uint32_t score_key(float s)
{
    const uint32_t u = __float_as_uint(s + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int wave_excl_scan(int v, int lane, int &total)
{
    int incl = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int t = __shfl_up(incl, d);
        if (lane >= d) incl += t;
    }
    total = __shfl(incl, kWave - 1);
    return incl - v;
}

// KPT > 0: row length <= KPT * 1024 and keys live in registers; KPT == 0: keys are re-read.
template <int KPT>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const float *__restrict__ scores,
                                                             int32_t *__restrict__ idx_out,
                                                             const SelectRows rows)
{
    __shared__ int hist[256];
    __shared__ int bcast[2];                       // chosen digit, remaining k
    __shared__ int cnt_gt[kChunkTiles * kSelWaves];
    __shared__ int cnt_eq[kChunkTiles * kSelWaves];
    __shared__ int chunk_tot[2];

    const int r = blockIdx.x;
    const int len = rows.len[r];
    const int k = rows.k[r];
    if (k <= 0 || len <= 0) return;                // uniform over the workgroup
    const float *__restrict__ row = scores + rows.begin[r];
    int32_t *__restrict__ out = idx_out + rows.out_off[r];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int n_tiles = (len + kSelThreads - 1) / kSelThreads;

    constexpr int NREG = KPT > 0 ? KPT : 1;
    uint32_t keys[NREG];
    if (KPT > 0) {
#pragma unroll
        for (int j = 0; j < NREG; ++j) {
            const int e = j * kSelThreads + tid;
            keys[j] = e < len ? score_key(row[e]) : 0u;
        }
    }
    // ---- radix select: T = key of the k-th entry in descending order --------------------
    uint32_t prefix = 0, mask = 0;
    int remaining = k;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        if (KPT > 0) {
#pragma unroll
            for (int j = 0; j < NREG; ++j) {
                const int e = j * kSelThreads + tid;
                if (e < len && (keys[j] & mask) == prefix) atomicAdd(&hist[(keys[j] >> shift) & 255u], 1);
            }
        } else {
            for (int j = 0; j < n_tiles; ++j) {
                const int e = j * kSelThreads + tid;
                if (e < len) {
                    const uint32_t key = score_key(row[e]);
                    if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
                }
            }
        }
        __syncthreads();
        if (wave == 0) {
            // lane l owns bins 4l..4l+3; suffix sums locate the bin that holds the remaining-th entry
            const int b0 = hist[4 * lane], b1 = hist[4 * lane + 1], b2 = hist[4 * lane + 2], b3 = hist[4 * lane + 3];
            const int mine = b0 + b1 + b2 + b3;
            int total;
            const int below = wave_excl_scan(mine, lane, total);   // entries in lower lanes' bins
            const int above = total - below - mine;                 // entries in higher lanes' bins
            if (above < remaining && remaining <= above + mine) {   // exactly one lane
                int acc = above, digit = 4 * lane + 3;
                if (acc + b3 >= remaining) { digit = 4 * lane + 3; }
                else if ((acc += b3) + b2 >= remaining) { digit = 4 * lane + 2; }
                else if ((acc += b2) + b1 >= remaining) { digit = 4 * lane + 1; }
                else { acc += b1; digit = 4 * lane; }
                bcast[0] = digit;
                bcast[1] = remaining - acc;
            }
        }
        __syncthreads();
        prefix |= (uint32_t)bcast[0] << shift;
        mask |= 255u << shift;
        remaining = bcast[1];
        // the next pass's zeroing of hist is separated from these reads by its own barrier
    }
    const uint32_t T = prefix;
    const int quota_eq = remaining;                // entries equal to T that are taken

    // ---- ordered compaction ----------------------------------------------------------------
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
    int base_gt = 0, base_eq = 0;
    constexpr int TPC = KPT > 0 ? KPT : kChunkTiles;   // tiles per compaction round (unrolled)
    for (int tile0 = 0; tile0 < n_tiles; tile0 += TPC) {
        const int tiles = min(TPC, n_tiles - tile0);
#pragma unroll
        for (int j = 0; j < TPC; ++j) {
            if (j < tiles) {
                const int e = (tile0 + j) * kSelThreads + tid;
                const bool valid = e < len;
                const uint32_t key = KPT > 0 ? keys[KPT > 0 ? j : 0] : (valid ? score_key(row[e]) : 0u);
                const uint64_t m_gt = __ballot(valid && key > T);
                const uint64_t m_eq = __ballot(valid && key == T);
                if (lane == 0) {
                    cnt_gt[j * kSelWaves + wave] = __popcll(m_gt);
                    cnt_eq[j * kSelWaves + wave] = __popcll(m_eq);
                }
            }
        }
        __syncthreads();
        if (wave == 0) {
            // exclusive scan of the (tile, wave) counts in index order; 8 entries per lane
            const int n_ent = tiles * kSelWaves;
            int g[8], q[8], sg = 0, sq = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int x = lane * 8 + i;
                g[i] = x < n_ent ? cnt_gt[x] : 0;
                q[i] = x < n_ent ? cnt_eq[x] : 0;
                sg += g[i];
                sq += q[i];
            }
            int tg, tq;
            int pg = wave_excl_scan(sg, lane, tg);
            int pq = wave_excl_scan(sq, lane, tq);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int x = lane * 8 + i;
                if (x < n_ent) { cnt_gt[x] = pg; cnt_eq[x] = pq; }
                pg += g[i];
                pq += q[i];
            }
            if (lane == 0) { chunk_tot[0] = tg; chunk_tot[1] = tq; }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < TPC; ++j) {
            if (j < tiles) {
                const int e = (tile0 + j) * kSelThreads + tid;
                const bool valid = e < len;
                const uint32_t key = KPT > 0 ? keys[KPT > 0 ? j : 0] : (valid ? score_key(row[e]) : 0u);
                const bool is_gt = valid && key > T, is_eq = valid && key == T;
                const uint64_t m_gt = __ballot(is_gt);
                const uint64_t m_eq = __ballot(is_eq);
                const int gt_before = base_gt + cnt_gt[j * kSelWaves + wave] + __popcll(m_gt & lt_mask);
                const int eq_before = base_eq + cnt_eq[j * kSelWaves + wave] + __popcll(m_eq & lt_mask);
                if (is_gt) out[gt_before + min(eq_before, quota_eq)] = e;
                else if (is_eq && eq_before < quota_eq) out[gt_before + eq_before] = e;
            }
        }
        base_gt += chunk_tot[0];
        base_eq += chunk_tot[1];
        __syncthreads();                           // cnt_* and chunk_tot are rewritten next round
    }
}

} // namespace


// rows given as (begin, len) pairs so that callers with gaps between rows (decode contexts with
// slack) can use the same kernel; arguments are already validated
kvs_status launch_select(const float *scores, int32_t n_rows, const int64_t *begin, const int64_t *len,
                         const int32_t *k_row, int32_t *idx_out, hipStream_t hs)
{
    int64_t out_base = 0;
    for (int32_t r0 = 0; r0 < n_rows; r0 += kMaxRowsPerLaunch) {
        const int nr = (n_rows - r0) < kMaxRowsPerLaunch ? (n_rows - r0) : kMaxRowsPerLaunch;
        SelectRows rows;
        int64_t max_len = 0;
        for (int i = 0; i < kMaxRowsPerLaunch; ++i) {
            const bool live = i < nr;
            rows.begin[i] = live ? begin[r0 + i] : 0;
            rows.len[i] = live ? (int32_t)len[r0 + i] : 0;
            rows.k[i] = live ? k_row[r0 + i] : 0;
            rows.out_off[i] = out_base;
            if (live) {
                out_base += k_row[r0 + i];
                if (k_row[r0 + i] > 0 && len[r0 + i] > max_len) max_len = len[r0 + i];
            }
        }
        if (max_len == 0) continue;
        dim3 grid(nr), block(kSelThreads);
        if (max_len <= 4 * kSelThreads) hipLaunchKernelGGL(select_kernel<4>, grid, block, 0, hs, scores, idx_out, rows);
        else if (max_len <= 16 * kSelThreads) hipLaunchKernelGGL(select_kernel<16>, grid, block, 0, hs, scores, idx_out, rows);
        else if (max_len <= 32 * kSelThreads) hipLaunchKernelGGL(select_kernel<32>, grid, block, 0, hs, scores, idx_out, rows);
        else hipLaunchKernelGGL(select_kernel<0>, grid, block, 0, hs, scores, idx_out, rows);
        kvs_status st = check_launch("kvs_select_topk");
        if (st != KVS_OK) return st;
    }
    return KVS_OK;
}

} // namespace kvs

extern "C" kvs_status kvs_select_topk(const float *scores, int32_t n_rows, const int64_t *row_off,
                                      const int32_t *k_row, int32_t *idx_out,
                                      void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace kvs;
    (void)workspace;
    (void)workspace_bytes;
    if (n_rows < 0) return fail(KVS_EINVAL, "kvs_select_topk: n_rows < 0");
    if (n_rows == 0) return KVS_OK;
    if (!row_off || !k_row) return fail(KVS_EINVAL, "kvs_select_topk: row_off/k_row is NULL");
    int64_t total_k = 0;
    for (int32_t r = 0; r < n_rows; ++r) {
        const int64_t len = row_off[r + 1] - row_off[r];
        if (len < 0) return fail(KVS_EINVAL, "kvs_select_topk: row_off decreases at row %d", r);
        if (len > 0x7fffffffLL) return fail(KVS_EINVAL, "kvs_select_topk: row %d longer than 2^31-1", r);
        if (k_row[r] < 0 || k_row[r] > len) return fail(KVS_EINVAL, "kvs_select_topk: k_row[%d]=%d outside [0,%lld]", r, k_row[r], (long long)len);
        total_k += k_row[r];
    }
    if (total_k == 0) return KVS_OK;
    if (!scores || !idx_out) return fail(KVS_EINVAL, "kvs_select_topk: scores/idx_out is NULL");
    // (begin, len) view of the packed rows
    constexpr int kStack = 256;
    int64_t lens_stack[kStack];
    int64_t *lens = n_rows <= kStack ? lens_stack : new (std::nothrow) int64_t[n_rows];
    if (!lens) return fail(KVS_EINVAL, "kvs_select_topk: out of host memory");
    for (int32_t r = 0; r < n_rows; ++r) lens[r] = row_off[r + 1] - row_off[r];
    kvs_status st = launch_select(scores, n_rows, row_off, lens, k_row, idx_out, (hipStream_t)stream);
    if (lens != lens_stack) delete[] lens;
    return st;
}
