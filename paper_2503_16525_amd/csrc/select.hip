// kvs_select_topk: exact top-k of each row of a ragged fp32 score matrix (Alg. 1 step 4),
// order (score descending, index ascending), indices emitted in ascending order.
//
// One workgroup of 1024 lanes (16 waves) owns a row; wave w owns the w-th contiguous sixteenth of
// it, so everything that depends on element order is wave-local except 16 totals.  Scores are
// mapped to order-preserving unsigned keys held in registers (rows up to 49152 entries) or re-read
// from L2 (longer rows).  The key T of the k-th entry is found by an MSB-first radix select with
// digits of 10, 11 and 11 bits:
//   pass 1  histogram of the leading digit over the whole row.  fp32 scores share most of their
//           leading bits, so the histogram is kept in 4 interleaved copies (copy = lane & 3):
//           lanes that meet in one bin land in different LDS banks instead of serialising;
//   pass 2/3 only the keys that share T's leading digit (a few percent of the row) matter; they are
//           copied to an LDS list and histogrammed from there (if they do not fit, the passes rerun
//           over the row).
// The answer is { key > T } plus the first (k - #{key > T}) entries with key == T in index order,
// written by an order-preserving compaction: ballots are counted on the scalar unit, each wave
// keeps a running offset, and a selected lane's slot is
//     #greater before it + min(#equal before it, quota of equals).
// When no tie is cut (the usual case) the predicate collapses to key >= T.  Integer counting only:
// the result is exact and identical from run to run.
#include "kvs_internal.h"

#include <new>

namespace kvs {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;   // 16
constexpr int kMaxRowsPerLaunch = 64;
constexpr int kSurvCap = 6144;                   // LDS list of keys sharing the threshold's leading digit
constexpr int kCopies = 4;                        // interleaved copies of the leading-digit histogram
constexpr int kHist1Ints = 1024 * kCopies;

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

// inclusive prefix sum over the 64 lanes with DPP row shifts and row broadcasts (no LDS round trips)
__device__ __forceinline__ int wave_incl_scan(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
    return v;
}

__device__ __forceinline__ int lanes_below(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
}

// KPT > 0: row length <= KPT * 1024 and keys live in registers; KPT == 0: keys are re-read.
//
// Slots that hold no element (past the end of the row or of the wave's chunk) carry key 0.  Real
// scores never map to a key below 2^22 (-inf maps to 0x007fffff; only NaN patterns go lower), so
// key 0 sits alone in leading-digit bin 0, never reaches the threshold, and no validity mask has to
// be carried through the passes.
template <int KPT>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const float *__restrict__ scores,
                                                             int32_t *__restrict__ idx_out,
                                                             const SelectRows rows)
{
    __shared__ int hist1[kHist1Ints];               // 1024 leading-digit bins x kCopies interleaved copies
    __shared__ int hist2[2048], hist3[2048];        // second / third digit (candidates only)
    __shared__ uint32_t surv[kSurvCap];
    __shared__ int wave_tot[kSelWaves], wave_tot2[kSelWaves];
    __shared__ int bcast[3];                        // chosen digit, rank inside it, entries in it

    const int r = blockIdx.x;
    const int len = rows.len[r];
    const int k = rows.k[r];
    if (k <= 0 || len <= 0) return;                 // uniform over the workgroup
    const float *__restrict__ row = scores + rows.begin[r];
    int32_t *__restrict__ out = idx_out + rows.out_off[r];
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int nj = (len + kSelThreads - 1) / kSelThreads;    // keys per lane
    const uint32_t e0 = (uint32_t)(wave * nj) * kWave + lane; // this lane's first element; slot j holds e0 + 64 j

    constexpr int NREG = KPT > 0 ? KPT : 1;
    uint32_t keys[NREG];
    if constexpr (KPT > 0) {
        // unconditional, clamped loads so that all of them are in flight together
#pragma unroll
        for (int j = 0; j < NREG; ++j) {
            const uint32_t e = e0 + j * kWave;
            const uint32_t key = score_key(row[min(e, (uint32_t)len - 1)]);
            keys[j] = (j < nj && e < (uint32_t)len) ? key : 0u;
        }
    }
    // f(e, key) for every slot of this lane, in element order, without branches
    auto for_keys = [&](auto f) {
        if constexpr (KPT > 0) {
#pragma unroll
            for (int j = 0; j < NREG; ++j) f(e0 + j * kWave, keys[j]);
        } else {
            for (int j = 0; j < nj; ++j) {
                const uint32_t e = e0 + j * kWave;
                const uint32_t key = score_key(row[min(e, (uint32_t)len - 1)]);
                f(e, e < (uint32_t)len ? key : 0u);
            }
        }
    };
    // Each thread holds the count `mine` of the bins it owns (bins ascending with tid).  Finds the
    // thread whose bins hold the remaining-th entry counted from the top; that thread calls
    // resolve(rank_from_top_inside_its_bins).  Every thread must call this.
    auto find_owner = [&](int mine, int remaining, auto resolve) {
        const int incl = wave_incl_scan(mine);
        const int wtot = __builtin_amdgcn_readlane(incl, kWave - 1);
        if (lane == 0) wave_tot[wave] = wtot;
        __syncthreads();
        int above = wtot - incl;                                 // higher lanes of this wave
        for (int w = wave + 1; w < kSelWaves; ++w) above += wave_tot[w];
        if (above < remaining && remaining <= above + mine) resolve(remaining - above);
        __syncthreads();
    };
    // thread t owns bins 2t and 2t+1 of a 2048-bin histogram
    auto find_bin2 = [&](const int *h, int rem) {
        const int b_lo = h[2 * tid], b_hi = h[2 * tid + 1];
        find_owner(b_lo + b_hi, rem, [&](int rank) {
            if (rank <= b_hi) { bcast[0] = 2 * tid + 1; bcast[1] = rank; bcast[2] = b_hi; }
            else { bcast[0] = 2 * tid; bcast[1] = rank - b_hi; bcast[2] = b_lo; }
        });
    };

#pragma unroll
    for (int i = 0; i < kHist1Ints / kSelThreads; ++i) hist1[i * kSelThreads + tid] = 0;
    hist2[tid] = 0; hist2[tid + kSelThreads] = 0;
    hist3[tid] = 0; hist3[tid + kSelThreads] = 0;
    __syncthreads();

    // ---- pass 1: leading 10 bits over the whole row ---------------------------------------------
    const uint32_t copy = lane & (kCopies - 1);
    for_keys([&](uint32_t, uint32_t key) { atomicAdd(&hist1[(key >> 22) * kCopies + copy], 1); });
    __syncthreads();
    {
        int c = 0;
#pragma unroll
        for (int i = 0; i < kCopies; ++i) c += hist1[tid * kCopies + i];
        find_owner(c, k, [&](int rank) { bcast[0] = tid; bcast[1] = rank; bcast[2] = c; });
    }
    const uint32_t d1 = (uint32_t)bcast[0];
    int remaining = bcast[1];
    const int n_cand = bcast[2];
    uint32_t T;
    int eq_total;
    if (n_cand <= kSurvCap) {
        // ---- copy the candidates to LDS (wave-local offsets, 16 totals exchanged) ---------------
        int mine = 0;
        for_keys([&](uint32_t, uint32_t key) { mine += __popcll(__ballot((key >> 22) == d1)); });
        if (lane == 0) wave_tot2[wave] = mine;
        __syncthreads();
        uint32_t base = 0;
        for (int w = 0; w < wave; ++w) base += wave_tot2[w];
        for_keys([&](uint32_t, uint32_t key) {
            const bool hit = (key >> 22) == d1;
            const uint64_t m = __ballot(hit);
            if (hit) surv[base + lanes_below(m)] = key;
            base += __popcll(m);
        });
        __syncthreads();
        // ---- passes 2 and 3 on the list ------------------------------------------------------------
        for (uint32_t i = tid; i < (uint32_t)n_cand; i += kSelThreads) atomicAdd(&hist2[(surv[i] >> 11) & 2047u], 1);
        __syncthreads();
        find_bin2(hist2, remaining);
        const uint32_t d2 = (uint32_t)bcast[0];
        remaining = bcast[1];
        for (uint32_t i = tid; i < (uint32_t)n_cand; i += kSelThreads) {
            const uint32_t key = surv[i];
            if (((key >> 11) & 2047u) == d2) atomicAdd(&hist3[key & 2047u], 1);
        }
        __syncthreads();
        find_bin2(hist3, remaining);
        T = (d1 << 22) | (d2 << 11) | (uint32_t)bcast[0];
        remaining = bcast[1];
        eq_total = bcast[2];
    } else {
        // ---- too many candidates for the list: passes 2 and 3 rerun over the row ------------------
        for_keys([&](uint32_t, uint32_t key) {
            if ((key >> 22) == d1) atomicAdd(&hist2[(key >> 11) & 2047u], 1);
        });
        __syncthreads();
        find_bin2(hist2, remaining);
        const uint32_t p2 = (d1 << 11) | (uint32_t)bcast[0];
        remaining = bcast[1];
        for_keys([&](uint32_t, uint32_t key) {
            if ((key >> 11) == p2) atomicAdd(&hist3[key & 2047u], 1);
        });
        __syncthreads();
        find_bin2(hist3, remaining);
        T = (p2 << 11) | (uint32_t)bcast[0];
        remaining = bcast[1];
        eq_total = bcast[2];
    }
    if (T == 0u) T = 1u;                             // only reachable with NaN scores: never select padding
    const int quota_eq = remaining;                  // entries equal to T that are taken
    const bool all_eq_taken = quota_eq == eq_total;  // no tie is cut: the answer is { key >= T }

    // ---- ordered compaction ---------------------------------------------------------------------
    int n_sel = 0, n_eq = 0;                         // this wave's totals (scalar)
    if (all_eq_taken) {
        for_keys([&](uint32_t, uint32_t key) { n_sel += __popcll(__ballot(key >= T)); });
    } else {
        for_keys([&](uint32_t, uint32_t key) {
            n_sel += __popcll(__ballot(key > T));
            n_eq += __popcll(__ballot(key == T));
        });
    }
    if (lane == 0) { wave_tot[wave] = n_sel; wave_tot2[wave] = n_eq; }
    __syncthreads();
    uint32_t base_sel = 0, base_eq = 0;
    for (int w = 0; w < wave; ++w) { base_sel += wave_tot[w]; base_eq += wave_tot2[w]; }
    if (all_eq_taken) {
        for_keys([&](uint32_t e, uint32_t key) {
            const bool sel = key >= T;
            const uint64_t m = __ballot(sel);
            if (sel) out[base_sel + lanes_below(m)] = (int32_t)e;
            base_sel += __popcll(m);
        });
    } else {
        for_keys([&](uint32_t e, uint32_t key) {
            const bool is_gt = key > T, is_eq = key == T;
            const uint64_t m_gt = __ballot(is_gt), m_eq = __ballot(is_eq);
            const uint32_t gt_before = base_sel + lanes_below(m_gt);
            const uint32_t eq_before = base_eq + lanes_below(m_eq);
            if (is_gt) out[gt_before + min(eq_before, (uint32_t)quota_eq)] = (int32_t)e;
            else if (is_eq && eq_before < (uint32_t)quota_eq) out[gt_before + eq_before] = (int32_t)e;
            base_sel += __popcll(m_gt);
            base_eq += __popcll(m_eq);
        });
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
        else if (max_len <= 8 * kSelThreads) hipLaunchKernelGGL(select_kernel<8>, grid, block, 0, hs, scores, idx_out, rows);
        else if (max_len <= 16 * kSelThreads) hipLaunchKernelGGL(select_kernel<16>, grid, block, 0, hs, scores, idx_out, rows);
        else if (max_len <= 32 * kSelThreads) hipLaunchKernelGGL(select_kernel<32>, grid, block, 0, hs, scores, idx_out, rows);
        else if (max_len <= 36 * kSelThreads) hipLaunchKernelGGL(select_kernel<36>, grid, block, 0, hs, scores, idx_out, rows);
        else if (max_len <= 48 * kSelThreads) hipLaunchKernelGGL(select_kernel<48>, grid, block, 0, hs, scores, idx_out, rows);
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
