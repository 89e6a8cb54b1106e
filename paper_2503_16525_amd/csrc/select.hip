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
//
// Rows longer than 49152 entries do not fit one workgroup's registers.  With a workspace they are
// cut into parts of 32768 entries, one workgroup each, and the same select runs as four launches
// with the launch boundaries as the only synchronisation (no atomics between workgroups, no
// spinning): leading-digit histogram per part -> every part finds the threshold's leading digit
// from the row's histograms and sets its candidates aside -> one workgroup per row resolves the
// other two digits on the candidates and hands every part its threshold, its share of the tie
// and its place in the output -> the parts write.  Without a workspace such rows take the
// one-workgroup kernel, which then re-reads its keys from L2 on every sweep.
#include "kvs_internal.h"

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

// ---- top-k of one row whose leading-digit histogram already exists -------------------------------------
// kvs_deviation_topk: the scoring kernel has left the row's keys and the histogram of their leading
// kKeyHistBits bits (finite scores only; -inf entries, the non-candidates, are not counted and rank
// below everything that is).  One workgroup per 1024 keys and two launches finish the selection:
//   candidates  every workgroup reads the threshold's bin d1 off the histogram (the same answer in
//               each), counts its keys above that bin and copies its keys inside it, in index order,
//               to its segment of a candidate list;
//   write       every workgroup resolves the remaining 19 bits on the (few hundred) candidates of the
//               whole row in two small LDS histograms (10 + 9 bits), counts what the parts before it
//               contribute -- keys above the threshold, and keys equal to it, which are taken in
//               index order while the quota lasts -- and writes its own selection at that offset.
// The launch boundary is the only synchronisation between workgroups.  The histogram is stored with
// neighbouring bins 1 KiB apart (scores share their leading bits: the atomics of one scoring launch
// fall on a few dozen neighbouring bins, which would otherwise share a few cache lines -- measured,
// that layout more than doubles the scoring kernel's time); the write launch clears it for the next
// call.
constexpr int kFuThreads = 256;
constexpr int kFuWaves = kFuThreads / kWave;
constexpr int kFuKpt = 4;                          // keys per lane: one 16-byte load
constexpr int kFuPart = kFuThreads * kFuKpt;       // keys per workgroup
constexpr int kFuBinsPerThread = kKeyHistBins / kFuThreads;   // 32
constexpr int kCandCap = 4096;                     // candidates kept in LDS by the write launch

// Every thread holds the count `mine` of the bins it owns (bins ascending with the thread index).
// The thread whose bins hold the remaining-th entry counted from the top calls resolve(rank from
// the top inside its bins); returns the total over the workgroup.  Every thread must call this.
template <typename F>
__device__ __forceinline__ int fu_owner_from_top(int mine, int remaining, int *wave_tot, F resolve)
{
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int incl = wave_incl_scan(mine);
    const int wtot = __builtin_amdgcn_readlane(incl, kWave - 1);
    if (lane == 0) wave_tot[wave] = wtot;
    __syncthreads();
    int above = wtot - incl, total = 0;
#pragma unroll
    for (int w = 0; w < kFuWaves; ++w) {
        const int t = wave_tot[w];
        total += t;
        if (w > wave) above += t;
    }
    if (above < remaining && remaining <= above + mine) resolve(remaining - above);
    __syncthreads();
    return total;
}

// this lane's four keys of part `part`: elements part * kFuPart + 4 * tid + j; slots past the row carry
// key 0, below every real key
__device__ __forceinline__ void fu_load_keys(const uint32_t *__restrict__ keys, int n, int part, uint32_t (&key)[kFuKpt])
{
    const int e = part * kFuPart + kFuKpt * (int)threadIdx.x;
    if (e + kFuKpt <= n) {
        const uint4 v = *reinterpret_cast<const uint4 *>(keys + e);
        key[0] = v.x; key[1] = v.y; key[2] = v.z; key[3] = v.w;
    } else {
#pragma unroll
        for (int j = 0; j < kFuKpt; ++j) key[j] = e + j < n ? keys[e + j] : 0u;
    }
}

struct FusedRow {          // what the candidates launch leaves for the write launch
    int d1;                // leading bits of the threshold key; -1: fewer finite scores than k
    int rank;              // the threshold is the rank-th key of bin d1 from the top (d1 < 0: -inf entries to take)
};

__global__ __launch_bounds__(kFuThreads) void fused_cand_kernel(const uint32_t *__restrict__ keys, const uint32_t *__restrict__ hist,
                                                                int n, int k, uint32_t *__restrict__ cand,
                                                                int2 *__restrict__ part_rec /* (candidates, keys above d1) */,
                                                                FusedRow *__restrict__ row_rec)
{
    __shared__ int wave_tot[kFuWaves], wave_tot2[kFuWaves], bcast[2], found[2], range_tot[kFuThreads];
    const int part = blockIdx.x;
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    uint32_t key[kFuKpt];
    fu_load_keys(keys, n, part, key);
    // Thread (wave w, lane l) owns the 32 bins of range rho = 4 l + w, bins 32 rho .. 32 rho + 31: bin
    // 32 rho + i sits at (32 w + i) * 64 + l, so every load below is one coalesced 256-byte row per wave.
    static_assert(kFuBinsPerThread == 32 && kFuWaves == 4, "matches key_hist_slot");
    const int rho = 4 * (int)lane + wave;
    int c[kFuBinsPerThread], quad[kFuBinsPerThread / 4], mine = 0;
#pragma unroll
    for (int i = 0; i < kFuBinsPerThread; ++i) {
        c[i] = 0;
#pragma unroll
        for (int r = 0; r < kKeyHistCopies; ++r) c[i] += (int)hist[r * kKeyHistBins + (32 * wave + i) * 64 + (int)lane];
    }
#pragma unroll
    for (int q = 0; q < kFuBinsPerThread / 4; ++q) {
        quad[q] = (c[4 * q] + c[4 * q + 1]) + (c[4 * q + 2] + c[4 * q + 3]);
        mine += quad[q];
    }
    // the scan runs over the ranges in bin order: thread t takes range t's total
    range_tot[rho] = mine;
    if (tid < 2) { bcast[tid] = -1; found[tid] = -1; }
    __syncthreads();
    const int n_finite = fu_owner_from_top(range_tot[tid], k, wave_tot, [&](int rank) { bcast[0] = (int)tid; bcast[1] = rank; });
    if (bcast[0] == rho) {
        // this thread holds the counts of the range the threshold falls into: from the top, first the
        // group of four bins, then the bin inside it
        int rank = bcast[1];
        int q = kFuBinsPerThread / 4 - 1;
#pragma unroll
        for (int i = kFuBinsPerThread / 4 - 1; i > 0; --i)
            if (q == i && rank > quad[i]) { rank -= quad[i]; q = i - 1; }
        int c4[4] = {0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < kFuBinsPerThread / 4; ++i)
            if (q == i) { c4[0] = c[4 * i]; c4[1] = c[4 * i + 1]; c4[2] = c[4 * i + 2]; c4[3] = c[4 * i + 3]; }
        int b = 3;
        if (rank > c4[3]) { rank -= c4[3]; b = 2; if (rank > c4[2]) { rank -= c4[2]; b = 1; if (rank > c4[1]) { rank -= c4[1]; b = 0; } } }
        found[0] = rho * kFuBinsPerThread + 4 * q + b;
        found[1] = rank;
    }
    __syncthreads();
    const int d1 = found[0];
    // this part's keys above the threshold's bin, and those inside it (index order kept)
    int n_above = 0, n_in = 0;
    bool in[kFuKpt];
#pragma unroll
    for (int j = 0; j < kFuKpt; ++j) {
        const int bin = (int)(key[j] >> kKeyHistShift);
        // without a threshold bin every finite score is taken: "above" then means finite
        n_above += d1 >= 0 ? (bin > d1) : (key[j] > kKeyNegInf);
        in[j] = d1 >= 0 && bin == d1;
        n_in += in[j];
    }
    const int incl = wave_incl_scan(n_in);
    const int wtot = __builtin_amdgcn_readlane(incl, kWave - 1);
    n_above = wave_sum_i32(n_above);
    if (lane == 0) { wave_tot[wave] = wtot; wave_tot2[wave] = n_above; }
    __syncthreads();
    int at = incl - n_in, total_in = 0, total_above = 0;
#pragma unroll
    for (int w = 0; w < kFuWaves; ++w) {
        if (w < wave) at += wave_tot[w];
        total_in += wave_tot[w];
        total_above += wave_tot2[w];
    }
    uint32_t *__restrict__ seg = cand + (size_t)part * kFuPart;
#pragma unroll
    for (int j = 0; j < kFuKpt; ++j)
        if (in[j]) seg[at++] = key[j];
    if (tid == 0) {
        part_rec[part] = make_int2(total_in, total_above);
        if (part == 0) *row_rec = FusedRow{d1, d1 >= 0 ? found[1] : k - n_finite};
    }
}

__global__ __launch_bounds__(kFuThreads) void fused_write_kernel(const uint32_t *__restrict__ keys, uint32_t *__restrict__ hist,
                                                                 int n, int k, int n_parts, const uint32_t *__restrict__ cand,
                                                                 const int2 *__restrict__ part_rec, const FusedRow *__restrict__ row_rec,
                                                                 int32_t *__restrict__ out)
{
    __shared__ __align__(16) int h2[1024], h3[512];
    __shared__ uint32_t list[kCandCap];
    __shared__ int cand_begin[kFusedMaxParts + 1];     // candidates of the parts before q
    __shared__ int above_begin[kFusedMaxParts + 1];    // keys above the threshold's bin in the parts before q
    __shared__ int wave_tot[kFuWaves], wave_tot2[kFuWaves], bcast[2];
    const int part = blockIdx.x;
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    uint32_t key[kFuKpt];
    fu_load_keys(keys, n, part, key);
    const FusedRow row = *row_rec;
    // Rows of up to kSpecParts parts fetch the first kSpec candidates of every part right away, together
    // with the records that say how many there are: when no part has more (a few hundred candidates
    // spread over the row) the list is complete without a second, dependent trip to memory.
    constexpr int kSpec = 32, kSpecParts = 32, kSpecPerThread = kSpec * kSpecParts / kFuThreads;
    const bool speculate = n_parts <= kSpecParts;       // uniform
    uint32_t spec[kSpecPerThread];
    if (speculate) {
#pragma unroll
        for (int r = 0; r < kSpecPerThread; ++r) {
            const int flat = (int)tid + r * kFuThreads, q = flat / kSpec, i = flat % kSpec;
            spec[r] = q < n_parts ? cand[(size_t)q * kFuPart + i] : 0u;
        }
    }
    // the histogram has been read by every workgroup of the launch before: clear it for the next call
    if (part == 0)
        for (int i = tid; i < kKeyHistCopies * kKeyHistBins; i += kFuThreads) hist[i] = 0u;
    // prefix sums over the parts (thread q holds part q; n_parts <= kFuThreads)
    {
        const int2 rec = (int)tid < n_parts ? part_rec[tid] : make_int2(0, 0);
        const int ic = wave_incl_scan(rec.x), ia = wave_incl_scan(rec.y);
        if (lane == kWave - 1) { wave_tot[wave] = ic; wave_tot2[wave] = ia; }
        if (tid == 0) { cand_begin[0] = 0; above_begin[0] = 0; bcast[0] = 0; bcast[1] = 0; }
        __syncthreads();
        int bc = 0, ba = 0;
        for (int w = 0; w < wave; ++w) { bc += wave_tot[w]; ba += wave_tot2[w]; }
        if ((int)tid < n_parts) { cand_begin[tid + 1] = bc + ic; above_begin[tid + 1] = ba + ia; }
        if (rec.x > kSpec) bcast[1] = 1;                // a part with more candidates than were fetched ahead (any writer)
        for (int i = tid; i < 1024; i += kFuThreads) h2[i] = 0;
        for (int i = tid; i < 512; i += kFuThreads) h3[i] = 0;
        __syncthreads();
    }
    const int n_cand = cand_begin[n_parts];
    const bool listed = n_cand <= kCandCap;            // uniform
    const bool spec_ok = bcast[1] == 0;                // uniform
    // candidate f of the row, in index order: entry f - cand_begin[q] of part q's segment
    auto fetch = [&](int f) -> uint32_t {
        int lo = 0, hi = n_parts;                       // largest q with cand_begin[q] <= f
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (cand_begin[mid] <= f) lo = mid; else hi = mid;
        }
        return cand[(size_t)lo * kFuPart + (f - cand_begin[lo])];
    };
    if (listed) {
        if (speculate && spec_ok) {
#pragma unroll
            for (int r = 0; r < kSpecPerThread; ++r) {
                const int flat = (int)tid + r * kFuThreads, q = flat / kSpec, i = flat % kSpec;
                if (q < n_parts && i < cand_begin[q + 1] - cand_begin[q]) list[cand_begin[q] + i] = spec[r];
            }
        } else {
            for (int f = tid; f < n_cand; f += kFuThreads) list[f] = fetch(f);
        }
        __syncthreads();
    }
    // g(key) over the candidates [0, upto) of the row
    auto for_cands = [&](int upto, auto g) {
        for (int f = tid; f < upto; f += kFuThreads) g(listed ? list[f] : fetch(f));
    };
    uint32_t T;
    int quota_eq;
    if (row.d1 < 0) {
        T = kKeyNegInf;                                 // every finite score, then -inf entries, lowest indices first
        quota_eq = row.rank;
    } else {
        int remaining = row.rank;
        for_cands(n_cand, [&](uint32_t kk) { atomicAdd(&h2[(kk >> 9) & 1023u], 1); });
        if (tid < 2) bcast[tid] = 0;                    // (stays defined if NaN scores leave a digit without an owner)
        __syncthreads();
        {
            const int4 b = *reinterpret_cast<const int4 *>(&h2[4 * tid]);
            fu_owner_from_top(b.x + b.y + b.z + b.w, remaining, wave_tot, [&](int rank) {
                int bin = 3;
                if (rank > b.w) { rank -= b.w; bin = 2; if (rank > b.z) { rank -= b.z; bin = 1; if (rank > b.y) { rank -= b.y; bin = 0; } } }
                bcast[0] = 4 * (int)tid + bin;
                bcast[1] = rank;
            });
        }
        const uint32_t d2 = (uint32_t)bcast[0];
        remaining = bcast[1];
        __syncthreads();
        for_cands(n_cand, [&](uint32_t kk) { if (((kk >> 9) & 1023u) == d2) atomicAdd(&h3[kk & 511u], 1); });
        if (tid < 2) bcast[tid] = 0;
        __syncthreads();
        {
            const int2 b = *reinterpret_cast<const int2 *>(&h3[2 * tid]);
            fu_owner_from_top(b.x + b.y, remaining, wave_tot, [&](int rank) {
                int bin = 1;
                if (rank > b.y) { rank -= b.y; bin = 0; }
                bcast[0] = 2 * (int)tid + bin;
                bcast[1] = rank;
            });
        }
        T = ((uint32_t)row.d1 << kKeyHistShift) | (d2 << 9) | (uint32_t)bcast[0];
        quota_eq = bcast[1];
    }
    if (T == 0u) T = 1u;                                // only reachable with NaN scores: never select padding
    quota_eq = max(quota_eq, 0);

    // what the parts before this one contribute
    int gt_before, eq_before;
    if (row.d1 < 0) {
        gt_before = above_begin[part];                  // their finite scores
        eq_before = part * kFuPart - gt_before;         // and their -inf entries (earlier parts are full)
    } else {
        int g = 0, e = 0;
        for_cands(cand_begin[part], [&](uint32_t kk) { g += kk > T; e += kk == T; });
        g = wave_sum_i32(g);
        e = wave_sum_i32(e);
        if (lane == 0) { wave_tot[wave] = g; wave_tot2[wave] = e; }
        __syncthreads();
        gt_before = above_begin[part];
        eq_before = 0;
#pragma unroll
        for (int w = 0; w < kFuWaves; ++w) { gt_before += wave_tot[w]; eq_before += wave_tot2[w]; }
        __syncthreads();
    }
    // ---- ordered write of this part: { key > T } and the entries equal to T while the quota lasts ----
    int n_gt = 0, n_eq = 0;
#pragma unroll
    for (int j = 0; j < kFuKpt; ++j) { n_gt += key[j] > T; n_eq += key[j] == T; }
    const int ig = wave_incl_scan(n_gt), ie = wave_incl_scan(n_eq);
    if (lane == kWave - 1) { wave_tot[wave] = ig; wave_tot2[wave] = ie; }
    __syncthreads();
    uint32_t gt = (uint32_t)(gt_before + ig - n_gt), eq = (uint32_t)(eq_before + ie - n_eq);
    for (int w = 0; w < wave; ++w) { gt += wave_tot[w]; eq += wave_tot2[w]; }
    const int32_t e0 = part * kFuPart + kFuKpt * (int)tid;
#pragma unroll
    for (int j = 0; j < kFuKpt; ++j) {
        const bool is_gt = key[j] > T, is_eq = key[j] == T;
        const uint32_t slot = gt + min(eq, (uint32_t)quota_eq);
        // (with well-formed scores every slot is below k; the guard keeps NaN rows inside the output)
        if ((is_gt || (is_eq && eq < (uint32_t)quota_eq)) && slot < (uint32_t)k) out[slot] = e0 + j;
        gt += is_gt;
        eq += is_eq;
    }
}

// ---- rows cut into parts: one workgroup per part, four launches ------------------------------------
constexpr int kPartKpt = 32;
constexpr int kPartLen = kPartKpt * kSelThreads;      // entries per part
constexpr int kOneWgMax = 48 * kSelThreads;           // longest row whose keys one workgroup holds in registers
constexpr int kMaxParts = 64;                         // parts per group of launches

struct LongParts {
    int64_t begin[kMaxParts];      // first score of the part
    int64_t cand_off[kMaxParts];   // the part's segment of the candidate list
    int64_t out_off[kMaxParts];    // where the row's indices go in idx_out
    int32_t len[kMaxParts];
    int32_t local0[kMaxParts];     // row-local index of the part's first entry
    int32_t row_first[kMaxParts];  // first part of the part's row
    int32_t row_parts[kMaxParts];  // parts of that row
    int32_t k[kMaxParts];          // the row's k
};

struct PartKeys {
    uint32_t key[kPartKpt];
    uint32_t e0;                   // part-local index of slot 0; slot j holds e0 + 64 j
};

// wave w owns the w-th contiguous sixteenth of the part (as in select_kernel); empty slots carry key 0
__device__ __forceinline__ void load_part(const float *__restrict__ row, int len, PartKeys &pk)
{
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int nj = (len + kSelThreads - 1) / kSelThreads;
    pk.e0 = (uint32_t)(wave * nj) * kWave + lane;
#pragma unroll
    for (int j = 0; j < kPartKpt; ++j) {
        const uint32_t e = pk.e0 + j * kWave;
        const uint32_t key = score_key(row[min(e, (uint32_t)len - 1)]);
        pk.key[j] = (j < nj && e < (uint32_t)len) ? key : 0u;
    }
}

// Every thread holds the count `mine` of the bins it owns (bins ascending with the thread index).
// The thread whose bins hold the remaining-th entry counted from the top calls
// resolve(rank from the top inside its bins).  Every thread of the workgroup must call this.
template <typename F>
__device__ __forceinline__ void owner_from_top(int mine, int remaining, int *wave_tot, F resolve)
{
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int incl = wave_incl_scan(mine);
    const int wtot = __builtin_amdgcn_readlane(incl, kWave - 1);
    if (lane == 0) wave_tot[wave] = wtot;
    __syncthreads();
    int above = wtot - incl;
    for (int w = wave + 1; w < kSelWaves; ++w) above += wave_tot[w];
    if (above < remaining && remaining <= above + mine) resolve(remaining - above);
    __syncthreads();
}

// thread t owns bins 2t and 2t+1 of a 2048-bin histogram: bcast = (bin, rank inside it, its count)
__device__ __forceinline__ void bin_from_top_2048(const int *h, int rem, int *wave_tot, int *bcast)
{
    const int tid = threadIdx.x;
    const int b_lo = h[2 * tid], b_hi = h[2 * tid + 1];
    owner_from_top(b_lo + b_hi, rem, wave_tot, [&](int rank) {
        if (rank <= b_hi) { bcast[0] = 2 * tid + 1; bcast[1] = rank; bcast[2] = b_hi; }
        else { bcast[0] = 2 * tid; bcast[1] = rank - b_hi; bcast[2] = b_lo; }
    });
}

// launch 1: leading-digit histogram of every part, hist[part][1024]
__global__ __launch_bounds__(kSelThreads) void select_part_hist_kernel(const float *__restrict__ scores, const LongParts lp,
                                                                       int *__restrict__ hist)
{
    __shared__ int h[kHist1Ints];
    const int part = blockIdx.x, tid = threadIdx.x;
    PartKeys pk;
    load_part(scores + lp.begin[part], lp.len[part], pk);
#pragma unroll
    for (int i = 0; i < kHist1Ints / kSelThreads; ++i) h[i * kSelThreads + tid] = 0;
    __syncthreads();
    const uint32_t copy = tid & (kCopies - 1);
#pragma unroll
    for (int j = 0; j < kPartKpt; ++j) atomicAdd(&h[(pk.key[j] >> 22) * kCopies + copy], 1);
    __syncthreads();
    int c = 0;
#pragma unroll
    for (int i = 0; i < kCopies; ++i) c += h[tid * kCopies + i];
    hist[part * 1024 + tid] = c;
}

// launch 2: every part finds the leading digit d1 of the row's threshold from the row's part
// histograms, counts its entries above that digit and copies those with that digit to its segment
__global__ __launch_bounds__(kSelThreads) void select_part_cand_kernel(const float *__restrict__ scores, const LongParts lp,
                                                                       const int *__restrict__ hist, uint32_t *__restrict__ cand,
                                                                       int4 *__restrict__ part_rec /* (candidates, above d1, -, -) */,
                                                                       int4 *__restrict__ row_rec /* at the row's first part: (d1, rank in d1, -, -) */)
{
    __shared__ int wave_tot[kSelWaves], wave_tot2[kSelWaves], bcast[3];
    const int part = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    PartKeys pk;
    load_part(scores + lp.begin[part], lp.len[part], pk);
    const int first = lp.row_first[part], n_parts = lp.row_parts[part];
    if (tid < 3) bcast[tid] = 0;       // (always overwritten: the row holds at least k entries)
    int c = 0;
    for (int q = 0; q < n_parts; ++q) c += hist[(first + q) * 1024 + tid];
    owner_from_top(c, lp.k[part], wave_tot, [&](int rank) { bcast[0] = tid; bcast[1] = rank; });
    const uint32_t d1 = (uint32_t)bcast[0];
    int mine = 0, above = 0;
#pragma unroll
    for (int j = 0; j < kPartKpt; ++j) {
        // (an empty slot never counts: with NaN scores the threshold's digit can be the empty slots' own)
        mine += __popcll(__ballot((pk.key[j] >> 22) == d1 && pk.e0 + j * kWave < (uint32_t)lp.len[part]));
        above += __popcll(__ballot((pk.key[j] >> 22) > d1));
    }
    if (lane == 0) { wave_tot[wave] = mine; wave_tot2[wave] = above; }
    __syncthreads();
    uint32_t at = 0;
    int n_cand = 0, n_above = 0;
    for (int w = 0; w < kSelWaves; ++w) {
        if (w < wave) at += wave_tot[w];
        n_cand += wave_tot[w];
        n_above += wave_tot2[w];
    }
    uint32_t *__restrict__ seg = cand + lp.cand_off[part];
#pragma unroll
    for (int j = 0; j < kPartKpt; ++j) {
        const bool hit = (pk.key[j] >> 22) == d1 && pk.e0 + j * kWave < (uint32_t)lp.len[part];
        const uint64_t m = __ballot(hit);
        if (hit) seg[at + lanes_below(m)] = pk.key[j];
        at += __popcll(m);
    }
    if (tid == 0) {
        part_rec[part] = make_int4(n_cand, n_above, 0, 0);
        if (part == first) row_rec[part] = make_int4((int)d1, bcast[1], 0, 0);
    }
}

// launch 3: one workgroup per row (the one of the row's first part; the others leave at once)
// resolves the second and third digit on the candidates of all parts, then gives every part the
// threshold, the number of entries equal to it that the part takes (the tie goes to the lowest
// indices, i.e. to the earlier parts first) and the part's place in the output
__global__ __launch_bounds__(kSelThreads) void select_row_threshold_kernel(const LongParts lp, const uint32_t *__restrict__ cand,
                                                                           const int4 *__restrict__ part_rec, const int4 *__restrict__ row_rec,
                                                                           int4 *__restrict__ part_thr /* (T, equals taken, entries the part writes, -) */,
                                                                           long long *__restrict__ part_out)
{
    __shared__ int hist2[2048], hist3[2048];
    __shared__ int wave_tot[kSelWaves], bcast[3];
    __shared__ int cnt[kMaxParts][2];
    const int part = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1);
    if (lp.row_first[part] != part) return;             // uniform
    const int n_parts = lp.row_parts[part];
    const uint32_t d1 = (uint32_t)row_rec[part].x;
    int remaining = row_rec[part].y;
    hist2[tid] = 0; hist2[tid + kSelThreads] = 0;
    hist3[tid] = 0; hist3[tid + kSelThreads] = 0;
    if (tid < 2 * kMaxParts) (&cnt[0][0])[tid] = 0;
    if (tid < 3) bcast[tid] = 0;       // NaN scores can leave a digit without an owner: stay defined
    __syncthreads();
    for (int q = 0; q < n_parts; ++q) {
        const uint32_t *__restrict__ seg = cand + lp.cand_off[part + q];
        const int n = part_rec[part + q].x;
        for (int i = tid; i < n; i += kSelThreads) atomicAdd(&hist2[(seg[i] >> 11) & 2047u], 1);
    }
    __syncthreads();
    bin_from_top_2048(hist2, remaining, wave_tot, bcast);
    const uint32_t d2 = (uint32_t)bcast[0];
    remaining = bcast[1];
    for (int q = 0; q < n_parts; ++q) {
        const uint32_t *__restrict__ seg = cand + lp.cand_off[part + q];
        const int n = part_rec[part + q].x;
        for (int i = tid; i < n; i += kSelThreads) {
            const uint32_t key = seg[i];
            if (((key >> 11) & 2047u) == d2) atomicAdd(&hist3[key & 2047u], 1);
        }
    }
    __syncthreads();
    bin_from_top_2048(hist3, remaining, wave_tot, bcast);
    uint32_t T = (d1 << 22) | (d2 << 11) | (uint32_t)bcast[0];
    const int quota_eq = bcast[1];
    if (T == 0u) T = 1u;                                 // only reachable with NaN scores: never select padding
    for (int q = 0; q < n_parts; ++q) {
        const uint32_t *__restrict__ seg = cand + lp.cand_off[part + q];
        const int n = part_rec[part + q].x;
        int gt = 0, eq = 0;
        for (int i = tid; i < n; i += kSelThreads) {
            const uint32_t key = seg[i];
            gt += key > T;
            eq += key == T;
        }
        gt = wave_sum_i32(gt);
        eq = wave_sum_i32(eq);
        if (lane == 0) { atomicAdd(&cnt[q][0], gt); atomicAdd(&cnt[q][1], eq); }
    }
    __syncthreads();
    if (tid == 0) {
        long long at = lp.out_off[part];
        int eq_left = max(quota_eq, 0), room = lp.k[part];
        for (int q = 0; q < n_parts; ++q) {
            const int n_eq = cnt[q][1];
            const int take = min(eq_left, n_eq);
            // with well-formed scores the parts' counts add up to k exactly; the allotment keeps the
            // writes inside the row's k entries whatever NaN scores do to the counts
            const int n_out = min(part_rec[part + q].y + cnt[q][0] + take, room);
            part_thr[part + q] = make_int4((int)T, take, n_out, 0);
            part_out[part + q] = at;
            at += n_out;
            room -= n_out;
            eq_left -= take;
        }
    }
}

// launch 4: every part writes its selected entries, in index order, at its place
__global__ __launch_bounds__(kSelThreads) void select_part_write_kernel(const float *__restrict__ scores, const LongParts lp,
                                                                        const int4 *__restrict__ part_thr, const long long *__restrict__ part_out,
                                                                        int32_t *__restrict__ idx_out)
{
    __shared__ int wave_tot[kSelWaves], wave_tot2[kSelWaves];
    const int part = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    PartKeys pk;
    load_part(scores + lp.begin[part], lp.len[part], pk);
    const int4 thr = part_thr[part];
    const uint32_t T = (uint32_t)thr.x;
    const uint32_t quota_eq = (uint32_t)thr.y, n_out = (uint32_t)thr.z;
    int32_t *__restrict__ out = idx_out + part_out[part];
    const uint32_t local0 = (uint32_t)lp.local0[part];
    // entries equal to T count as selected while the part's share of the tie lasts (index order)
    int n_gt = 0, n_eq = 0;
#pragma unroll
    for (int j = 0; j < kPartKpt; ++j) {
        n_gt += __popcll(__ballot(pk.key[j] > T));
        n_eq += __popcll(__ballot(pk.key[j] == T));
    }
    if (lane == 0) { wave_tot[wave] = n_gt; wave_tot2[wave] = n_eq; }
    __syncthreads();
    uint32_t base_gt = 0, base_eq = 0;
    for (int w = 0; w < wave; ++w) { base_gt += wave_tot[w]; base_eq += wave_tot2[w]; }
#pragma unroll
    for (int j = 0; j < kPartKpt; ++j) {
        const uint32_t key = pk.key[j];
        const bool is_gt = key > T, is_eq = key == T;
        const uint64_t m_gt = __ballot(is_gt), m_eq = __ballot(is_eq);
        const uint32_t gt_before = base_gt + lanes_below(m_gt);
        const uint32_t eq_before = base_eq + lanes_below(m_eq);
        const int32_t e = (int32_t)(local0 + pk.e0 + j * kWave);
        const uint32_t slot = gt_before + min(eq_before, quota_eq);
        if ((is_gt || (is_eq && eq_before < quota_eq)) && slot < n_out) out[slot] = e;
        base_gt += __popcll(m_gt);
        base_eq += __popcll(m_eq);
    }
}

constexpr size_t sel_align(size_t x) { return (x + 255) & ~(size_t)255; }

// workspace of one group of parts holding `entries` scores
constexpr size_t long_group_bytes(int parts, int64_t entries)
{
    return sel_align(sizeof(int) * 1024 * (size_t)parts) + sel_align(sizeof(uint32_t) * (size_t)entries) +
           3 * sel_align(sizeof(int4) * (size_t)parts) + sel_align(sizeof(long long) * (size_t)parts);
}

kvs_status launch_long_group(const float *scores, const LongParts &lp, int parts, int64_t entries, int32_t *idx_out,
                             void *workspace, hipStream_t hs)
{
    char *ws = (char *)workspace;
    int *hist = (int *)ws;                  ws += sel_align(sizeof(int) * 1024 * (size_t)parts);
    uint32_t *cand = (uint32_t *)ws;        ws += sel_align(sizeof(uint32_t) * (size_t)entries);
    int4 *part_rec = (int4 *)ws;            ws += sel_align(sizeof(int4) * (size_t)parts);
    int4 *row_rec = (int4 *)ws;             ws += sel_align(sizeof(int4) * (size_t)parts);
    int4 *part_thr = (int4 *)ws;            ws += sel_align(sizeof(int4) * (size_t)parts);
    long long *part_out = (long long *)ws;
    const dim3 grid(parts), block(kSelThreads);
    kvs_status st;
    hipLaunchKernelGGL(select_part_hist_kernel, grid, block, 0, hs, scores, lp, hist);
    if ((st = check_launch("kvs_select_topk(part histograms)")) != KVS_OK) return st;
    hipLaunchKernelGGL(select_part_cand_kernel, grid, block, 0, hs, scores, lp, hist, cand, part_rec, row_rec);
    if ((st = check_launch("kvs_select_topk(part candidates)")) != KVS_OK) return st;
    hipLaunchKernelGGL(select_row_threshold_kernel, grid, block, 0, hs, lp, cand, part_rec, row_rec, part_thr, part_out);
    if ((st = check_launch("kvs_select_topk(row threshold)")) != KVS_OK) return st;
    hipLaunchKernelGGL(select_part_write_kernel, grid, block, 0, hs, scores, lp, part_thr, part_out, idx_out);
    return check_launch("kvs_select_topk(part write)");
}

} // namespace

size_t select_workspace_bytes(int32_t n_rows, int64_t n_scores)
{
    // every row may end in a short part; groups of launches reuse the same workspace one after the other
    const int64_t parts = n_scores / kPartLen + n_rows;
    const int group = (int)(parts < kMaxParts ? parts : kMaxParts);
    return long_group_bytes(group, n_scores < (int64_t)group * kPartLen ? n_scores : (int64_t)group * kPartLen) + 256;
}

// rows given as (begin, len) pairs so that callers with gaps between rows (decode contexts with
// slack) can use the same kernel; arguments are already validated.  workspace may be NULL.
kvs_status launch_select(const float *scores, int32_t n_rows, const int64_t *begin, const int64_t *len,
                         const int32_t *k_row, int32_t *idx_out, void *workspace, size_t workspace_bytes, hipStream_t hs)
{
    // a row goes the several-workgroups way if it is too long for one workgroup's registers and
    // the workspace holds it
    auto parts_of = [&](int32_t r) { return (len[r] + kPartLen - 1) / kPartLen; };
    auto is_long = [&](int32_t r) {
        return workspace && k_row[r] > 0 && len[r] > kOneWgMax && parts_of(r) <= kMaxParts &&
               long_group_bytes((int)parts_of(r), len[r]) <= workspace_bytes;
    };
    int64_t out_base = 0;
    bool any_long = false;
    for (int32_t r0 = 0; r0 < n_rows; r0 += kMaxRowsPerLaunch) {
        const int nr = (n_rows - r0) < kMaxRowsPerLaunch ? (n_rows - r0) : kMaxRowsPerLaunch;
        SelectRows rows;
        int64_t max_len = 0;
        for (int i = 0; i < kMaxRowsPerLaunch; ++i) {
            const bool live = i < nr;
            const bool lng = live && is_long(r0 + i);
            any_long |= lng;
            rows.begin[i] = live ? begin[r0 + i] : 0;
            rows.len[i] = live ? (int32_t)len[r0 + i] : 0;
            rows.k[i] = live && !lng ? k_row[r0 + i] : 0;
            rows.out_off[i] = out_base;
            if (live) {
                out_base += k_row[r0 + i];
                if (rows.k[i] > 0 && len[r0 + i] > max_len) max_len = len[r0 + i];
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
    if (!any_long) return KVS_OK;
    // the long rows, in groups of parts that share the workspace one group after the other
    LongParts lp = {};
    int parts = 0;
    int64_t entries = 0;
    out_base = 0;
    for (int32_t r = 0; r <= n_rows; ++r) {
        const bool lng = r < n_rows && is_long(r);
        const int p = lng ? (int)parts_of(r) : 0;
        if (parts > 0 && (r == n_rows || (lng && (parts + p > kMaxParts || long_group_bytes(parts + p, entries + len[r]) > workspace_bytes)))) {
            const kvs_status st = launch_long_group(scores, lp, parts, entries, idx_out, workspace, hs);
            if (st != KVS_OK) return st;
            lp = LongParts{};
            parts = 0;
            entries = 0;
        }
        if (r == n_rows) break;
        if (lng) {
            for (int q = 0; q < p; ++q) {
                const int64_t at = (int64_t)q * kPartLen;
                lp.begin[parts + q] = begin[r] + at;
                lp.len[parts + q] = (int32_t)(len[r] - at < kPartLen ? len[r] - at : kPartLen);
                lp.local0[parts + q] = (int32_t)at;
                lp.cand_off[parts + q] = entries + at;
                lp.out_off[parts + q] = out_base;
                lp.row_first[parts + q] = parts;
                lp.row_parts[parts + q] = p;
                lp.k[parts + q] = k_row[r];
            }
            parts += p;
            entries += len[r];
        }
        out_base += k_row[r];
    }
    return KVS_OK;
}

} // namespace kvs

namespace kvs {
namespace {

// ---- the scratch of kvs_select_topk_static -----------------------------------------------------------
// Device memory that belongs to the library instead of the caller: room for one group of parts of
// rows up to kStaticMaxRow scores (part histograms, candidate keys, per-part records), 4.3 MB that
// every device the library runs on holds until the process ends.  In host code the array's name
// is only a handle: the address the kernels get comes from hipGetSymbolAddress, asked once per
// device with that device current (every device has its own copy at its own address).
constexpr int64_t kStaticMaxRow = (int64_t)1 << 20;
constexpr size_t kStaticScratchBytes = long_group_bytes((int)(kStaticMaxRow / kPartLen), kStaticMaxRow);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::atomic<void *> g_scratch_ptr[kMaxDevices];

kvs_status static_scratch(void **out)
{
    const int dev = current_device();
    if (dev < 0 || dev >= kMaxDevices) return fail(KVS_EHIP, "kvs_select_topk_static: no current device, or more than %d devices", kMaxDevices);
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(KVS_EHIP, "kvs_select_topk_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return KVS_OK;
}

// ---- the scratch of kvs_deviation_topk: key histogram (zero when the library is loaded, and left
// zero by every selecting launch), the row's keys, the candidate segments and the per-part records ----
struct FusedDeviceScratch {
    uint32_t hist[kKeyHistCopies * kKeyHistBins];
    uint32_t keys[kFusedMaxTokens];
    uint32_t cand[kFusedMaxTokens];
    int2 part_rec[kFusedMaxParts];
    FusedRow row_rec;
};
static __device__ __align__(256) FusedDeviceScratch fused_mem;
std::atomic<FusedDeviceScratch *> g_fused_mem[kMaxDevices];

} // namespace

kvs_status fused_scratch(FusedScratch *out)
{
    const int dev = current_device();
    if (dev < 0 || dev >= kMaxDevices) return fail(KVS_EHIP, "kvs_deviation_topk: no current device, or more than %d devices", kMaxDevices);
    FusedDeviceScratch *m = g_fused_mem[dev].load(std::memory_order_acquire);
    if (!m) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(fused_mem));
        if (e != hipSuccess || !p) return fail(KVS_EHIP, "kvs_deviation_topk: hipGetSymbolAddress: %s", hipGetErrorString(e));
        m = (FusedDeviceScratch *)p;
        g_fused_mem[dev].store(m, std::memory_order_release);
    }
    out->hist = m->hist;
    out->keys = m->keys;
    out->mem = m;
    return KVS_OK;
}

kvs_status launch_select_from_hist(const FusedScratch &fs, int32_t n, int32_t k, int32_t *idx_out, hipStream_t hs)
{
    if (n > kFusedMaxTokens) return fail(KVS_EINVAL, "kvs_deviation_topk: %d tokens are more than the library's key scratch holds", n);
    FusedDeviceScratch *m = (FusedDeviceScratch *)fs.mem;
    const int parts = (n + kFuPart - 1) / kFuPart;
    static_assert(kFusedMaxParts <= kFuThreads && kFusedMaxParts * kFuPart == kFusedMaxTokens, "one thread per part in the prefix sums");
    hipLaunchKernelGGL(fused_cand_kernel, dim3(parts), dim3(kFuThreads), 0, hs, m->keys, m->hist, n, k, m->cand, m->part_rec, &m->row_rec);
    kvs_status st = check_launch("kvs_deviation_topk(candidates)");
    if (st != KVS_OK) return st;
    hipLaunchKernelGGL(fused_write_kernel, dim3(parts), dim3(kFuThreads), 0, hs, m->keys, m->hist, n, k, parts, m->cand, m->part_rec,
                       &m->row_rec, idx_out);
    return check_launch("kvs_deviation_topk(write)");
}

namespace {
} // namespace
} // namespace kvs

extern "C" kvs_status kvs_select_topk_static(const float *scores, int32_t n_rows, const int64_t *row_off,
                                             const int32_t *k_row, int32_t *idx_out, void *stream)
{
    using namespace kvs;
    // the address is looked up before anything else, so a call with n_rows = 0 is a way to get the
    // one-time lookup done (outside a stream capture, say) without launching anything
    void *ws = nullptr;
    const kvs_status st = static_scratch(&ws);
    if (st != KVS_OK) return st;
    if (n_rows > 0 && row_off)
        for (int32_t r = 0; r < n_rows; ++r)
            if (row_off[r + 1] - row_off[r] > kStaticMaxRow)
                return fail(KVS_EINVAL, "kvs_select_topk_static: row %d has %lld scores, the library's own scratch holds rows up to %lld",
                            r, (long long)(row_off[r + 1] - row_off[r]), (long long)kStaticMaxRow);
    return kvs_select_topk(scores, n_rows, row_off, k_row, idx_out, ws, kStaticScratchBytes, stream);
}

extern "C" kvs_status kvs_select_topk(const float *scores, int32_t n_rows, const int64_t *row_off,
                                      const int32_t *k_row, int32_t *idx_out,
                                      void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace kvs;
    if (n_rows < 0) return fail(KVS_EINVAL, "kvs_select_topk: n_rows < 0");
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return fail(KVS_EINVAL, "kvs_select_topk: workspace must be 256-byte aligned");
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
    // (begin, len) view of the packed rows, a stack table of 256 rows at a time (no host allocation)
    constexpr int kStack = 256;
    int64_t lens[kStack];
    int64_t out_base = 0;
    for (int32_t r0 = 0; r0 < n_rows; r0 += kStack) {
        const int32_t nr = n_rows - r0 < kStack ? n_rows - r0 : kStack;
        int64_t k_here = 0;
        for (int32_t r = 0; r < nr; ++r) {
            lens[r] = row_off[r0 + r + 1] - row_off[r0 + r];
            k_here += k_row[r0 + r];
        }
        if (k_here > 0) {
            const kvs_status st = launch_select(scores, nr, row_off + r0, lens, k_row + r0, idx_out + out_base, workspace,
                                                workspace_bytes, (hipStream_t)stream);
            if (st != KVS_OK) return st;
        }
        out_base += k_here;
    }
    return KVS_OK;
}
