// kvs_match_tokens: the KV Retriever's token-sequence matching (Sec. 5.1; App. E Alg. 3, Eq. (7)).
//
// The algorithm as stated is a sequential scan: candidate windows in ascending order j, for each the
// target windows i with the same hash in ascending order, each (i, j) extended token by token, a
// target position recorded the first time it is reached.  What it ends with does not depend on the
// scan, only on its order: target position p belongs to the smallest (j, i), in lexicographic order,
// among the pairs of equal-hash window starts whose stretch of equal tokens from (i, j) reaches p;
// its partner is j + p - i; and the output lists the pairs by (j, i, p).  That statement is what
// runs here, in parallel:
//
//   1. match_hash_kernel    Eq. (7) for every window of both sequences, each from its own w tokens
//                           (Horner; nothing rolls, so no carried state between threads); clears the
//                           tables.
//   2. match_insert_kernel  a chained hash table over the target's window hashes (one atomic
//                           exchange per window; the order inside a chain does not matter below).
//   3. match_seed_kernel    a lane per candidate window walks its chain.  A pair (i, j) whose
//                           predecessor (i-1, j-1) is an equal-hash pair with equal tokens is skipped:
//                           the predecessor reaches everything (i, j) reaches and comes earlier in
//                           the order.  Each remaining pair is extended by its whole wavefront, 1024
//                           positions per trip, and claims the positions it reaches with a 64-bit
//                           atomic minimum on (j, i).  A stretch of R equal tokens costs R atomics
//                           instead of the scan's R^2 / 2 comparisons.
//   4. match_mark_kernel    partner of every target position; counts the maximal stretches of
//                           positions with the same (j, i) per block of 1024 positions.
//   5. match_segments_kernel  numbers the stretches in position order (start, end, key).
//   6. match_order_kernel   a wavefront per stretch adds up the lengths of the stretches that come
//                           before it in (j, i, start) order and writes its pairs there: the lists
//                           come out in the scan's order of discovery.
//
// Cost: reading both sequences a few times plus one atomic per matched position; the stretches are
// few (tens to hundreds for a prompt assembled from earlier requests), so step 6's all-pairs count
// is small.  Worst cases are bounded, not fast: sequences of one repeated token make every pair of
// windows an equal-hash pair (n_target x n_candidate chain steps), and a target whose matched
// positions alternate makes n_target / 2 stretches (step 6 is quadratic in them).
#include "kvs_internal.h"

namespace kvs {
namespace {

constexpr int kMatchThreads = 256;
constexpr int kMatchChunk = 1024;          // target positions per workgroup in steps 4 and 5
constexpr uint64_t kNoMatch = ~0ull;

struct MatchWs {
    uint32_t *ht;          // [n_target]    window hashes of the target (first n_target - w + 1 used)
    uint32_t *hc;          // [n_candidate] window hashes of the candidate
    int32_t *head;         // [table]       first target window of each slot's chain, -1: none
    int32_t *next;         // [n_target]    next target window of the same slot
    uint64_t *best;        // [n_target]    smallest (j << 32 | i) that reaches the position
    uint32_t *chunk_count; // [chunks]      stretches that start in each block of kMatchChunk positions
    int32_t *seg_start;    // [n_target]    stretch s covers positions seg_start[s] .. seg_end[s]-1
    int32_t *seg_end;
    uint64_t *seg_key;     // [n_target]
    uint32_t *counters;    // [0] matched positions, [1] stretches
};

__host__ __device__ inline int64_t round256(int64_t x) { return (x + 255) & ~(int64_t)255; }

inline int table_bits(int64_t windows)
{
    int bits = 6;
    while (((int64_t)1 << bits) < 2 * windows) ++bits;
    return bits;
}

inline size_t carve(MatchWs *ws, char *base, int64_t n_t, int64_t n_c, int bits)
{
    const int64_t chunks = (n_t + kMatchChunk - 1) / kMatchChunk;
    int64_t off = 0;
    auto take = [&](int64_t bytes) { char *p = base ? base + off : nullptr; off += round256(bytes); return p; };
    char *best = take(8 * n_t), *seg_key = take(8 * n_t);
    char *ht = take(4 * n_t), *hc = take(4 * n_c), *head = take(4 * ((int64_t)1 << bits)), *next = take(4 * n_t);
    char *cc = take(4 * chunks), *ss = take(4 * n_t), *se = take(4 * n_t), *ct = take(256);
    if (ws) {
        ws->best = (uint64_t *)best; ws->seg_key = (uint64_t *)seg_key;
        ws->ht = (uint32_t *)ht; ws->hc = (uint32_t *)hc; ws->head = (int32_t *)head; ws->next = (int32_t *)next;
        ws->chunk_count = (uint32_t *)cc; ws->seg_start = (int32_t *)ss; ws->seg_end = (int32_t *)se; ws->counters = (uint32_t *)ct;
    }
    return (size_t)off;
}

// x mod m for any 64-bit x without a division: with r = floor((2^64 - 1) / m), the estimate
// q = floor(x r / 2^64) falls short of floor(x / m) by at most 2, so two conditional subtractions finish.
// (q <= x/m because r <= 2^64/m; and x/m - q < x (2^64/m - r) / 2^64 + 1 <= x (1 + 1/m) / 2^64 + 1 < 3.)
struct Modulus {
    uint64_t m, r;
};
__device__ __forceinline__ uint64_t reduce(uint64_t x, const Modulus &md)
{
    uint64_t rem = x - __umul64hi(x, md.r) * md.m;
    rem = rem >= md.m ? rem - md.m : rem;
    rem = rem >= md.m ? rem - md.m : rem;
    return rem;
}
template <typename Tokens>
__device__ __forceinline__ uint32_t window_hash(Tokens tok, int64_t i, int w, uint32_t b, const Modulus &md)
{
    uint64_t h = 0;
    for (int x = 0; x < w; ++x) h = reduce(h * (uint64_t)b + (uint64_t)(uint32_t)tok[i + x], md);   // h < m < 2^32: no overflow
    return (uint32_t)h;
}
__device__ __forceinline__ uint32_t slot_of(uint32_t h, int bits) { return (h * 2654435761u) >> (32 - bits); }

// Windows up to this long are hashed out of LDS: a workgroup's 256 windows overlap in all but 255
// tokens, and a Horner chain over global memory would pay one memory latency per token.
constexpr int kHashLdsWindow = 768;

// hashes of the windows that start at base .. base+255 (those below n_windows) of one sequence
__device__ __forceinline__ void hash_block(const int32_t *__restrict__ tok, int64_t n, int64_t n_windows, int64_t base, int w, uint32_t b,
                                           const Modulus &md, int32_t *tile, uint32_t *__restrict__ out)
{
    const int64_t i = base + threadIdx.x;
    if (w <= kHashLdsWindow) {
        const int64_t span = min((int64_t)kMatchThreads + w - 1, n - base);
        __syncthreads();                                   // the tile's previous readers are done
        for (int64_t x = threadIdx.x; x < span; x += kMatchThreads) tile[x] = tok[base + x];
        __syncthreads();
        if (i < n_windows) out[i] = window_hash(tile, (int64_t)threadIdx.x, w, b, md);
    } else if (i < n_windows) {
        out[i] = window_hash(tok, i, w, b, md);
    }
}

__global__ __launch_bounds__(kMatchThreads) void match_hash_kernel(
    const int32_t *__restrict__ target, int64_t n_t, const int32_t *__restrict__ cand, int64_t n_c,
    int w, uint32_t b, Modulus md, int bits, MatchWs ws)
{
    __shared__ int32_t tile[kMatchThreads + kHashLdsWindow];
    const int64_t tid = (int64_t)blockIdx.x * kMatchThreads + threadIdx.x, nth = (int64_t)gridDim.x * kMatchThreads;
    const int64_t wt = n_t - w + 1, wc = n_c - w + 1, table = (int64_t)1 << bits;
    for (int64_t i = tid; i < n_t; i += nth) ws.best[i] = kNoMatch;
    for (int64_t s = tid; s < table; s += nth) ws.head[s] = -1;
    if (tid < 4) ws.counters[tid] = 0u;
    // the first blocks_t workgroups hash the target's windows, the others the candidate's (one block of
    // 256 windows each; every thread of a workgroup takes part in staging its block's tokens)
    const int64_t blocks_t = (wt + kMatchThreads - 1) / kMatchThreads;
    if ((int64_t)blockIdx.x < blocks_t) hash_block(target, n_t, wt, (int64_t)blockIdx.x * kMatchThreads, w, b, md, tile, ws.ht);
    else hash_block(cand, n_c, wc, ((int64_t)blockIdx.x - blocks_t) * kMatchThreads, w, b, md, tile, ws.hc);
}

__global__ __launch_bounds__(kMatchThreads) void match_insert_kernel(int64_t wt, int bits, MatchWs ws)
{
    const int64_t i = (int64_t)blockIdx.x * kMatchThreads + threadIdx.x;
    if (i >= wt) return;
    ws.next[i] = atomicExch(&ws.head[slot_of(ws.ht[i], bits)], (int32_t)i);
}

// the whole wavefront extends the pair of window starts (i, j): positions i+k while both sequences
// last and the tokens agree; each reached position keeps the smallest key.  Ends at the first
// disagreement or at the end of a sequence, whichever comes first.  A trip compares 1024 positions,
// all of its loads in flight together: the loop pays one memory latency per trip, and the
// atomics return nothing to wait for.
constexpr int kClaimUnroll = 16;
__device__ __forceinline__ void claim_stretch(const int32_t *__restrict__ target, int64_t n_t, const int32_t *__restrict__ cand,
                                              int64_t n_c, int32_t i, int32_t j, uint64_t *__restrict__ best, int lane)
{
    const uint64_t key = ((uint64_t)(uint32_t)j << 32) | (uint32_t)i;
    const int64_t room = min(n_t - i, n_c - j);
    for (int64_t k0 = 0; k0 < room; k0 += kClaimUnroll * kWave) {
        int32_t a[kClaimUnroll], c[kClaimUnroll];
#pragma unroll
        for (int u = 0; u < kClaimUnroll; ++u) {
            const int64_t k = min(k0 + u * kWave + lane, room - 1);     // clamped: every load is inside both sequences
            a[u] = target[i + k];
            c[u] = cand[j + k];
        }
        bool open = true;                       // uniform: no disagreement so far in this trip
#pragma unroll
        for (int u = 0; u < kClaimUnroll; ++u) {
            const int64_t k = k0 + u * kWave + lane;
            const unsigned long long agree = __ballot(k < room && a[u] == c[u]);
            const int first_bad = ~agree ? __ffsll((long long)~agree) - 1 : kWave;
            if (open && lane < first_bad) atomicMin((unsigned long long *)&best[i + k], (unsigned long long)key);
            open = open && first_bad == kWave;
        }
        if (!open) break;
    }
}

__global__ __launch_bounds__(kMatchThreads) void match_seed_kernel(
    const int32_t *__restrict__ target, int64_t n_t, const int32_t *__restrict__ cand, int64_t n_c,
    int w, int bits, MatchWs ws)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wc = n_c - w + 1;
    const int64_t j = (int64_t)blockIdx.x * kMatchThreads + threadIdx.x;
    const bool live = j < wc;
    const uint32_t hj = live ? ws.hc[j] : 0u;
    // what the predecessor test needs from the candidate's side
    const bool has_prev = live && j > 0;
    const uint32_t hj_prev = has_prev ? ws.hc[j - 1] : 0u;
    const int32_t tok_prev = has_prev ? cand[j - 1] : -1;
    int32_t cur = live ? ws.head[slot_of(hj, bits)] : -1;
    while (__any(cur >= 0)) {
        // everything one chain step needs, requested together: one memory latency per step
        const bool on = cur >= 0;
        const int32_t prev = on && cur > 0 ? cur - 1 : 0;
        const uint32_t h_cur = on ? ws.ht[cur] : 0u;
        const uint32_t h_before = on ? ws.ht[prev] : 0u;
        const int32_t tok_before = on ? target[prev] : -1;
        const int32_t nxt = on ? ws.next[cur] : -1;
        bool first_of_its_stretch = false;
        if (on && h_cur == hj) {
            const bool shadowed = has_prev && cur > 0 && h_before == hj_prev && tok_before == tok_prev;
            first_of_its_stretch = !shadowed;
        }
        unsigned long long todo = __ballot(first_of_its_stretch);
        while (todo) {                                  // uniform
            const int src = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            const int32_t si = __builtin_amdgcn_readlane(cur, src);
            const int32_t sj = (int32_t)(j - lane + src);
            claim_stretch(target, n_t, cand, n_c, si, sj, ws.best, lane);
        }
        cur = nxt;
    }
}

// flags of the four consecutive positions a thread owns in steps 4 and 5
struct Flags {
    uint64_t key[4];
    bool start[4], end[4];
};
__device__ __forceinline__ Flags read_flags(const uint64_t *__restrict__ best, int64_t p0, int64_t n_t)
{
    Flags f;
    uint64_t before = p0 > 0 && p0 - 1 < n_t ? best[p0 - 1] : kNoMatch;
    uint64_t k[5];
#pragma unroll
    for (int u = 0; u < 5; ++u) k[u] = p0 + u < n_t ? best[p0 + u] : kNoMatch;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        f.key[u] = k[u];
        const bool matched = k[u] != kNoMatch;          // positions past the end read as unmatched
        f.start[u] = matched && (u == 0 ? before : k[u - 1]) != k[u];
        f.end[u] = matched && k[u + 1] != k[u];
    }
    return f;
}

__global__ __launch_bounds__(kMatchThreads) void match_mark_kernel(int64_t n_t, int32_t *__restrict__ match_cand, MatchWs ws)
{
    __shared__ uint32_t tot[2];
    if (threadIdx.x < 2) tot[threadIdx.x] = 0u;
    __syncthreads();
    const int64_t p0 = (int64_t)blockIdx.x * kMatchChunk + 4 * threadIdx.x;
    const Flags f = read_flags(ws.best, p0, n_t);
    uint32_t starts = 0, matched = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        if (p0 + u < n_t) {
            const bool mt = f.key[u] != kNoMatch;
            const int32_t j = (int32_t)(f.key[u] >> 32), i = (int32_t)(uint32_t)f.key[u];
            match_cand[p0 + u] = mt ? j + (int32_t)(p0 + u - i) : -1;
            matched += mt ? 1u : 0u;
            starts += f.start[u] ? 1u : 0u;
        }
    }
    // workgroup totals: wavefront sums, then one LDS atomic per wavefront
    for (int o = 32; o > 0; o >>= 1) { starts += __shfl_xor(starts, o); matched += __shfl_xor(matched, o); }
    if ((threadIdx.x & (kWave - 1)) == 0) { atomicAdd(&tot[0], starts); atomicAdd(&tot[1], matched); }
    __syncthreads();
    if (threadIdx.x == 0) {
        ws.chunk_count[blockIdx.x] = tot[0];
        if (tot[1]) atomicAdd(&ws.counters[0], tot[1]);
    }
}

__global__ __launch_bounds__(kMatchThreads) void match_segments_kernel(int64_t n_t, MatchWs ws)
{
    __shared__ uint32_t wave_tot[kMatchThreads / kWave];
    __shared__ uint32_t base_sh;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    // stretches that start in the blocks before this one
    uint32_t before = 0;
    for (int64_t c = threadIdx.x; c < (int64_t)blockIdx.x; c += kMatchThreads) before += ws.chunk_count[c];
    for (int o = 32; o > 0; o >>= 1) before += __shfl_xor(before, o);
    if (lane == 0) wave_tot[wave] = before;
    __syncthreads();
    if (threadIdx.x == 0) base_sh = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
    __syncthreads();
    const uint32_t base = base_sh;
    __syncthreads();
    const int64_t p0 = (int64_t)blockIdx.x * kMatchChunk + 4 * threadIdx.x;
    const Flags f = read_flags(ws.best, p0, n_t);
    uint32_t mine = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) mine += f.start[u] ? 1u : 0u;
    // exclusive scan over the workgroup in thread order
    uint32_t incl = mine;
    for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
    }
    if (lane == kWave - 1) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t run = base + incl - mine;
    for (int v = 0; v < wave; ++v) run += wave_tot[v];
    // run = stretches that start before this thread's first position; a position's stretch is the
    // last one that started at or before it
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        if (f.start[u]) {
            ws.seg_start[run] = (int32_t)(p0 + u);
            ws.seg_key[run] = f.key[u];
            ++run;
        }
        if (f.end[u]) ws.seg_end[run - 1] = (int32_t)(p0 + u + 1);
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == kMatchThreads - 1) ws.counters[1] = run;
}

__global__ __launch_bounds__(kMatchThreads) void match_order_kernel(int32_t *__restrict__ target_matches, int32_t *__restrict__ cand_matches,
                                                                    int64_t *__restrict__ n_matches, MatchWs ws)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = ((int64_t)blockIdx.x * kMatchThreads + threadIdx.x) >> 6, n_waves = ((int64_t)gridDim.x * kMatchThreads) >> 6;
    if (wave == 0 && lane == 0 && n_matches) *n_matches = (int64_t)ws.counters[0];
    if (!target_matches && !cand_matches) return;
    const int64_t n_seg = ws.counters[1];
    for (int64_t s = wave; s < n_seg; s += n_waves) {
        const uint64_t key = ws.seg_key[s];
        const int32_t start = ws.seg_start[s], len = ws.seg_end[s] - start;
        uint32_t offset = 0;
        for (int64_t o = lane; o < n_seg; o += kWave) {
            const uint64_t ko = ws.seg_key[o];
            const int32_t so = ws.seg_start[o];
            if (ko < key || (ko == key && so < start)) offset += (uint32_t)(ws.seg_end[o] - so);
        }
        for (int x = 32; x > 0; x >>= 1) offset += __shfl_xor(offset, x);
        const int32_t j = (int32_t)(key >> 32), i = (int32_t)(uint32_t)key;
        for (int32_t t = lane; t < len; t += kWave) {
            if (target_matches) target_matches[offset + t] = start + t;
            if (cand_matches) cand_matches[offset + t] = j + (start + t - i);
        }
    }
}

__global__ void match_none_kernel(int64_t n_t, int32_t *__restrict__ match_cand, int64_t *__restrict__ n_matches)
{
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid < n_t && match_cand) match_cand[tid] = -1;
    if (tid == 0 && n_matches) *n_matches = 0;
}

constexpr int64_t kMatchMaxTokens = (int64_t)1 << 26;

} // namespace

size_t match_workspace_bytes(int64_t n_target, int64_t n_candidate)
{
    if (n_target <= 0 || n_candidate <= 0 || n_target > kMatchMaxTokens || n_candidate > kMatchMaxTokens) return 256;
    return carve(nullptr, nullptr, n_target, n_candidate, table_bits(n_target));
}

} // namespace kvs

extern "C" kvs_status kvs_match_tokens(const int32_t *target, int64_t n_target, const int32_t *candidate, int64_t n_candidate,
                                       int32_t window, uint32_t hash_base, uint32_t hash_modulus,
                                       int32_t *match_cand, int32_t *target_matches, int32_t *candidate_matches,
                                       int64_t *n_matches, void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace kvs;
    if (n_target < 0 || n_candidate < 0) return fail(KVS_EINVAL, "kvs_match_tokens: negative length");
    if (window <= 0) return fail(KVS_EINVAL, "kvs_match_tokens: window %d", window);
    if (hash_modulus == 0) return fail(KVS_EINVAL, "kvs_match_tokens: modulus 0");
    if (n_target > kMatchMaxTokens || n_candidate > kMatchMaxTokens)
        return fail(KVS_EUNSUPPORTED, "kvs_match_tokens: sequences of more than %lld tokens", (long long)kMatchMaxTokens);
    if (!n_matches) return fail(KVS_EINVAL, "kvs_match_tokens: n_matches is NULL");
    if (n_target > 0 && (!target || !match_cand)) return fail(KVS_EINVAL, "kvs_match_tokens: NULL target or match_cand");
    if (n_candidate > 0 && !candidate) return fail(KVS_EINVAL, "kvs_match_tokens: NULL candidate");
    hipStream_t hs = (hipStream_t)stream;
    const int64_t wt = n_target - window + 1, wc = n_candidate - window + 1;
    if (wt <= 0 || wc <= 0) {        // no window fits one of the sequences: nothing can match
        const unsigned blocks = (unsigned)((n_target + 255) / 256);
        hipLaunchKernelGGL(match_none_kernel, dim3(blocks ? blocks : 1u), dim3(256), 0, hs, n_target, match_cand, n_matches);
        return check_launch("kvs_match_tokens");
    }
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return fail(KVS_EINVAL, "kvs_match_tokens: workspace must be a 256-byte aligned device buffer");
    const int bits = table_bits(n_target);
    MatchWs ws;
    const size_t need = carve(&ws, (char *)workspace, n_target, n_candidate, bits);
    if (workspace_bytes < need) return fail(KVS_EWORKSPACE, "kvs_match_tokens: workspace of %zu bytes, %zu needed", workspace_bytes, need);
    const Modulus md = {(uint64_t)hash_modulus, ~0ull / (uint64_t)hash_modulus};
    const unsigned hash_blocks = (unsigned)((wt + kMatchThreads - 1) / kMatchThreads + (wc + kMatchThreads - 1) / kMatchThreads);
    hipLaunchKernelGGL(match_hash_kernel, dim3(hash_blocks), dim3(kMatchThreads), 0, hs, target, n_target, candidate, n_candidate,
                       (int)window, hash_base, md, bits, ws);
    hipLaunchKernelGGL(match_insert_kernel, dim3((unsigned)((wt + kMatchThreads - 1) / kMatchThreads)), dim3(kMatchThreads), 0, hs, wt, bits, ws);
    hipLaunchKernelGGL(match_seed_kernel, dim3((unsigned)((wc + kMatchThreads - 1) / kMatchThreads)), dim3(kMatchThreads), 0, hs,
                       target, n_target, candidate, n_candidate, (int)window, bits, ws);
    const unsigned chunks = (unsigned)((n_target + kMatchChunk - 1) / kMatchChunk);
    hipLaunchKernelGGL(match_mark_kernel, dim3(chunks), dim3(kMatchThreads), 0, hs, n_target, match_cand, ws);
    const bool lists = target_matches || candidate_matches;
    if (lists) hipLaunchKernelGGL(match_segments_kernel, dim3(chunks), dim3(kMatchThreads), 0, hs, n_target, ws);
    hipLaunchKernelGGL(match_order_kernel, dim3(lists ? 256u : 1u), dim3(kMatchThreads), 0, hs, target_matches, candidate_matches, n_matches, ws);
    return check_launch("kvs_match_tokens");
}
