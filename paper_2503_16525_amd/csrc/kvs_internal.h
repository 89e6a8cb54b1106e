// Internal helpers shared by the HIP translation units of libkvshare_hip.so.
// Nothing here is part of the ABI (see include/kvs.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include <atomic>

#include "kvs.h"

namespace kvs {

// thread-local error text behind kvs_last_error()
void set_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));
kvs_status fail(kvs_status st, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
kvs_status check_launch(const char *what);

inline size_t elem_bytes(int32_t dtype) { return dtype == KVS_F32 ? 4 : 2; }

// Validates a kvs_shape for the kernels that exist; on failure the status says why.
kvs_status check_shape(const kvs_shape *s);

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// One-time set-up per device (kernel attributes, device queries).  The HIP runtime keeps function
// attributes per device, so the "done" flag is per device as well.  The set-up calls are idempotent:
// two host threads that race through one only repeat the same calls, and the flag is published
// with release/acquire ordering.  Devices past the table simply repeat the set-up on every call.
constexpr int kMaxDevices = 64;
struct DeviceOnce {
    std::atomic<int> done[kMaxDevices];
};
inline int current_device()
{
    int dev = -1;
    return hipGetDevice(&dev) == hipSuccess ? dev : -1;
}
template <typename F>
inline kvs_status once_per_device(DeviceOnce &once, F setup)
{
    const int dev = current_device();
    const bool tracked = dev >= 0 && dev < kMaxDevices;
    if (tracked && once.done[dev].load(std::memory_order_acquire)) return KVS_OK;
    const kvs_status st = setup();
    if (st == KVS_OK && tracked) once.done[dev].store(1, std::memory_order_release);
    return st;
}

// exact top-k over rows given as (begin, len) pairs of one score array (select.hip); the workspace
// (may be NULL) lets rows too long for one workgroup spread over several
kvs_status launch_select(const float *scores, int32_t n_rows, const int64_t *begin, const int64_t *len,
                         const int32_t *k_row, int32_t *idx_out, void *workspace, size_t workspace_bytes, hipStream_t stream);
size_t select_workspace_bytes(int32_t n_rows, int64_t n_scores);
size_t decode_workspace_bytes(const kvs_shape *shape, int32_t batch, int64_t n_rows);
size_t colsum_workspace_bytes(const kvs_shape *shape, int64_t n_tokens);
size_t impact_workspace_bytes(const kvs_shape *shape, int64_t n_tokens);
size_t match_workspace_bytes(int64_t n_target, int64_t n_candidate);
kvs_status launch_colsum_valu(const kvs_shape *shape, int64_t n, const void *q, const void *k, float scale,
                              float *lse, float *alpha, hipStream_t st);

// ---- deviation scoring and top-k in one call (kvs_deviation_topk) ----------------------------------
// The scoring kernel leaves, beside the scores, every token's order-preserving key and a histogram
// of the keys' leading kKeyHistBits bits (device-scope integer atomics: the counts do not depend
// on the order in which they arrive); two short launches of one workgroup per 1024 keys then find
// the k-th key from the histogram and write the index list.  Keys, histogram and the records the
// two launches exchange live in device memory that belongs to the library.
constexpr int kKeyHistBits = 13;
constexpr int kKeyHistBins = 1 << kKeyHistBits;
constexpr int kKeyHistShift = 32 - kKeyHistBits;
constexpr int kFusedMaxParts = 256;              // selecting workgroups per row, 1024 keys each
constexpr int kFusedMaxTokens = kFusedMaxParts * 1024;
constexpr int kFusedMinTokens = 12 * 1024;       // up to here kvs_deviation_topk runs as the two separate calls
struct FusedScratch {
    uint32_t *hist;   // [kKeyHistCopies][kKeyHistBins], all zero between calls (the selecting launch clears what it read)
    uint32_t *keys;   // [kFusedMaxTokens]
    void *mem;        // the whole scratch block (select.hip)
};
kvs_status fused_scratch(FusedScratch *out);
// where the counter of leading-bits value `bin` lives in the histogram: neighbouring bins are kept
// 64 counters (256 bytes) apart, which spreads the few dozen bins that one launch's scores fall
// into over the memory channels.  Measured on the 32k layer, time of the scoring kernel: no
// histogram 22.9 us; bins side by side 47 us; 64 bytes apart 29 us; 128 to 512 bytes apart 25.5 us;
// 1 KiB apart 30 us; 2 KiB apart 33 us.  Several copies of the histogram (a scoring workgroup adding
// to copy = its index mod the copies, so that fewer atomics meet at one address) were slower: 2
// copies +5 us, 4 copies +16 us on the whole call.
constexpr int kKeyHistCopies = 1;
__host__ __device__ constexpr uint32_t key_hist_slot(uint32_t bin) { return ((bin & 127u) << 6) | (bin >> 7); }
static_assert(kKeyHistBits == 13, "the slot map is written for 8192 bins");
static_assert(kKeyHistCopies == 1, "key_hist_count adds to the one histogram");
kvs_status launch_select_from_hist(const FusedScratch &fs, int32_t n, int32_t k, int32_t *idx_out, hipStream_t stream);

constexpr int kWave = 64;

// monotone map fp32 -> uint32 (larger score <=> larger key); -0 is first folded onto +0.  Real
// scores never map below 2^22 (-inf maps to 0x007fffff; only NaN patterns go lower).
__device__ __forceinline__ uint32_t score_key(float s)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, s + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
constexpr uint32_t kKeyNegInf = 0x007fffffu;

// Counts the keys of the lanes that are active here and pass `counted` into the leading-bits histogram.
// Integer counts: the histogram does not depend on the order in which the atomics land.
// PER_BIN: one atomic per distinct bin of the wavefront instead of one per lane.  The scores of neighbouring
// tokens fall into a dozen bins or so and the memory side executes atomics to one address one after the
// other; measured, the grouping takes the decode scoring launch from 15.5 to ~10 us (a wave there has 64
// tokens and nothing else to do), but makes kvs_deviation_topk 1.7 us slower: its scoring workgroups stream
// V and their 32-token epilogue is short, so a serial loop over bins at the end of every workgroup costs
// more than the atomics it saves (2.7 us for the per-lane add).
template <bool PER_BIN>
__device__ __forceinline__ void key_hist_count(uint32_t *__restrict__ key_hist, uint32_t key, bool counted)
{
    const uint32_t bin = key >> kKeyHistShift;
    if (!PER_BIN) {
        if (counted) __hip_atomic_fetch_add(key_hist + key_hist_slot(bin), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    const int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    unsigned long long todo = __ballot(counted);
    while (todo) {                                             // uniform over the active lanes
        const int leader = __ffsll((long long)todo) - 1;
        const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader);
        const unsigned long long same = __ballot(counted && bin == b);
        if (lane == leader)
            __hip_atomic_fetch_add(key_hist + key_hist_slot(b), (uint32_t)__popcll(same), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        todo &= ~same;
    }
}

// ---- wavefront primitives (64 lanes) ------------------------------------------------------

// value of `v` taken from the lane `ctrl` selects inside the same 16-lane row (DPP)
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
        0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}

// sum over each aligned group of 16 lanes, result in every lane of the group; fixed order
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_f32<0x128>(v); // row_ror:8
    v += dpp_f32<0x124>(v); // row_ror:4
    v += dpp_f32<0x122>(v); // row_ror:2
    v += dpp_f32<0x121>(v); // row_ror:1
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
    v = row16_sum(v);
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_f32<0x128>(v));
    v = fmaxf(v, dpp_f32<0x124>(v));
    v = fmaxf(v, dpp_f32<0x122>(v));
    v = fmaxf(v, dpp_f32<0x121>(v));
    v = fmaxf(v, __shfl_xor(v, 16));
    v = fmaxf(v, __shfl_xor(v, 32));
    return v;
}

__device__ __forceinline__ int wave_sum_i32(int v)
{
    v += dpp_i32<0x128>(v);
    v += dpp_i32<0x124>(v);
    v += dpp_i32<0x122>(v);
    v += dpp_i32<0x121>(v);
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

// 16-byte streaming (non-temporal) load: data that is read once should not displace reusable lines
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 stream_load16(const uint4 *p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// exact bf16 -> fp32 widening of the two halves of a packed pair
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16, round to nearest even (finite inputs; NaN keeps a quiet pattern)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

} // namespace kvs
