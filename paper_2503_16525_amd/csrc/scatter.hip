// kvs_scatter_kv: the KV Writer step -- rows of freshly recomputed K/V overwrite the reused
// entries of the cache at the selected positions.  A pure copy, and a small one (tens of MB): a
// wavefront takes 8 KiB of selected rows, reads their positions and issues every 16-byte load of
// those rows (K and V) before the first store, so the index load and the data loads are in flight
// together and only the stores wait for both.  Consecutive lanes move consecutive pieces of a
// row, so the gather side (dense k_new / v_new) and the scatter side (whole cache rows of >= 512
// bytes) are both coalesced.  The new rows are read once (streaming loads); the cache rows are
// stored normally: the attention that follows reads them.
//
// Measured on the 32k layer (cold buffers, kernel time): 5.7 / 9.1 / 15.5 us for 12 / 36 / 72 MB,
// i.e. about 3.7 us that do not depend on the size (launch, one round trip for the loads, the
// drain of the stores) plus the bytes at 6.2 TB/s.  One, two or four rows per wavefront and
// non-temporal stores all land within 10 % of each other; the first version (one piece per lane
// behind its own index load) was no slower than four rows per wavefront.
#include "kvs_internal.h"

namespace kvs {
namespace {

constexpr int kScatThreads = 256;
constexpr int kScatWaves = kScatThreads / kWave;
// PPL: 16-byte pieces of a row per lane (row bytes / 1024, rounded up); kRows: selected rows per
// wavefront, 8 KiB of K and V together for rows up to 2 KiB
template <int PPL, int kRows>
__global__ __launch_bounds__(kScatThreads) void scatter_kernel(
    int64_t n_rows, int64_t n_sel, int pieces_per_row, int n_kv_heads,
    const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new,
    const int32_t *__restrict__ sel_pos,
    uint4 *__restrict__ k_cache, uint4 *__restrict__ v_cache,
    uint8_t *__restrict__ reused, float *__restrict__ dev_v)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = (int64_t)blockIdx.x * kScatWaves + (threadIdx.x >> 6);
    const int64_t s0 = wave * kRows;
    if (s0 >= n_sel) return;
    int64_t pos[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const int64_t s = s0 + r < n_sel ? s0 + r : n_sel - 1;     // (the last wavefront repeats its last row: same bytes twice)
        pos[r] = sel_pos[s];
    }
    uint4 kv[kRows][PPL], vv[kRows][PPL];
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const int64_t s = s0 + r < n_sel ? s0 + r : n_sel - 1;
#pragma unroll
        for (int i = 0; i < PPL; ++i) {
            const int piece = lane + i * kWave;
            const int pc = piece < pieces_per_row ? piece : pieces_per_row - 1;
            kv[r][i] = stream_load16(k_new + s * pieces_per_row + pc);
            vv[r][i] = stream_load16(v_new + s * pieces_per_row + pc);
        }
    }
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const int64_t p = pos[r];
        if (p < 0 || p >= n_rows) continue;        // memory safety only; the caller guarantees the range
#pragma unroll
        for (int i = 0; i < PPL; ++i) {
            const int piece = lane + i * kWave;
            if (piece < pieces_per_row) {
                k_cache[p * pieces_per_row + piece] = kv[r][i];
                v_cache[p * pieces_per_row + piece] = vv[r][i];
            }
        }
        if (lane == 0 && reused) reused[p] = 0;
        if (dev_v && lane < n_kv_heads) dev_v[(int64_t)lane * n_rows + p] = 0.f;
    }
}

} // namespace
} // namespace kvs

extern "C" kvs_status kvs_scatter_kv(const kvs_shape *shape, int64_t n_rows,
                                     const void *k_new, const void *v_new,
                                     const int32_t *sel_pos, int64_t n_sel,
                                     void *k_cache, void *v_cache, uint8_t *reused, float *dev_v,
                                     void *stream)
{
    using namespace kvs;
    kvs_status st = check_shape(shape);
    if (st != KVS_OK) return st;
    if (n_rows < 0 || n_sel < 0) return fail(KVS_EINVAL, "kvs_scatter_kv: negative size");
    if (n_sel > n_rows) return fail(KVS_EINVAL, "kvs_scatter_kv: n_sel %lld exceeds the cache rows %lld", (long long)n_sel, (long long)n_rows);
    if (n_sel == 0) return KVS_OK;
    if (!k_new || !v_new || !sel_pos || !k_cache || !v_cache) return fail(KVS_EINVAL, "kvs_scatter_kv: NULL pointer");
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache))
        return fail(KVS_EINVAL, "kvs_scatter_kv: K/V pointers must be 16-byte aligned");
    if (shape->n_kv_heads > 64) return fail(KVS_EUNSUPPORTED, "kvs_scatter_kv: more than 64 kv heads");
    const int64_t row_bytes = (int64_t)shape->n_kv_heads * shape->head_dim * (int64_t)elem_bytes(shape->dtype);
    const int ppr = (int)(row_bytes / 16);
    const int ppl = (ppr + kWave - 1) / kWave;
    hipStream_t hs = (hipStream_t)stream;
#define KVS_SCAT(P, R)                                                                                                   \
    do {                                                                                                                 \
        const int64_t waves = (n_sel + (R) - 1) / (R), blocks = (waves + kScatWaves - 1) / kScatWaves;                   \
        if (blocks > 0x7fffffff) return fail(KVS_EINVAL, "kvs_scatter_kv: too many rows");                               \
        hipLaunchKernelGGL((scatter_kernel<P, R>), dim3((unsigned)blocks), dim3(kScatThreads), 0, hs, n_rows, n_sel, ppr, \
                           shape->n_kv_heads, (const uint4 *)k_new, (const uint4 *)v_new, sel_pos, (uint4 *)k_cache,      \
                           (uint4 *)v_cache, reused, dev_v);                                                              \
    } while (0)
    if (ppl <= 1) KVS_SCAT(1, 4);
    else if (ppl <= 2) KVS_SCAT(2, 2);
    else if (ppl <= 4) KVS_SCAT(4, 1);
    else if (ppl <= 8) KVS_SCAT(8, 1);
    else if (ppl <= 16) KVS_SCAT(16, 1);
    else return fail(KVS_EUNSUPPORTED, "kvs_scatter_kv: rows of %lld bytes", (long long)row_bytes);
#undef KVS_SCAT
    return check_launch("kvs_scatter_kv");
}
