// kvs_scatter_kv: the KV Writer step -- rows of freshly recomputed K/V overwrite the reused
// entries of the cache at the selected positions.  A pure copy: every lane moves one 16-byte
// piece, consecutive lanes move consecutive pieces of the same row, so both the gather side
// (dense k_new/v_new) and the scatter side (whole cache rows of >= 512 bytes) are coalesced.
#include "kvs_internal.h"

namespace kvs {
namespace {

constexpr int kScatThreads = 256;

__global__ __launch_bounds__(kScatThreads) void scatter_kernel(
    int64_t n_rows, int64_t n_sel, int pieces_per_row, int n_kv_heads,
    const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new,
    const int32_t *__restrict__ sel_pos,
    uint4 *__restrict__ k_cache, uint4 *__restrict__ v_cache,
    uint8_t *__restrict__ reused, float *__restrict__ dev_v)
{
    const int64_t total = n_sel * pieces_per_row;
    for (int64_t e = (int64_t)blockIdx.x * kScatThreads + threadIdx.x; e < total;
         e += (int64_t)gridDim.x * kScatThreads) {
        const int64_t s = e / pieces_per_row;
        const int piece = (int)(e - s * pieces_per_row);
        const int64_t p = sel_pos[s];
        if (p < 0 || p >= n_rows) continue; // memory safety only; the caller guarantees range
        const uint4 kv = stream_load16(k_new + e);
        const uint4 vv = stream_load16(v_new + e);
        k_cache[p * pieces_per_row + piece] = kv;
        v_cache[p * pieces_per_row + piece] = vv;
        if (piece == 0 && reused) reused[p] = 0;
        if (dev_v && piece < n_kv_heads) dev_v[(int64_t)piece * n_rows + p] = 0.f;
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
    const int64_t row_bytes = (int64_t)shape->n_kv_heads * shape->head_dim * (int64_t)elem_bytes(shape->dtype);
    const int ppr = (int)(row_bytes / 16);
    if (shape->n_kv_heads > ppr) return fail(KVS_EUNSUPPORTED, "kvs_scatter_kv: row shorter than 16 bytes per head");
    const int64_t total = n_sel * ppr;
    int64_t blocks = (total + kScatThreads - 1) / kScatThreads;
    if (blocks > 1 << 20) blocks = 1 << 20;
    hipLaunchKernelGGL(scatter_kernel, dim3((unsigned)blocks), dim3(kScatThreads), 0, (hipStream_t)stream,
                       n_rows, n_sel, ppr, shape->n_kv_heads, (const uint4 *)k_new, (const uint4 *)v_new,
                       sel_pos, (uint4 *)k_cache, (uint4 *)v_cache, reused, dev_v);
    return check_launch("kvs_scatter_kv");
}
