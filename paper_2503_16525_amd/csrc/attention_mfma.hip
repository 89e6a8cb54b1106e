// placeholder until the matrix-core kernel lands: reports no supported shape
#include "attention.h"
namespace kvs {
bool attention_mfma_supports(const kvs_shape *) { return false; }
kvs_status launch_attention_mfma(const kvs_shape *, const AttnBatch &, int64_t, const void *, const int32_t *,
                                 const void *, const void *, float, void *, float *, hipStream_t)
{
    return fail(KVS_EUNSUPPORTED, "kvs_partial_attention: matrix-core path not built");
}
} // namespace kvs
