// Placeholder: the matrix-core prefill path is under construction; bf16 inputs
// run through the fp32 kernel until it lands.
#include "kda_common.h"

namespace kda {

kda_status chunk_f32_dispatch(const kda_dims *, const void *, const void *, const void *,
                              const void *, const void *, const float *, const int32_t *, void *,
                              float *, hipStream_t);

size_t chunk_mfma_workspace_size(const kda_dims *, bool) { return 0; }

kda_status chunk_mfma_dispatch(const kda_dims *d, const void *q, const void *k, const void *v,
                               const void *log_alpha, const void *beta, const float *h0,
                               const int32_t *cu, void *o, float *hT, void *, size_t,
                               hipStream_t stream)
{
    return chunk_f32_dispatch(d, q, k, v, log_alpha, beta, h0, cu, o, hT, stream);
}

}  // namespace kda
