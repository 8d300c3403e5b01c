// Fine-grained top-k sparsifier (contrast point).  Placeholder until the
// radix-select kernels land: the entry points exist and report EUNSUPPORTED.
#include <hip/hip_runtime.h>

#include "plan.h"

extern "C" {

size_t topk_workspace_bytes(int64_t n, int32_t dtype) { return 256; }

covap_status_t topk_compress(const void *grad, void *residual, int64_t n, int64_t k, int32_t dtype,
                             float ef_coeff, void *out_vals, uint32_t *out_idx, void *workspace,
                             size_t ws_bytes, void *stream)
{
    return covap::fail(COVAP_EUNSUPPORTED, "topk_compress: not built yet");
}

}  // extern "C"
