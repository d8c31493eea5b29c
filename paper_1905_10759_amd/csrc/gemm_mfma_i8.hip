// int8 +-1 matrix-core variant of the HBMM contraction (comparison point only).
#include "kernels.h"

namespace hbmm {

hipError_t launch_mfma_i8_gemm(const uint32_t *, const float *, int64_t, int64_t, int, const uint32_t *,
                               const float *, int64_t, int64_t, int, int64_t, int64_t, int64_t, float *,
                               int64_t, hipStream_t)
{
    return hipErrorNotSupported;
}

}  // namespace hbmm
