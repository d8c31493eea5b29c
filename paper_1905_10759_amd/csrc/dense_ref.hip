// Dense comparison GEMM on unquantised operands (the "classical matrix multiply" role).
#include "kernels.h"

namespace hbmm {

hipError_t launch_dense_ref(const void *, int64_t, const void *, int64_t, int, int64_t, int64_t, int64_t,
                            float *, int64_t, hipStream_t)
{
    return hipErrorNotSupported;
}

}  // namespace hbmm
