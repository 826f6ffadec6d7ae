// HiF4 GEMM kernels (placeholder until the MFMA path lands).
#include "hif4_common.h"

namespace hif4 {

int launch_gemm(int, const void *, const uint32_t *, int64_t, const uint8_t *, const uint32_t *, const int32_t *, int,
                int64_t, int64_t, int64_t, void *, int64_t, int, void *, hipStream_t)
{
    return HIF4_ERR_UNSUPPORTED;
}

} // namespace hif4
