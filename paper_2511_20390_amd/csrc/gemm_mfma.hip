// placeholder until the MFMA GEMM lands
#include "free_internal.h"
namespace freemi {
bool mfma_linear_supported(int32_t, int32_t, int32_t) { return false; }
int32_t launch_linear_mfma(const bf16_t*, const bf16_t*, const float*, int32_t, int32_t, int32_t, int32_t,
                           bf16_t*, float*, RowVec, hipStream_t) { return FREE_ERR_SHAPE; }
}
