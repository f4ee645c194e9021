// placeholder until the MFMA attention lands
#include "free_internal.h"
namespace freemi {
bool mfma_attention_supported(int32_t, int32_t) { return false; }
int32_t launch_attention_mfma(const bf16_t*, int32_t, int32_t, int32_t, int32_t, bf16_t*, hipStream_t) {
    return FREE_ERR_SHAPE;
}
}
