// bf16 MFMA per-axis attention forward for gfx950 (placeholder until the kernels land).
#include "ta_internal.h"

namespace ta {

bool mfma_forward_supports(int32_t, int32_t, int, int* kernel_id) {
    if (kernel_id) *kernel_id = K_GENERIC;
    return false;
}

hipError_t launch_mfma_forward(const HopParams&, int, hipStream_t) { return hipErrorNotSupported; }

}  // namespace ta
