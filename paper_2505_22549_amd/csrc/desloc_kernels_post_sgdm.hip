// Update-then-average DES-LOC-SGDM step kernels (the SGDM appendix listing's ordering).
#include "desloc_post_kernel.h"

namespace desloc {

hipError_t launch_step_post_sgdm(uint32_t mask, int grad_bf16, const LaunchArgs& a, hipStream_t stream) {
    return launch_post_fn(select_post_kernel<KIND_SGDM, false>(mask, a.M, grad_bf16, a.strided), mask, a,
                          stream);
}

}  // namespace desloc
