// Update-then-average DES-LOC-Adam step kernels without the AMSGrad state.
#include "desloc_post_kernel.h"

namespace desloc {

hipError_t launch_step_post_adam_ams(int kind, uint32_t mask, int grad_bf16, const LaunchArgs& a,
                                     hipStream_t stream);

hipError_t launch_step_post_adam(int kind, uint32_t mask, int amsgrad, int grad_bf16,
                                 const LaunchArgs& a, hipStream_t stream) {
    if (amsgrad) return launch_step_post_adam_ams(kind, mask, grad_bf16, a, stream);
    StepKernelFn fn = kind == KIND_ADAM_LITERAL
                          ? select_post_kernel<KIND_ADAM_LITERAL, false>(mask, a.M, grad_bf16, a.strided)
                          : select_post_kernel<KIND_ADAM, false>(mask, a.M, grad_bf16, a.strided);
    return launch_post_fn(fn, mask, a, stream);
}

}  // namespace desloc
