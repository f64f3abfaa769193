// Update-then-average DES-LOC-Adam step kernels with the AMSGrad state vt = max(v, vt).
#include "desloc_post_kernel.h"

namespace desloc {

hipError_t launch_step_post_adam_ams(int kind, uint32_t mask, int grad_bf16, const LaunchArgs& a,
                                     hipStream_t stream) {
    StepKernelFn fn = kind == KIND_ADAM_LITERAL
                          ? select_post_kernel<KIND_ADAM_LITERAL, true>(mask, a.M, grad_bf16, a.strided)
                          : select_post_kernel<KIND_ADAM, true>(mask, a.M, grad_bf16, a.strided);
    return launch_post_fn(fn, mask, a, stream);
}

}  // namespace desloc
