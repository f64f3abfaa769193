// Instantiations of the fused DES-LOC step kernel for: KIND_ADOPT_T0.
// (One translation unit per update-rule family so that they compile in parallel.)
#include "desloc_step_kernel.h"

namespace desloc {

hipError_t launch_step_adopt_t0(int kind, uint32_t mask, int grad_bf16, const LaunchArgs& a,
                               hipStream_t stream) {
    StepKernelFn fn = nullptr;
    switch (kind) {
        case KIND_ADOPT_T0: fn = select_kernel<KIND_ADOPT_T0>(mask, a.M, grad_bf16); break;
        default: break;
    }
    if (fn == nullptr) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fn, dim3(a.n_chunks), dim3(WG_THREADS), 0, stream, a);
    return hipGetLastError();
}

}  // namespace desloc
