// Instantiations of the fused DES-LOC step kernel for: KIND_ADOPT_T0.
// (One translation unit per update-rule family so that they compile in parallel.)
#include "desloc_step_kernel.h"

namespace desloc {

hipError_t launch_step_adopt_t0(int kind, uint32_t mask, int grad_bf16, const LaunchArgs& a,
                               hipStream_t stream, uint32_t* resident_out) {
    StepKernelFn fn = nullptr;
    switch (kind) {
        case KIND_ADOPT_T0: fn = select_kernel<KIND_ADOPT_T0>(mask, a.M, grad_bf16, a.strided); break;
        default: break;
    }
    return launch_or_query(fn, mask, a, stream, resident_out);
}

}  // namespace desloc
