// Instantiations of the fused DES-LOC step kernel for: KIND_ADAM KIND_ADAM_LITERAL.
// (One translation unit per update-rule family so that they compile in parallel.)
#include "desloc_step_kernel.h"

namespace desloc {

hipError_t launch_step_adam(int kind, uint32_t mask, int grad_bf16, const LaunchArgs& a,
                               hipStream_t stream) {
    StepKernelFn fn = nullptr;
    switch (kind) {
        case KIND_ADAM: fn = select_kernel<KIND_ADAM>(mask, a.M, grad_bf16, a.strided); break;
        case KIND_ADAM_LITERAL: fn = select_kernel<KIND_ADAM_LITERAL>(mask, a.M, grad_bf16, a.strided); break;
        default: break;
    }
    if (fn == nullptr) return hipErrorInvalidValue;
    if (a.lds_bytes > 65536u) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           static_cast<int>(a.lds_bytes));
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(fn, dim3(a.n_chunks, mask == 0 ? a.M : 1), dim3(STEP_WG_THREADS), a.lds_bytes, stream,
                       a);
    return hipGetLastError();
}

}  // namespace desloc
