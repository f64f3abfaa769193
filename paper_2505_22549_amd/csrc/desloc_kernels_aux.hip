// Dispatcher over the per-family step launchers, plus the two small service kernels:
// state initialisation (Alg. 1, local-init line) and the replica mean E_m[.] used by
// desloc_read_state for the averaged iterate of the paper's analysis.
#include "desloc_step_kernel.h"

namespace desloc {

hipError_t launch_step_adam(int, uint32_t, int, const LaunchArgs&, hipStream_t, uint32_t*);
hipError_t launch_step_adopt(int, uint32_t, int, const LaunchArgs&, hipStream_t, uint32_t*);
hipError_t launch_step_adopt_t0(int, uint32_t, int, const LaunchArgs&, hipStream_t, uint32_t*);
hipError_t launch_step_sgdm(int, uint32_t, int, const LaunchArgs&, hipStream_t, uint32_t*);
hipError_t launch_step_post_adam(int, uint32_t, int, int, const LaunchArgs&, hipStream_t);
hipError_t launch_step_post_sgdm(uint32_t, int, const LaunchArgs&, hipStream_t);

hipError_t launch_step(int kind, uint32_t mask, int grad_bf16, const LaunchArgs& a,
                       hipStream_t stream, uint32_t* resident_out) {
    if (a.n_chunks == 0 && resident_out == nullptr) return hipSuccess;
    switch (kind) {
        case KIND_ADAM:
        case KIND_ADAM_LITERAL: return launch_step_adam(kind, mask, grad_bf16, a, stream, resident_out);
        case KIND_ADOPT:
        case KIND_ADOPT_AVGNORM: return launch_step_adopt(kind, mask, grad_bf16, a, stream, resident_out);
        case KIND_ADOPT_T0: return launch_step_adopt_t0(kind, mask, grad_bf16, a, stream, resident_out);
        case KIND_SGDM: return launch_step_sgdm(kind, mask, grad_bf16, a, stream, resident_out);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_step_post(int kind, uint32_t mask, int amsgrad, int grad_bf16, const LaunchArgs& a,
                            hipStream_t stream) {
    if (a.n_chunks == 0) return hipSuccess;
    if (kind == KIND_SGDM) return launch_step_post_sgdm(mask, grad_bf16, a, stream);
    if (kind == KIND_ADAM || kind == KIND_ADAM_LITERAL)
        return launch_step_post_adam(kind, mask, amsgrad, grad_bf16, a, stream);
    return hipErrorInvalidValue;
}

// u^m = v^m = 0 for every replica; optionally x^m = x^0.  A grid-stride pass per segment:
// not a hot path, it runs once per context.
__global__ void __launch_bounds__(WG_THREADS) init_states_kernel(const uint64_t* __restrict__ row,
                                                                  int M, uint64_t numel, int has_v,
                                                                  int has_vmax, int broadcast) {
    const uint64_t stride = static_cast<uint64_t>(gridDim.x) * WG_THREADS;
    for (uint64_t e = static_cast<uint64_t>(blockIdx.x) * WG_THREADS + threadIdx.x; e < numel;
         e += stride) {
        const float x0 = broadcast ? reinterpret_cast<const float*>(row[0])[e] : 0.0f;
        for (int m = 0; m < M; ++m) {
            reinterpret_cast<float*>(row[1 * M + m])[e] = 0.0f;
            if (has_v) reinterpret_cast<float*>(row[2 * M + m])[e] = 0.0f;
            if (has_vmax) reinterpret_cast<float*>(row[ARR_VMAX * M + m])[e] = 0.0f;
            if (broadcast && m > 0) reinterpret_cast<float*>(row[0 * M + m])[e] = x0;
        }
    }
}

hipError_t launch_init_states(const uint64_t* d_ptrs, int M, const uint64_t* seg_numel,
                              uint64_t n_segs, int has_v, int has_vmax, int broadcast,
                              hipStream_t stream) {
    for (uint64_t s = 0; s < n_segs; ++s) {
        if (seg_numel[s] == 0) continue;
        uint64_t blocks = (seg_numel[s] + WG_THREADS - 1) / WG_THREADS;
        if (blocks > 16384) blocks = 16384;
        hipLaunchKernelGGL(init_states_kernel, dim3(static_cast<uint32_t>(blocks)), dim3(WG_THREADS),
                           0, stream, d_ptrs + s * N_ARRAYS * static_cast<uint64_t>(M), M, seg_numel[s],
                           has_v, has_vmax, broadcast);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

__global__ void __launch_bounds__(WG_THREADS) replica_mean_kernel(const uint64_t* __restrict__ row,
                                                                   int M, int is_bf16,
                                                                   uint64_t offset, uint64_t numel,
                                                                   float* __restrict__ out) {
    const uint64_t stride = static_cast<uint64_t>(gridDim.x) * WG_THREADS;
    for (uint64_t i = static_cast<uint64_t>(blockIdx.x) * WG_THREADS + threadIdx.x; i < numel;
         i += stride) {
        float sum = 0.0f;
        for (int m = 0; m < M; ++m) {
            float val;
            if (is_bf16)
                val = widen_bf16(reinterpret_cast<const uint16_t*>(row[m])[offset + i]);
            else
                val = reinterpret_cast<const float*>(row[m])[offset + i];
            sum = (m == 0) ? val : sum + val;
        }
        out[i] = sum / static_cast<float>(M);
    }
}

hipError_t launch_replica_mean(const uint64_t* row, int M, int is_bf16, uint64_t offset,
                               uint64_t numel, float* out, hipStream_t stream) {
    if (numel == 0) return hipSuccess;
    uint64_t blocks = (numel + WG_THREADS - 1) / WG_THREADS;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(replica_mean_kernel, dim3(static_cast<uint32_t>(blocks)), dim3(WG_THREADS), 0,
                       stream, row, M, is_bf16, offset, numel, out);
    return hipGetLastError();
}

}  // namespace desloc
