// Dispatcher over the per-family step launchers, plus the two small service kernels:
// state initialisation (Alg. 1, local-init line) and the replica mean E_m[.] used by
// desloc_read_state for the averaged iterate of the paper's analysis.
#include "desloc_step_kernel.h"

namespace desloc {

hipError_t launch_step_adam(int, uint32_t, int, const LaunchArgs&, hipStream_t);
hipError_t launch_step_adopt(int, uint32_t, int, const LaunchArgs&, hipStream_t);
hipError_t launch_step_adopt_t0(int, uint32_t, int, const LaunchArgs&, hipStream_t);
hipError_t launch_step_sgdm(int, uint32_t, int, const LaunchArgs&, hipStream_t);

hipError_t launch_step(int kind, uint32_t mask, int grad_bf16, const LaunchArgs& a,
                       hipStream_t stream) {
    if (a.n_chunks == 0) return hipSuccess;
    switch (kind) {
        case KIND_ADAM:
        case KIND_ADAM_LITERAL: return launch_step_adam(kind, mask, grad_bf16, a, stream);
        case KIND_ADOPT:
        case KIND_ADOPT_AVGNORM: return launch_step_adopt(kind, mask, grad_bf16, a, stream);
        case KIND_ADOPT_T0: return launch_step_adopt_t0(kind, mask, grad_bf16, a, stream);
        case KIND_SGDM: return launch_step_sgdm(kind, mask, grad_bf16, a, stream);
        default: return hipErrorInvalidValue;
    }
}

// u^m = v^m = 0 for every replica; optionally x^m = x^0 (same chunk decomposition as the
// step kernel, so it is one launch whatever the number of tensors).
__global__ void __launch_bounds__(WG_THREADS) init_states_kernel(LaunchArgs a, int has_v,
                                                                  int broadcast) {
    const uint32_t c = blockIdx.x;
    const uint32_t s = a.chunk_seg[c];
    const uint64_t numel = a.segs[s].numel;
    const uint64_t start = (static_cast<uint64_t>(c) - a.segs[s].chunk0) * a.chunk_elems;
    const uint64_t left = numel - start;
    const uint32_t len = left < a.chunk_elems ? static_cast<uint32_t>(left) : a.chunk_elems;
    const int M = a.M;
    const uint64_t* __restrict__ P = a.ptrs + static_cast<uint64_t>(s) * 4u * M;
    for (uint32_t off = threadIdx.x; off < len; off += WG_THREADS) {
        const uint64_t e = start + off;
        const float x0 = broadcast ? reinterpret_cast<const float*>(P[0])[e] : 0.0f;
        for (int m = 0; m < M; ++m) {
            reinterpret_cast<float*>(P[1 * M + m])[e] = 0.0f;
            if (has_v) reinterpret_cast<float*>(P[2 * M + m])[e] = 0.0f;
            if (broadcast && m > 0) reinterpret_cast<float*>(P[0 * M + m])[e] = x0;
        }
    }
}

hipError_t launch_init_states(const LaunchArgs& a, int has_v, int broadcast, hipStream_t stream) {
    if (a.n_chunks == 0) return hipSuccess;
    hipLaunchKernelGGL(init_states_kernel, dim3(a.n_chunks), dim3(WG_THREADS), 0, stream, a, has_v,
                       broadcast);
    return hipGetLastError();
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
