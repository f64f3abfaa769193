// Per-replica global L2 norm of the gradient, for norm-based clipping (the clipping the
// paper's model table says its experiments used).  Two deterministic levels:
//   1. sumsq_partial_kernel: one workgroup per (run of up to 65536 elements of a segment, replica) sums
//      g^2 in fp64 -- each lane over its own elements in address order, then a fixed shuffle
//      tree across the 64 lanes of a wave, then the 4 waves in order through LDS -- and writes
//      one partial;
//   2. sumsq_final_kernel: one workgroup per replica sums the partials the same way and
//      turns the sum into norm and scale = norm > rho ? rho / norm : 1.
// No atomics: the result does not depend on scheduling, so every run gives the same bits.
#include "desloc_step_kernel.h"

namespace desloc {

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;  // valid in lane 0
}

// Sum over the workgroup, valid in thread 0.  lds: at least WG_THREADS / 64 doubles.
__device__ __forceinline__ double block_sum(double v, double* lds) {
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    double total = 0.0;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 0; w < WG_THREADS / 64; ++w) total += lds[w];
    }
    return total;
}

// Adds g^2 over [start, start + len) of one gradient array to acc: lanes tid, tid + nthreads, ...
// each take 4-vectors in address order; a ragged tail of 1..3 elements goes one at a time.
template <bool BF16>
__device__ __forceinline__ void add_squares(double& acc, const void* g, uint64_t start, uint32_t len,
                                            uint32_t tid, uint32_t nthreads) {
    for (uint32_t off = tid * VEC; off < len; off += nthreads * VEC) {
        if (off + VEC <= len) {
            float v[VEC];
            ld_grad<VEC, BF16>(v, g, start + off);
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc += static_cast<double>(v[j]) * static_cast<double>(v[j]);
        } else {
            for (uint32_t k = off; k < len; ++k) {
                float v[1];
                ld_grad<1, BF16>(v, g, start + k);
                acc += static_cast<double>(v[0]) * static_cast<double>(v[0]);
            }
        }
    }
}

// One partial per (workgroup, replica).  Strided layouts: workgroup c sums chunk c of
// a.chunk_elems elements.  Table layouts: workgroup c sums the run of elements runs[c] of one
// segment (runs never cross segments; the gradient of a segment is contiguous whatever the
// step kernels' chunk records look like).  All lanes of the workgroup share the run.
template <bool BF16>
__global__ void __launch_bounds__(WG_THREADS) sumsq_partial_kernel(LaunchArgs a, const DiagChunk* __restrict__ runs,
                                                                    double* __restrict__ partials) {
    __shared__ double lds[WG_THREADS / 64];
    const uint32_t c = blockIdx.x, m = blockIdx.y;
    const uint32_t Mrow = static_cast<uint32_t>(a.M);
    double acc = 0.0;
    if (a.strided) {
        const uint64_t start = static_cast<uint64_t>(c) * a.chunk_elems;
        const uint64_t left = a.numel0 - start;
        const uint32_t len = left < a.chunk_elems ? static_cast<uint32_t>(left) : a.chunk_elems;
        const void* g = reinterpret_cast<const void*>(a.base[ARR_G] + m * a.rstride[ARR_G]);
        add_squares<BF16>(acc, g, start, len, threadIdx.x, WG_THREADS);
    } else {
        const DiagChunk r = runs[c];
        const void* g = reinterpret_cast<const void*>(
            a.ptrs[(static_cast<uint64_t>(r.seg) * N_ARRAYS + ARR_G) * Mrow + m]);
        add_squares<BF16>(acc, g, r.start, r.len, threadIdx.x, WG_THREADS);
    }
    const double total = block_sum(acc, lds);
    if (threadIdx.x == 0) partials[static_cast<uint64_t>(m) * gridDim.x + c] = total;
}

__global__ void __launch_bounds__(WG_THREADS) sumsq_final_kernel(const double* __restrict__ partials,
                                                                  uint32_t n_partials, float rho,
                                                                  float* __restrict__ norms,
                                                                  float* __restrict__ gscale) {
    __shared__ double lds[WG_THREADS / 64];
    const uint32_t m = blockIdx.x;
    const double* p = partials + static_cast<uint64_t>(m) * n_partials;
    double acc = 0.0;
    for (uint32_t i = threadIdx.x; i < n_partials; i += WG_THREADS) acc += p[i];
    const double total = block_sum(acc, lds);
    if (threadIdx.x == 0) {
        const float nrm = static_cast<float>(sqrt(total));
        norms[m] = nrm;
        gscale[m] = nrm > rho ? rho / nrm : 1.0f;
    }
}

// ---- batched per-tensor diagnostic and snapshot copy over tensor-aligned records ----

// Lane-local walk over one record in address order: up to 3 leading elements until the element
// index is a multiple of 4 (thread t takes element t), then 4-vectors (thread t takes vectors
// t, t + 256, ...; four of them per trip so that their loads are in flight together), then up to
// 3 trailing elements.  one(i) handles the element at record-relative index i; vec(i0, n) handles
// n <= 4 vectors whose first elements are i0, i0 + 1024, ... (in that order).
template <typename F1, typename FV>
__device__ __forceinline__ void walk_record(const DiagChunk& c, bool vec_ok, F1&& one, FV&& vec) {
    const uint32_t t = threadIdx.x;
    if (!vec_ok) {
        for (uint32_t i = t; i < c.len; i += WG_THREADS) one(i);
        return;
    }
    uint32_t head = (4u - static_cast<uint32_t>(c.start & 3u)) & 3u;
    if (head > c.len) head = c.len;
    if (t < head) one(t);
    const uint32_t nvec = (c.len - head) / 4u;
    uint32_t v = t;
    for (; v + 3u * WG_THREADS < nvec; v += 4u * WG_THREADS) vec(head + 4u * v, 4);
    for (; v < nvec; v += WG_THREADS) vec(head + 4u * v, 1);
    const uint32_t done = head + 4u * nvec;
    if (done + t < c.len) one(done + t);
}

// Adds sum (s - r)^2 and sum r^2 over the record c (s, r: segment bases of the state and of the
// reference) to this lane's dd and rr: 128-bit loads where vec_ok, four vectors of each array in flight.
__device__ __forceinline__ void record_sums(const float* s_base, const float* r_base, const DiagChunk& c, bool vec_ok,
                                            double& dd, double& rr) {
    const float* s = s_base + c.start;
    const float* r = r_base + c.start;
    auto add = [&](float x32, float y32) {
        const double x = static_cast<double>(x32), y = static_cast<double>(y32);
        dd += (x - y) * (x - y);
        rr += y * y;
    };
    walk_record(
        c, vec_ok, [&](uint32_t i) { add(*as_global<float>(s + i), *as_global<float>(r + i)); },
        [&](uint32_t i0, int n) {
            float a[4][4], b[4][4];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (q < n) {
                    ld_f32<4>(a[q], s + i0 + q * (4 * WG_THREADS));
                    ld_f32<4>(b[q], r + i0 + q * (4 * WG_THREADS));
                }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (q < n) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) add(a[q][j], b[q][j]);
                }
        });
}

// Relative-rate-of-change diagnostic: partial sums of (s - ref)^2 and ref^2 over the elements
// [offset, offset + numel) of one segment, for every replica (grid.y); workgroup b takes the `chunk`
// elements from offset + b * chunk on, walked like a record of the batched form (so any tensor offset is
// fine).  part[0 .. M*P) holds the difference sums, part[M*P ..) the reference sums, P = partials per
// replica over all launches, p0 = this launch's first.  vec_ok: every state and reference base is
// 16-byte aligned.
__global__ void __launch_bounds__(WG_THREADS) diff_sumsq_partial_kernel(
    const uint64_t* __restrict__ s_row, const uint64_t* __restrict__ r_row, uint64_t offset,
    uint64_t numel, uint32_t chunk, uint32_t P, uint32_t p0, int vec_ok, double* __restrict__ part) {
    __shared__ double lds[WG_THREADS / 64];
    const uint32_t m = blockIdx.y, M = gridDim.y;
    const uint64_t start = static_cast<uint64_t>(blockIdx.x) * chunk;
    const uint64_t left = numel - start;
    const DiagChunk c{offset + start, 0u, left < chunk ? static_cast<uint32_t>(left) : chunk};
    double dd = 0.0, rr = 0.0;
    record_sums(reinterpret_cast<const float*>(s_row[m]), reinterpret_cast<const float*>(r_row[m]), c, vec_ok != 0, dd, rr);
    const double tdd = block_sum(dd, lds);
    __syncthreads();
    const double trr = block_sum(rr, lds);
    if (threadIdx.x == 0) {
        part[static_cast<uint64_t>(m) * P + p0 + blockIdx.x] = tdd;
        part[static_cast<uint64_t>(M + m) * P + p0 + blockIdx.x] = trr;
    }
}

// One workgroup per (replica, quantity): out[q * M + m] = sqrt(sum of its partials).
__global__ void __launch_bounds__(WG_THREADS) diff_sumsq_final_kernel(const double* __restrict__ part,
                                                                       uint32_t P, float* __restrict__ out) {
    __shared__ double lds[WG_THREADS / 64];
    const double* p = part + static_cast<uint64_t>(blockIdx.x) * P;
    double acc = 0.0;
    for (uint32_t i = threadIdx.x; i < P; i += WG_THREADS) acc += p[i];
    const double total = block_sum(acc, lds);
    if (threadIdx.x == 0) out[blockIdx.x] = static_cast<float>(sqrt(total));
}

__global__ void __launch_bounds__(WG_THREADS) diag_partial_kernel(const uint64_t* __restrict__ ptrs, int which,
                                                                   const uint64_t* __restrict__ ref,
                                                                   const DiagChunk* __restrict__ chunks, uint32_t P,
                                                                   int vec_ok, double* __restrict__ part) {
    __shared__ double lds[WG_THREADS / 64];
    const uint32_t m = blockIdx.y, M = gridDim.y;
    const DiagChunk c = chunks[blockIdx.x];
    double dd = 0.0, rr = 0.0;
    record_sums(reinterpret_cast<const float*>(ptrs[(static_cast<uint64_t>(c.seg) * N_ARRAYS + which) * M + m]),
                reinterpret_cast<const float*>(ref[static_cast<uint64_t>(c.seg) * M + m]), c, vec_ok != 0, dd, rr);
    const double tdd = block_sum(dd, lds);
    __syncthreads();
    const double trr = block_sum(rr, lds);
    if (threadIdx.x == 0) {
        part[static_cast<uint64_t>(m) * P + blockIdx.x] = tdd;
        part[static_cast<uint64_t>(M + m) * P + blockIdx.x] = trr;
    }
}

// One wave per (tensor, replica): sums the tensor's partial sums in a fixed order.
__global__ void __launch_bounds__(64) diag_final_kernel(const double* __restrict__ part, uint32_t P,
                                                         const uint32_t* __restrict__ first,
                                                         const uint32_t* __restrict__ count,
                                                         float* __restrict__ change, float* __restrict__ base) {
    const uint64_t k = blockIdx.x;
    const uint32_t m = blockIdx.y, M = gridDim.y;
    const uint32_t p0 = first[k], n = count[k];
    const double* pd = part + static_cast<uint64_t>(m) * P + p0;
    const double* pr = part + static_cast<uint64_t>(M + m) * P + p0;
    double dd = 0.0, rr = 0.0;
    for (uint32_t i = threadIdx.x; i < n; i += 64) {
        dd += pd[i];
        rr += pr[i];
    }
    dd = wave_sum(dd);
    rr = wave_sum(rr);
    if (threadIdx.x == 0) {
        change[k * M + m] = static_cast<float>(sqrt(dd));
        base[k * M + m] = static_cast<float>(sqrt(rr));
    }
}

// Snapshot copy, one 256-lane workgroup per record: for lists of many small tensors, whose records are
// mostly short (a workgroup per 1 KiB run would then be mostly start-up).
__global__ void __launch_bounds__(WG_THREADS) snapshot_copy_wide_kernel(const uint64_t* __restrict__ ptrs, int which,
                                                                         const uint64_t* __restrict__ dst,
                                                                         const DiagChunk* __restrict__ chunks, int vec_ok) {
    const uint32_t m = blockIdx.y, M = gridDim.y;
    const DiagChunk c = chunks[blockIdx.x];
    const float* s = reinterpret_cast<const float*>(ptrs[(static_cast<uint64_t>(c.seg) * N_ARRAYS + which) * M + m]) + c.start;
    float* d = reinterpret_cast<float*>(dst[static_cast<uint64_t>(c.seg) * M + m]) + c.start;
    walk_record(
        c, vec_ok != 0, [&](uint32_t i) { *as_global<float>(d + i) = *as_global<float>(s + i); },
        [&](uint32_t i0, int n) {
            float a[4][4];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (q < n) ld_f32<4>(a[q], s + i0 + q * (4 * WG_THREADS));
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (q < n) st_f32<4>(d + i0 + q * (4 * WG_THREADS), a[q]);
        });
}

// Snapshot copy of long records: single-wave workgroups, COPY_TILES of them per record; each copies up to four 1 KiB runs
// of its record (wave-contiguous, consecutive), all four loads in flight before the first store -- the shape
// a one-read, one-write stream runs fastest with on MI355X.  Address order inside a record as in
// walk_record: up to 3 leading elements until the element index is a multiple of 4 and up to 3 trailing
// ones go one at a time (first workgroup of the record), everything between as 128-bit vectors.
enum : uint32_t { COPY_WAVE_VECS = 4u * 64u, COPY_TILES = DIAG_CHUNK_ELEMS / (4u * COPY_WAVE_VECS) };

__global__ void __launch_bounds__(64) snapshot_copy_kernel(const uint64_t* __restrict__ ptrs, int which,
                                                            const uint64_t* __restrict__ dst,
                                                            const DiagChunk* __restrict__ chunks, int vec_ok) {
    const uint32_t m = blockIdx.y, M = gridDim.y, t = threadIdx.x;
    const DiagChunk c = chunks[blockIdx.x / COPY_TILES];
    const uint32_t sub = blockIdx.x % COPY_TILES;
    const uint32_t first = sub * 4u * COPY_WAVE_VECS;  // elements (vec_ok: counted after the head)
    if (first >= c.len) return;
    const float* s = reinterpret_cast<const float*>(ptrs[(static_cast<uint64_t>(c.seg) * N_ARRAYS + which) * M + m]) + c.start;
    float* d = reinterpret_cast<float*>(dst[static_cast<uint64_t>(c.seg) * M + m]) + c.start;
    auto one = [&](uint32_t i) { *as_global<float>(d + i) = *as_global<float>(s + i); };
    if (!vec_ok) {
        const uint32_t end = first + 4u * COPY_WAVE_VECS < c.len ? first + 4u * COPY_WAVE_VECS : c.len;
        for (uint32_t i = first + t; i < end; i += 64u) one(i);
        return;
    }
    uint32_t head = (4u - static_cast<uint32_t>(c.start & 3u)) & 3u;
    if (head > c.len) head = c.len;
    const uint32_t nvec = (c.len - head) / 4u;
    if (sub == 0) {
        if (t < head) one(t);
        const uint32_t done = head + 4u * nvec;
        if (done + t < c.len) one(done + t);
    }
    const uint32_t v0 = sub * COPY_WAVE_VECS + t;
    float a[4][4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (v0 + q * 64u < nvec) ld_f32<4>(a[q], s + head + 4u * (v0 + q * 64u));
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (v0 + q * 64u < nvec) st_f32<4>(d + head + 4u * (v0 + q * 64u), a[q]);
}

hipError_t launch_state_change_tensors(const uint64_t* d_ptrs, int which, const uint64_t* d_ref, uint32_t M,
                                       const DiagChunk* d_chunks, uint32_t P, const uint32_t* d_first,
                                       const uint32_t* d_count, uint64_t n_tensors, int vec_ok, double* d_part,
                                       float* d_change, float* d_base, hipStream_t stream) {
    if (P != 0) {
        hipLaunchKernelGGL(diag_partial_kernel, dim3(P, M), dim3(WG_THREADS), 0, stream, d_ptrs, which, d_ref, d_chunks,
                           P, vec_ok, d_part);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(diag_final_kernel, dim3(static_cast<uint32_t>(n_tensors), M), dim3(64), 0, stream, d_part, P,
                       d_first, d_count, d_change, d_base);
    return hipGetLastError();
}

hipError_t launch_snapshot_copy(const uint64_t* d_ptrs, int which, const uint64_t* d_dst, uint32_t M,
                                const DiagChunk* d_chunks, uint32_t P, uint64_t numel, int vec_ok, hipStream_t stream) {
    if (P == 0) return hipSuccess;
    // Mostly full records (at most a tenth of the 1 KiB runs of all records empty): sixteen single-wave
    // workgroups per record, 20 resident per compute unit (each waits for its record and two pointers
    // before its four loads, so it takes more waves than a copy with its addresses in kernel arguments
    // needs; 1.7B-parameter workload, M = 4: 6.7 TB/s at 20, 6.5 at 16 and at 24, 5.6 at 12).
    const uint64_t tiles = static_cast<uint64_t>(P) * COPY_TILES;
    if (tiles <= 0x7fffffffull && tiles * (4u * COPY_WAVE_VECS) <= numel + numel / 10u) {
        constexpr uint32_t COPY_LDS_LIMITER_BYTES = 8100;
        hipLaunchKernelGGL(snapshot_copy_kernel, dim3(static_cast<uint32_t>(tiles), M), dim3(64), COPY_LDS_LIMITER_BYTES,
                           stream, d_ptrs, which, d_dst, d_chunks, vec_ok);
        return hipGetLastError();
    }
    // Many short records: one 256-lane workgroup each, 16 waves per compute unit.
    constexpr uint32_t WIDE_COPY_LDS_LIMITER_BYTES = 160u * 1024u / 4u - 64u;
    hipLaunchKernelGGL(snapshot_copy_wide_kernel, dim3(P, M), dim3(WG_THREADS), WIDE_COPY_LDS_LIMITER_BYTES, stream,
                       d_ptrs, which, d_dst, d_chunks, vec_ok);
    return hipGetLastError();
}

hipError_t launch_state_change(const uint64_t* d_s_rows, const uint64_t* d_r_rows, uint32_t M,
                               uint32_t n_ranges, const uint64_t* row_index, const uint64_t* offsets,
                               const uint64_t* numels, uint32_t chunk, int vec_ok, double* d_part, uint32_t P,
                               float* d_out, hipStream_t stream) {
    uint32_t p0 = 0;
    for (uint32_t k = 0; k < n_ranges; ++k) {
        if (numels[k] == 0) continue;
        const uint32_t blocks = static_cast<uint32_t>((numels[k] + chunk - 1) / chunk);
        hipLaunchKernelGGL(diff_sumsq_partial_kernel, dim3(blocks, M), dim3(WG_THREADS), 0, stream,
                           d_s_rows + row_index[k] * N_ARRAYS * M, d_r_rows + row_index[k] * M, offsets[k],
                           numels[k], chunk, P, p0, vec_ok, d_part);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        p0 += blocks;
    }
    hipLaunchKernelGGL(diff_sumsq_final_kernel, dim3(2u * M), dim3(WG_THREADS), 0, stream, d_part, P, d_out);
    return hipGetLastError();
}

// a.n_chunks: partial sums per replica = chunks of a.chunk_elems elements (strided layouts) or
// entries of `runs` (table layouts).  d_partials holds M * a.n_chunks doubles.
hipError_t launch_grad_norms(const LaunchArgs& a, const DiagChunk* runs, int grad_bf16, float rho,
                             double* d_partials, float* d_norms, float* d_gscale, hipStream_t stream) {
    if (a.n_chunks == 0) {
        // no elements: norm 0, scale 1 for every replica
        hipLaunchKernelGGL(sumsq_final_kernel, dim3(a.M), dim3(WG_THREADS), 0, stream, d_partials, 0u, rho,
                           d_norms, d_gscale);
        return hipGetLastError();
    }
    if (!a.strided && runs == nullptr) return hipErrorInvalidValue;
    const dim3 grid(a.n_chunks, a.M);
    if (grad_bf16)
        hipLaunchKernelGGL(sumsq_partial_kernel<true>, grid, dim3(WG_THREADS), 0, stream, a, runs, d_partials);
    else
        hipLaunchKernelGGL(sumsq_partial_kernel<false>, grid, dim3(WG_THREADS), 0, stream, a, runs, d_partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(sumsq_final_kernel, dim3(a.M), dim3(WG_THREADS), 0, stream, d_partials, a.n_chunks,
                       rho, d_norms, d_gscale);
    return hipGetLastError();
}

}  // namespace desloc
