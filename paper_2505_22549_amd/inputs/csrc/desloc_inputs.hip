// Seeded synthetic inputs for the DES-LOC step library, generated on the GPU.
// INPUT GENERATOR ONLY: nothing of the optimizer's arithmetic lives here.
//
// Every value is a pure function of (seed, purpose, step t, replica m, tensor k,
// element i), so any single input can be regenerated anywhere.  The integer stream is
// the counter-based Philox4x32-10 generator of Salmon, Moraes, Dror and Shaw ("Parallel
// random numbers: as easy as 1, 2, 3", SC'11), written from the published round
// function; normals come from the Box-Muller transform in fp32.
//
//   counter = (i mod 2^32, k, t, m | purpose << 16),  key = (seed mod 2^32, i >> 32)
//
// Distributions (per tensor k a scale s_k, per replica a mean shift):
//   GAUSS      value = mean0 + mean_per_replica * m + s_k * Z0
//   STUDENT_T3 value = s_k * Z0 / sqrt((Z1^2 + Z2^2 + Z3^2) / 3)     (Student-t, nu = 3)
// Output fp32, or bf16 by round-to-nearest-even of the fp32 value.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

struct U4 { uint32_t x, y, z, w; };

__host__ __device__ inline U4 philox4x32_10(U4 c, uint32_t k0, uint32_t k1) {
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = static_cast<uint64_t>(M0) * c.x;
        const uint64_t p1 = static_cast<uint64_t>(M1) * c.z;
        U4 n;
        n.x = static_cast<uint32_t>(p1 >> 32) ^ c.y ^ k0;
        n.y = static_cast<uint32_t>(p1);
        n.z = static_cast<uint32_t>(p0 >> 32) ^ c.w ^ k1;
        n.w = static_cast<uint32_t>(p0);
        c = n;
        k0 += W0;
        k1 += W1;
    }
    return c;
}

// (0, 1] and [0, 1) uniforms with 24 random bits, exact in fp32.
__device__ inline float u01_open_low(uint32_t r) { return (static_cast<float>(r >> 8) + 1.0f) * 5.9604644775390625e-8f; }
__device__ inline float u01_open_high(uint32_t r) { return static_cast<float>(r >> 8) * 5.9604644775390625e-8f; }

__device__ inline void box_muller(uint32_t r0, uint32_t r1, float& z0, float& z1) {
    const float rad = sqrtf(-2.0f * logf(u01_open_low(r0)));
    const float ang = 6.283185307179586f * u01_open_high(r1);
    z0 = rad * cosf(ang);
    z1 = rad * sinf(ang);
}

__device__ inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t b = __float_as_uint(f);
    if ((b & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((b >> 16) | 0x40u);  // NaN
    b += 0x7fffu + ((b >> 16) & 1u);
    return static_cast<uint16_t>(b >> 16);
}

struct FillArgs {
    void* dst;               // packed buffer of one replica: tensors back to back
    const uint64_t* starts;  // device, [n_tensors + 1] prefix offsets into dst
    const float* scale;      // device, [n_tensors]
    uint64_t n_tensors;
    uint64_t total;
    uint64_t seed;
    uint32_t step, replica, purpose;
    int dist;                // 0 GAUSS, 1 STUDENT_T3
    int bf16;
    float mean0, mean_per_replica;
};

__global__ void __launch_bounds__(256) fill_kernel(FillArgs a) {
    const uint64_t stride = static_cast<uint64_t>(gridDim.x) * 256u;
    for (uint64_t p = static_cast<uint64_t>(blockIdx.x) * 256u + threadIdx.x; p < a.total; p += stride) {
        // tensor k with starts[k] <= p < starts[k+1] (zero-sized tensors are skipped)
        uint64_t lo = 0, hi = a.n_tensors;
        while (hi - lo > 1) {
            const uint64_t mid = (lo + hi) >> 1;
            if (a.starts[mid] <= p) lo = mid; else hi = mid;
        }
        const uint64_t k = lo, i = p - a.starts[lo];
        U4 c;
        c.x = static_cast<uint32_t>(i);
        c.y = static_cast<uint32_t>(k);
        c.z = a.step;
        c.w = a.replica | (a.purpose << 16);
        const U4 r = philox4x32_10(c, static_cast<uint32_t>(a.seed), static_cast<uint32_t>(i >> 32));
        float z0, z1, z2, z3;
        box_muller(r.x, r.y, z0, z1);
        float val;
        if (a.dist == 0) {
            val = a.mean0 + a.mean_per_replica * static_cast<float>(a.replica) + a.scale[k] * z0;
        } else {
            box_muller(r.z, r.w, z2, z3);
            val = a.scale[k] * z0 / sqrtf((z1 * z1 + z2 * z2 + z3 * z3) * (1.0f / 3.0f));
        }
        if (a.bf16) reinterpret_cast<uint16_t*>(a.dst)[p] = f32_to_bf16_rne(val);
        else reinterpret_cast<float*>(a.dst)[p] = val;
    }
}

// Plain copy of known size: the yardstick that hardware traffic counters are scaled by.
__global__ void __launch_bounds__(256) calibration_copy_kernel(const float4* __restrict__ src,
                                                               float4* __restrict__ dst, uint64_t n4) {
    const uint64_t stride = static_cast<uint64_t>(gridDim.x) * 256u;
    for (uint64_t i = static_cast<uint64_t>(blockIdx.x) * 256u + threadIdx.x; i < n4; i += stride)
        dst[i] = src[i];
}

// ---- streaming yardsticks: what the memory system gives a kernel of the step's shape ----
// R read streams and W write streams of equal length, swept together by single-wave
// workgroups, 1 KiB accesses per stream, streaming loads and write-through stores: the access
// pattern of the DES-LOC step without its arithmetic.  INPLACE: the writes go back to the first
// W read streams (as the step writes x, u, v back), else to W further streams.
typedef float v4f __attribute__((ext_vector_type(4)));

struct StreamArgs {
    uint64_t base;           // first stream; stream k starts k * stride_bytes further
    uint64_t stride_bytes;
    uint32_t paired;         // 1: halves of each 1 KiB access 32 KiB apart (groups of 64 KiB)
};

__device__ __forceinline__ v4f stream_load(uint64_t addr) {
    return __builtin_nontemporal_load(reinterpret_cast<const __attribute__((address_space(1))) v4f*>(addr));
}
__device__ __forceinline__ void stream_store(uint64_t addr, v4f val) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 2" ::"v"(reinterpret_cast<__attribute__((address_space(1))) v4f*>(addr)), "v"(val) : "memory");
}

// U: 1 KiB accesses per stream and wave (consecutive wave slots), all loads before any store.
template <int R, int W, bool INPLACE, int U>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(1, 3))) stream_kernel(StreamArgs a) {
    const uint32_t l = threadIdx.x;
    uint64_t off[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
        const uint32_t b = blockIdx.x * U + j;  // wave slot
        off[j] = a.paired ? static_cast<uint64_t>(b >> 6) * 65536u + (l >> 5) * 32768u + (b & 63u) * 512u + (l & 31u) * 16u
                          : static_cast<uint64_t>(b) * 1024u + l * 16u;
    }
    v4f t[U][R > 0 ? R : 1];
#pragma unroll
    for (int j = 0; j < U; ++j) {
        t[j][0] = v4f{1.0f, 2.0f, 3.0f, 4.0f};
#pragma unroll
        for (int r = 0; r < R; ++r) t[j][r] = stream_load(a.base + r * a.stride_bytes + off[j]);
    }
#pragma unroll
    for (int j = 0; j < U; ++j) {
        if constexpr (W == 0) {
            v4f s = t[j][0];
#pragma unroll
            for (int r = 1; r < R; ++r) s = s + t[j][r];
            // keeps the loads alive; the buffers hold zeros, so this store never happens
            if (s.x + s.y + s.z + s.w == 12345.678f) stream_store(a.base + off[j], s);
        } else {
            // every loaded value reaches a store: write stream w gets the sum of the read streams r = w (mod W)
#pragma unroll
            for (int w = 0; w < W; ++w) {
                v4f val = t[j][R > 0 ? w % (R > 0 ? R : 1) : 0];
#pragma unroll
                for (int r = w + W; r < R; r += W) val = val + t[j][r];
                stream_store(a.base + static_cast<uint64_t>(INPLACE ? w : R + w) * a.stride_bytes + off[j], val);
            }
        }
    }
}

typedef void (*StreamKernelFn)(StreamArgs);

// Shapes with one or two streams need several accesses in flight per wave to cover the memory
// latency (the step's shapes have R of them anyway).
StreamKernelFn pick_stream_kernel(int n_read, int n_write, int inplace, uint32_t* per_wave) {
    *per_wave = 1;
    if (n_read == 4 && n_write == 3 && inplace) return stream_kernel<4, 3, true, 1>;
    if (n_read == 3 && n_write == 2 && inplace) return stream_kernel<3, 2, true, 1>;
    if (n_read == 16 && n_write == 12 && inplace) return stream_kernel<16, 12, true, 1>;
    if (n_read == 32 && n_write == 24 && inplace) return stream_kernel<32, 24, true, 1>;
    *per_wave = 4;
    if (n_read == 1 && n_write == 0) return stream_kernel<1, 0, false, 4>;
    if (n_read == 0 && n_write == 1) return stream_kernel<0, 1, false, 4>;
    if (n_read == 1 && n_write == 1 && !inplace) return stream_kernel<1, 1, false, 4>;
    return nullptr;
}

__global__ void raw_kernel(const uint32_t* ctr, const uint32_t* key, uint32_t* out, uint64_t n) {
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n) return;
    U4 c{ctr[4 * i], ctr[4 * i + 1], ctr[4 * i + 2], ctr[4 * i + 3]};
    const U4 r = philox4x32_10(c, key[2 * i], key[2 * i + 1]);
    out[4 * i] = r.x; out[4 * i + 1] = r.y; out[4 * i + 2] = r.z; out[4 * i + 3] = r.w;
}

}  // namespace

extern "C" {

// Fills one replica's packed buffer.  All pointers are device pointers; asynchronous on
// `stream`.  Returns the hipError_t of the launch (0 = success).
int desloc_inputs_fill(void* dst, int bf16, uint64_t total, const uint64_t* d_starts,
                       const float* d_scale, uint64_t n_tensors, int dist, float mean0,
                       float mean_per_replica, uint64_t seed, uint32_t step, uint32_t replica,
                       uint32_t purpose, void* stream) {
    if (total == 0) return 0;
    if (dst == nullptr || d_starts == nullptr || d_scale == nullptr || n_tensors == 0) return 1;
    FillArgs a{dst, d_starts, d_scale, n_tensors, total, seed, step, replica, purpose, dist, bf16,
               mean0, mean_per_replica};
    uint64_t blocks = (total + 255u) / 256u;
    if (blocks > 262144u) blocks = 262144u;
    hipLaunchKernelGGL(fill_kernel, dim3(static_cast<uint32_t>(blocks)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), a);
    return static_cast<int>(hipGetLastError());
}

// Raw Philox4x32-10 blocks on the device: n counters (4 words each) and keys (2 words
// each) in, n output blocks (4 words each) out.  Used to check the integer stream
// against the host reference bit by bit.
int desloc_inputs_philox_raw(const uint32_t* d_ctr, const uint32_t* d_key, uint32_t* d_out,
                             uint64_t n, void* stream) {
    if (n == 0) return 0;
    hipLaunchKernelGGL(raw_kernel, dim3(static_cast<uint32_t>((n + 255u) / 256u)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), d_ctr, d_key, d_out, n);
    return static_cast<int>(hipGetLastError());
}

// Copies `bytes` (a multiple of 16) from src to dst on the device: reads exactly `bytes`
// and writes exactly `bytes`.  For calibrating FETCH_SIZE / WRITE_SIZE counters.
int desloc_inputs_calibration_copy(void* dst, const void* src, uint64_t bytes, void* stream) {
    if (bytes == 0) return 0;
    if (dst == nullptr || src == nullptr || bytes % 16u) return 1;
    const uint64_t n4 = bytes / 16u;
    uint64_t blocks = (n4 + 255u) / 256u;
    if (blocks > 65536u) blocks = 65536u;
    hipLaunchKernelGGL(calibration_copy_kernel, dim3(static_cast<uint32_t>(blocks)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const float4*>(src),
                       static_cast<float4*>(dst), n4);
    return static_cast<int>(hipGetLastError());
}

// One launch of a streaming yardstick: n_read read streams and n_write write streams of
// stream_bytes each (a multiple of 65536), stream k at base + k * stride_bytes; in place, the
// writes go to the first n_write read streams, otherwise to streams n_read .. n_read + n_write - 1.
// Shapes built: (1,0) (0,1) (1,1 not in place) and, in place, (3,2) (4,3) (16,12) (32,24).
// lds_bytes: dynamic-LDS request per 64-lane workgroup, never accessed (occupancy limiter, as
// in the step library).  paired: 1 = halves of each access 32 KiB apart (base and stride_bytes
// must then be multiples of 65536).  Returns 0, 1 for bad arguments, else the hipError_t.
int desloc_inputs_stream(void* base, uint64_t stride_bytes, uint64_t stream_bytes, int n_read, int n_write,
                         int inplace, int paired, uint32_t lds_bytes, void* stream) {
    uint32_t per_wave = 1;
    StreamKernelFn fn = pick_stream_kernel(n_read, n_write, inplace, &per_wave);
    if (fn == nullptr || base == nullptr || stream_bytes == 0 || stream_bytes % 65536u || stream_bytes > stride_bytes ||
        stream_bytes / 1024u > 0x3ffffffu || lds_bytes > 160u * 1024u)
        return 1;
    if (paired && (reinterpret_cast<uint64_t>(base) % 65536u || stride_bytes % 65536u)) return 1;
    if (lds_bytes > 65536u) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           static_cast<int>(lds_bytes));
        if (e != hipSuccess) return static_cast<int>(e);
    }
    StreamArgs a{reinterpret_cast<uint64_t>(base), stride_bytes, paired ? 1u : 0u};
    hipLaunchKernelGGL(fn, dim3(static_cast<uint32_t>(stream_bytes / 1024u / per_wave)), dim3(64), lds_bytes,
                       static_cast<hipStream_t>(stream), a);
    return static_cast<int>(hipGetLastError());
}

// The same block function on the host (no GPU needed), for known-answer tests.
void desloc_inputs_philox_host(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
    U4 c{ctr[0], ctr[1], ctr[2], ctr[3]};
    const U4 r = philox4x32_10(c, key[0], key[1]);
    out[0] = r.x; out[1] = r.y; out[2] = r.z; out[3] = r.w;
}

}  // extern "C"
