// The fused DES-LOC step kernel for gfx950 (CDNA4, wave64).
//
// One workgroup owns one chunk of consecutive elements of one segment; one lane owns
// a 128-bit vector of 4 consecutive elements FOR ALL M REPLICAS.  The replica average
// E_m[.] of a gated state (Alg. 1) is therefore an ascending-m sum in that lane's
// registers: deterministic, no atomics, no LDS, no cross-lane traffic, and it adds no
// memory traffic because the M values are the ones the update reads anyway.
//
// Two passes over the replicas:
//   pass 1  loads only the gated states of every replica and sums them;
//   pass 2  loads the gradient and the non-gated states, applies the update and stores.
// On a gated step the new state depends on the mean and the worker's own gradient only
// (s_t^m = UPDATE(E_m[s_{t-1}], gh^m)), so a gated state is read exactly once in pass 1
// and never again: every array is read once and written once on every kind of step.
// (Exception: Alg. 3's normaliser uses the worker's own previous v even when v is gated;
// the compile-time-M instantiations keep it in registers, the runtime-M one reloads it.)
//
// The sync mask, the update rule, the gradient dtype and (for the common replica
// counts) M are template parameters: the mask is uniform over the launch, so there is
// no divergence and no code for gates that do not fire.
//
// Arithmetic is fp32, one IEEE rounding per operation in the order written here; this
// file must be compiled with -ffp-contract=off and correctly rounded divide / sqrt.
#pragma once

#include "desloc_internal.h"

namespace desloc {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

#ifndef DESLOC_NONTEMPORAL
#define DESLOC_NONTEMPORAL 1
#endif
// Replicas whose loads are issued together in pass 2 before any store.
#ifndef DESLOC_PASS2_BLOCK
#define DESLOC_PASS2_BLOCK 4
#endif

template <int W>
__device__ __forceinline__ void ld_f32(float (&d)[W], const float* p) {
    if constexpr (W == 4) {
#if DESLOC_NONTEMPORAL
        v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
#else
        v4f t = *reinterpret_cast<const v4f*>(p);
#endif
        d[0] = t.x; d[1] = t.y; d[2] = t.z; d[3] = t.w;
    } else {
        d[0] = *p;
    }
}

template <int W>
__device__ __forceinline__ void st_f32(float* p, const float (&s)[W]) {
    if constexpr (W == 4) {
        v4f t = {s[0], s[1], s[2], s[3]};
#if DESLOC_NONTEMPORAL
        __builtin_nontemporal_store(t, reinterpret_cast<v4f*>(p));
#else
        *reinterpret_cast<v4f*>(p) = t;
#endif
    } else {
        *p = s[0];
    }
}

__device__ __forceinline__ float widen_bf16(uint32_t h16) { return __uint_as_float(h16 << 16); }

// Gradient load: fp32, or bf16 widened exactly (bf16 is the upper half of fp32).
template <int W, bool BF16>
__device__ __forceinline__ void ld_grad(float (&d)[W], const void* base, uint64_t e) {
    if constexpr (!BF16) {
        ld_f32<W>(d, reinterpret_cast<const float*>(base) + e);
    } else {
        const uint16_t* p = reinterpret_cast<const uint16_t*>(base) + e;
        if constexpr (W == 4) {
#if DESLOC_NONTEMPORAL
            v2u t = __builtin_nontemporal_load(reinterpret_cast<const v2u*>(p));
#else
            v2u t = *reinterpret_cast<const v2u*>(p);
#endif
            d[0] = widen_bf16(t.x & 0xffffu);
            d[1] = widen_bf16(t.x >> 16);
            d[2] = widen_bf16(t.y & 0xffffu);
            d[3] = widen_bf16(t.y >> 16);
        } else {
            d[0] = widen_bf16(*p);
        }
    }
}

// Coordinate-wise clip of Sec. 2.1: sgn(g) * min(|g|, rho).
__device__ __forceinline__ float clip_coord(float g, float rho) {
    float a = fabsf(g);
    float c = a < rho ? a : rho;
    return copysignf(c, g);
}

// The per-coordinate update of one worker.  xin / uin / vin are the worker's previous
// values, already replaced by the replica mean where the state is gated.  vnorm is the
// value Alg. 3's normaliser takes the root of.
template <int KIND>
__device__ __forceinline__ void update_coord(float g, float xin, float uin, float vin, float vnorm,
                                             const StepScalars& sc, float& xo, float& uo,
                                             float& vo) {
    const float gh = clip_coord(g, sc.rho);
    if constexpr (KIND == KIND_SGDM) {
        const float un = sc.b1 * uin + sc.omb1 * gh;
        uo = un;
        xo = xin - sc.lr * un;
        vo = 0.0f;
    } else if constexpr (KIND == KIND_ADAM || KIND == KIND_ADAM_LITERAL) {
        const float un = sc.b1 * uin + sc.omb1 * gh;
        const float vn = sc.b2 * vin + sc.omb2 * (gh * gh);
        uo = un;
        vo = vn;
        if constexpr (KIND == KIND_ADAM_LITERAL) {
            xo = xin - (sc.lr / sqrtf(vn + sc.eps2)) * un;
        } else {
            const float denom = sqrtf(vn) / sc.sbc2 + sc.eps;
            xo = xin - sc.step * (un / denom);
        }
    } else if constexpr (KIND == KIND_ADOPT_T0) {
        vo = gh * gh;
        uo = uin;
        xo = xin;
    } else {  // KIND_ADOPT, KIND_ADOPT_AVGNORM
        const float root = sqrtf(vnorm);
        const float nrm = root > sc.eps ? root : sc.eps;
        const float vn = sc.b2 * vin + sc.omb2 * (gh * gh);
        const float mn = sc.b1 * uin + sc.omb1 * (gh / nrm);
        vo = vn;
        uo = mn;
        xo = xin - sc.lr * mn;
    }
}

// All M replicas of W consecutive elements starting at element e of a segment.
// P is the segment's pointer row: P[a * M + m], a = 0 (x), 1 (u), 2 (v), 3 (g).
template <int KIND, int MASK, int MT, bool BF16, int W>
__device__ __forceinline__ void process(const uint64_t* __restrict__ P, int Mrt, uint64_t e,
                                        const StepScalars& sc) {
    constexpr bool HAS_V = KIND != KIND_SGDM;
    constexpr bool SX = (MASK & 1) != 0;
    constexpr bool SU = (MASK & 2) != 0;
    constexpr bool SV = HAS_V && (MASK & 4) != 0;
    // ADOPT's first step with v_0 = gh^2 leaves x and u at their incoming value: an
    // ungated x or u is then neither read nor written.
    constexpr bool TOUCH_X = SX || KIND != KIND_ADOPT_T0;
    constexpr bool TOUCH_U = SU || KIND != KIND_ADOPT_T0;
    constexpr bool READ_V = HAS_V && KIND != KIND_ADOPT_T0;
    constexpr bool LOCAL_V_NORM = (KIND == KIND_ADOPT) && SV;  // own previous v although v is gated
    constexpr int KM = MT ? MT : 1;
    constexpr int B = MT ? (MT < DESLOC_PASS2_BLOCK ? MT : DESLOC_PASS2_BLOCK) : DESLOC_PASS2_BLOCK;
    const int M = MT ? MT : Mrt;

    auto X = [&](int m) { return reinterpret_cast<float*>(P[0 * M + m]) + e; };
    auto U = [&](int m) { return reinterpret_cast<float*>(P[1 * M + m]) + e; };
    auto V = [&](int m) { return reinterpret_cast<float*>(P[2 * M + m]) + e; };
    auto G = [&](int m) { return reinterpret_cast<const void*>(P[3 * M + m]); };

    float xbar[W], ubar[W], vbar[W];
    float vkeep[KM][W];
#pragma unroll
    for (int j = 0; j < W; ++j) xbar[j] = ubar[j] = vbar[j] = 0.0f;

    // ---- pass 1: ascending-m sums of the gated states, then one division by M ----
    if constexpr (SX || SU || SV) {
        float t[W];
        if constexpr (SX) ld_f32<W>(xbar, X(0));
        if constexpr (SU) ld_f32<W>(ubar, U(0));
        if constexpr (SV) {
            ld_f32<W>(vbar, V(0));
            if constexpr (LOCAL_V_NORM && MT != 0) {
#pragma unroll
                for (int j = 0; j < W; ++j) vkeep[0][j] = vbar[j];
            }
        }
#pragma unroll MT ? MT : 1
        for (int m = 1; m < M; ++m) {
            if constexpr (SX) {
                ld_f32<W>(t, X(m));
#pragma unroll
                for (int j = 0; j < W; ++j) xbar[j] = xbar[j] + t[j];
            }
            if constexpr (SU) {
                ld_f32<W>(t, U(m));
#pragma unroll
                for (int j = 0; j < W; ++j) ubar[j] = ubar[j] + t[j];
            }
            if constexpr (SV) {
                ld_f32<W>(t, V(m));
                if constexpr (LOCAL_V_NORM && MT != 0) {
#pragma unroll
                    for (int j = 0; j < W; ++j) vkeep[m][j] = t[j];
                }
#pragma unroll
                for (int j = 0; j < W; ++j) vbar[j] = vbar[j] + t[j];
            }
        }
#pragma unroll
        for (int j = 0; j < W; ++j) {
            if constexpr (SX) xbar[j] = xbar[j] / sc.Mf;
            if constexpr (SU) ubar[j] = ubar[j] / sc.Mf;
            if constexpr (SV) vbar[j] = vbar[j] / sc.Mf;
        }
    }

    // ---- pass 2: blocks of B replicas: all loads of the block, then update + store ----
#pragma unroll MT ? MT : 1
    for (int m0 = 0; m0 < M; m0 += B) {
        float g[B][W], x[B][W], u[B][W], v[B][W], vn[B][W];
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const int m = m0 + b;
            if (MT == 0 && m >= M) break;
            ld_grad<W, BF16>(g[b], G(m), e);
            if constexpr (TOUCH_X && !SX) ld_f32<W>(x[b], X(m));
            if constexpr (TOUCH_U && !SU) ld_f32<W>(u[b], U(m));
            if constexpr (READ_V && !SV) ld_f32<W>(v[b], V(m));
            if constexpr (LOCAL_V_NORM && MT == 0) ld_f32<W>(vn[b], V(m));
        }
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const int m = m0 + b;
            if (MT == 0 && m >= M) break;
            float xo[W], uo[W], vo[W];
#pragma unroll
            for (int j = 0; j < W; ++j) {
                const float xin = SX ? xbar[j] : (TOUCH_X ? x[b][j] : 0.0f);
                const float uin = SU ? ubar[j] : (TOUCH_U ? u[b][j] : 0.0f);
                const float vin = SV ? vbar[j] : (READ_V ? v[b][j] : 0.0f);
                float vnorm = vin;
                if constexpr (LOCAL_V_NORM) vnorm = MT ? vkeep[MT ? m : 0][j] : vn[b][j];
                update_coord<KIND>(g[b][j], xin, uin, vin, vnorm, sc, xo[j], uo[j], vo[j]);
            }
            if constexpr (TOUCH_X) st_f32<W>(X(m), xo);
            if constexpr (TOUCH_U) st_f32<W>(U(m), uo);
            if constexpr (HAS_V) st_f32<W>(V(m), vo);
        }
    }
}

// blockIdx -> chunk.  Workgroups are dealt round-robin to the 8 XCDs (blockIdx % 8);
// with remap on, XCD j works through one contiguous range of chunks, which keeps each
// XCD's L2 / TLB working set to a few contiguous windows per array instead of the whole
// buffer.  The map is a bijection on [0, n) for any n.
__device__ __forceinline__ uint32_t chunk_of_block(uint32_t bid, uint32_t n, int remap) {
    if (!remap) return bid;
    const uint32_t q = n >> 3, r = n & 7u;
    const uint32_t xcd = bid & 7u, slot = bid >> 3;
    return xcd * q + (xcd < r ? xcd : r) + slot;
}

template <int KIND, int MASK, int MT, bool BF16>
__global__ void __launch_bounds__(WG_THREADS) step_kernel(LaunchArgs a) {
    const uint32_t c = chunk_of_block(blockIdx.x, a.n_chunks, a.xcd_remap);
    const uint32_t s = a.chunk_seg[c];
    const uint64_t numel = a.segs[s].numel;
    const uint64_t start = (static_cast<uint64_t>(c) - a.segs[s].chunk0) * a.chunk_elems;
    const uint64_t left = numel - start;
    const uint32_t len = left < a.chunk_elems ? static_cast<uint32_t>(left) : a.chunk_elems;
    const int M = MT ? MT : a.M;
    const uint64_t* __restrict__ P = a.ptrs + static_cast<uint64_t>(s) * 4u * M;

    for (uint32_t off = threadIdx.x * VEC; off < len; off += TILE_ELEMS) {
        if (off + VEC <= len) {
            process<KIND, MASK, MT, BF16, VEC>(P, a.M, start + off, a.sc);
        } else {
            // ragged tail of the segment: 1..3 elements, one at a time
            for (uint32_t k = off; k < len; ++k)
                process<KIND, MASK, MT, BF16, 1>(P, a.M, start + k, a.sc);
        }
    }
}

typedef void (*StepKernelFn)(LaunchArgs);

// Compile-time replica counts; index 0 is the runtime-M instantiation.
constexpr int MT_LIST[] = {0, 2, 4, 8};
constexpr int MT_COUNT = 4;

template <int KIND, int MT, bool BF16>
struct MaskRow {
    static StepKernelFn get(uint32_t mask) {
        switch (mask) {
            case 0: return step_kernel<KIND, 0, MT, BF16>;
            case 1: return step_kernel<KIND, 1, MT, BF16>;
            case 2: return step_kernel<KIND, 2, MT, BF16>;
            case 3: return step_kernel<KIND, 3, MT, BF16>;
            default: break;
        }
        if constexpr (KIND != KIND_SGDM) {
            switch (mask) {
                case 4: return step_kernel<KIND, 4, MT, BF16>;
                case 5: return step_kernel<KIND, 5, MT, BF16>;
                case 6: return step_kernel<KIND, 6, MT, BF16>;
                case 7: return step_kernel<KIND, 7, MT, BF16>;
                default: break;
            }
        }
        return nullptr;
    }
};

template <int KIND>
StepKernelFn select_kernel(uint32_t mask, int M, int bf16) {
    int mt = 0;
    for (int i = 1; i < MT_COUNT; ++i)
        if (MT_LIST[i] == M) mt = MT_LIST[i];
#define DESLOC_PICK(MTV)                                          \
    if (mt == MTV)                                                \
        return bf16 ? MaskRow<KIND, MTV, true>::get(mask)         \
                    : MaskRow<KIND, MTV, false>::get(mask);
    DESLOC_PICK(2)
    DESLOC_PICK(4)
    DESLOC_PICK(8)
    DESLOC_PICK(0)
#undef DESLOC_PICK
    return nullptr;
}

}  // namespace desloc
