// The fused DES-LOC step kernel for gfx950 (CDNA4, wave64).
//
// One workgroup (one wave) owns one share of one segment: a chunk of consecutive elements or,
// under the paired mapping, two runs of 128 elements 32 KiB apart; its addresses come from the
// kernel arguments (strided layouts) or from a chunk record and a pointer row in device memory
// (table layouts).  One lane owns a 128-bit vector of 4 consecutive elements FOR ALL M REPLICAS.  The replica average
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
// Steps on which no gate fires (the vast majority) couple no replicas, so their launch is
// replica-major: grid.y walks the replicas and at any moment the whole GPU streams through
// one replica's g, x, u, v only.  In streaming micro-benchmarks on MI355X the achieved HBM
// bandwidth falls by about 4 % per doubling of the number of concurrently swept address
// streams; in this kernel 4 read + 3 write streams instead of 4M + 3M measured 1-3 % faster,
// and the no-gate path needs neither the replica loop nor M as a template parameter.
//
// The sync mask, the update rule, the gradient dtype and (for the common replica
// counts) M are template parameters: the mask is uniform over the launch, so there is
// no divergence and no code for gates that do not fire.
//
// Arithmetic is fp32, one IEEE rounding per operation in the order written here; this
// file must be compiled with -ffp-contract=off and correctly rounded divide / sqrt.
#pragma once

#include <type_traits>

#include "desloc_internal.h"

namespace desloc {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

// Every tensor pointer reaches the kernel as a 64-bit integer (kernel argument or table
// entry), so the compiler cannot see its address space and would emit FLAT accesses.
// All of them are global memory: say so, and get global_load / global_store.
#ifdef DESLOC_FLAT_ADDRESSING  // A/B switch for measurements only
#define DESLOC_GLOBAL
#else
#define DESLOC_GLOBAL __attribute__((address_space(1)))
#endif
template <typename T>
__device__ __forceinline__ const DESLOC_GLOBAL T* as_global(const void* p) {
    return (const DESLOC_GLOBAL T*)(p);
}
template <typename T>
__device__ __forceinline__ DESLOC_GLOBAL T* as_global(void* p) {
    return (DESLOC_GLOBAL T*)(p);
}

// Streaming (non-temporal) cache policy: nothing is reused, so loads should not displace
// other data on their way in.  Loads and stores are switched separately.
#ifndef DESLOC_NONTEMPORAL
#define DESLOC_NONTEMPORAL 1
#endif
// Store cache policy: 0 default, 1 non-temporal, 2 write-through at device scope ("sc1"),
// 3 write-through at system scope ("sc0 sc1").  Measured on MI355X with a 4-read/3-write
// in-place stream: 2 and 3 are ~7 % faster than 1, which is faster than 0: written lines
// that nobody will read again should leave the L2 at once instead of aging there as dirty
// lines whose later eviction interferes with the read stream.
#ifndef DESLOC_STORE_POLICY
#define DESLOC_STORE_POLICY 2
#endif
// Replicas whose loads are issued together in pass 2 before any store.  Measured on MI355X
// with single-wave workgroups and the paired mapping: 4 is 1-2 % faster than 1 and 2 on gated
// steps with M = 4 replicas (all of a wave's loads are then in flight at once) and ties with
// them for M = 8; 8 is 1 % slower there.
#ifndef DESLOC_PASS2_BLOCK
#define DESLOC_PASS2_BLOCK 4
#endif

// Runtime replica counts (any M without a compile-time instantiation): replicas whose gated
// states are loaded together in pass 1, and replicas per block in pass 2.  Measured on MI355X
// (M = 4 and M = 8 forced through this path): 4 and 1 match the compile-time instantiations
// to within 0.5 %; 2, 4 in pass 2 and 2, 8 in pass 1 are 1-3 % slower, also for M = 12, 16, 32
// (compared in one process on the same buffers: gated steps with many replicas vary by up
// to 10 % from process to process with the physical placement of their 7M streams).
#ifndef DESLOC_RT_PASS1_BLOCK
#define DESLOC_RT_PASS1_BLOCK 4
#endif
#ifndef DESLOC_RT_PASS2_BLOCK
#define DESLOC_RT_PASS2_BLOCK 1
#endif

template <int W>
__device__ __forceinline__ void ld_f32(float (&d)[W], const float* p) {
    if constexpr (W == 4) {
#if DESLOC_NONTEMPORAL
        v4f t = __builtin_nontemporal_load(as_global<v4f>(p));
#else
        v4f t = *as_global<v4f>(p);
#endif
        d[0] = t.x; d[1] = t.y; d[2] = t.z; d[3] = t.w;
    } else {
        d[0] = *as_global<float>(p);
    }
}

template <int W>
__device__ __forceinline__ void st_f32(float* p, const float (&s)[W]) {
    if constexpr (W == 4) {
        v4f t = {s[0], s[1], s[2], s[3]};
#if DESLOC_STORE_POLICY == 1
        __builtin_nontemporal_store(t, as_global<v4f>(p));
#elif DESLOC_STORE_POLICY == 2
        // No builtin sets the scope bits of a 128-bit plain store, hence inline assembly.
        // The compiler cannot see inside it, so two of its duties are done by hand:
        //  - a store of more than 64 bits must not be followed at once by a VALU write to
        //    its data registers (the hazard recognizer would insert wait states): s_nop;
        //  - s_waitcnt bookkeeping: an extra outstanding store can only make the
        //    compiler's vmcnt(N) waits more conservative, never too weak.
        asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 2" ::"v"(as_global<v4f>(p)), "v"(t) : "memory");
#elif DESLOC_STORE_POLICY == 3
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 2" ::"v"(as_global<v4f>(p)), "v"(t) : "memory");
#else
        *as_global<v4f>(p) = t;
#endif
    } else {
        *as_global<float>(p) = s[0];
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
            v2u t = __builtin_nontemporal_load(as_global<v2u>(p));
#else
            v2u t = *as_global<v2u>(p);
#endif
            d[0] = widen_bf16(t.x & 0xffffu);
            d[1] = widen_bf16(t.x >> 16);
            d[2] = widen_bf16(t.y & 0xffffu);
            d[3] = widen_bf16(t.y >> 16);
        } else {
            d[0] = widen_bf16(*as_global<uint16_t>(p));
        }
    }
}

// Experimental: hardware reciprocal / square root (1 ulp) instead of the correctly rounded
// sequences.  Off by default: results are then no longer bit-identical to an IEEE host.
#ifndef DESLOC_APPROX_DIV_SQRT
#define DESLOC_APPROX_DIV_SQRT 0
#endif
__device__ __forceinline__ float fdiv(float a, float b) {
#if DESLOC_APPROX_DIV_SQRT
    return a * __builtin_amdgcn_rcpf(b);
#else
    return a / b;
#endif
}
__device__ __forceinline__ float fsqrt(float a) {
#if DESLOC_APPROX_DIV_SQRT
    return __builtin_amdgcn_sqrtf(a);
#else
    return sqrtf(a);
#endif
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
// gs is the replica's norm-clip factor (exactly 1 when clipping is coordinate-wise, and then
// the product is exact; in norm mode the host passes rho = +inf so clip_coord is the identity).
template <int KIND>
__device__ __forceinline__ void update_coord(float g, float gs, float xin, float uin, float vin,
                                             float vnorm, const StepScalars& sc, float& xo,
                                             float& uo, float& vo) {
    const float gh = clip_coord(g * gs, sc.rho);
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
            xo = xin - fdiv(sc.lr, fsqrt(vn + sc.eps2)) * un;
        } else {
            const float denom = fdiv(fsqrt(vn), sc.sbc2) + sc.eps;
            xo = xin - sc.step * fdiv(un, denom);
        }
    } else if constexpr (KIND == KIND_ADOPT_T0) {
        vo = gh * gh;
        uo = uin;
        xo = xin;
    } else {  // KIND_ADOPT, KIND_ADOPT_AVGNORM
        const float root = fsqrt(vnorm);
        const float nrm = root > sc.eps ? root : sc.eps;
        const float vn = sc.b2 * vin + sc.omb2 * (gh * gh);
        const float mn = sc.b1 * uin + sc.omb1 * fdiv(gh, nrm);
        vo = vn;
        uo = mn;
        xo = xin - sc.lr * mn;
    }
}

// Where a lane finds the base pointer of array a (0 x, 1 u, 2 v, 3 g) of replica m.
// TablePtrs reads the segment's pointer row in device memory (any M); RegPtrs holds a
// compile-time number of replicas in scalar registers, filled once per workgroup.
//
// The pointer table and the norm-clip factors are written before the launch and never during
// it.  Reading them through the constant address space tells the compiler so: the reads stay
// scalar loads (s_load through the scalar cache) even after the kernel's own stores, instead
// of becoming uniform vector loads at full memory latency ahead of every block of replicas.
template <typename T>
__device__ __forceinline__ T ld_const(const T* p) {
    return *(const __attribute__((address_space(4))) T*)(p);
}
struct TablePtrs {
    const uint64_t* __restrict__ row;  // row[a * M + m]
    int M;
    const float* __restrict__ gscale;  // null: factor 1
    __device__ __forceinline__ uint64_t get(int a, int m) const { return ld_const(row + (a * M + m)); }
    __device__ __forceinline__ float gs(int m) const { return gscale ? ld_const(gscale + m) : 1.0f; }
};
// Strided layouts with a runtime replica count: base + m * stride, formed in scalar registers
// (no table load ahead of the vector loads).
struct StridePtrs {
    const uint64_t* base;     // [N_ARRAYS], kernel arguments
    const uint64_t* rstride;  // [N_ARRAYS]
    const float* __restrict__ gscale;
    __device__ __forceinline__ uint64_t get(int a, int m) const {
        return base[a] + static_cast<uint64_t>(static_cast<uint32_t>(m)) * rstride[a];
    }
    __device__ __forceinline__ float gs(int m) const { return gscale ? ld_const(gscale + m) : 1.0f; }
};
template <int N, int NA = 4>
struct RegPtrs {
    uint64_t p[NA][N];
    float g_scale[N];
    __device__ __forceinline__ uint64_t get(int a, int m) const { return p[a][m]; }
    __device__ __forceinline__ float gs(int m) const { return g_scale[m]; }
};

// All M replicas of W consecutive elements starting at element e of a segment.
template <int KIND, int MASK, int MT, bool BF16, int W, typename PTRS>
__device__ __forceinline__ void process(const PTRS& P, int Mrt, uint64_t e,
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
    constexpr int B = MT ? (MT < DESLOC_PASS2_BLOCK ? MT : DESLOC_PASS2_BLOCK) : DESLOC_RT_PASS2_BLOCK;
    const int M = MT ? MT : Mrt;

    auto X = [&](int m) { return reinterpret_cast<float*>(P.get(0, m)) + e; };
    auto U = [&](int m) { return reinterpret_cast<float*>(P.get(1, m)) + e; };
    auto V = [&](int m) { return reinterpret_cast<float*>(P.get(2, m)) + e; };
    auto G = [&](int m) { return reinterpret_cast<const void*>(P.get(3, m)); };

    float xbar[W], ubar[W], vbar[W];
    float vkeep[KM][W];
#pragma unroll
    for (int j = 0; j < W; ++j) xbar[j] = ubar[j] = vbar[j] = 0.0f;

    // ---- pass 1: ascending-m sums of the gated states, then one division by M ----
    if constexpr ((SX || SU || SV) && MT != 0) {
        float t[W];
        if constexpr (SX) ld_f32<W>(xbar, X(0));
        if constexpr (SU) ld_f32<W>(ubar, U(0));
        if constexpr (SV) {
            ld_f32<W>(vbar, V(0));
            if constexpr (LOCAL_V_NORM) {
#pragma unroll
                for (int j = 0; j < W; ++j) vkeep[0][j] = vbar[j];
            }
        }
#pragma unroll
        for (int m = 1; m < MT; ++m) {
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
                if constexpr (LOCAL_V_NORM) {
#pragma unroll
                    for (int j = 0; j < W; ++j) vkeep[m][j] = t[j];
                }
#pragma unroll
                for (int j = 0; j < W; ++j) vbar[j] = vbar[j] + t[j];
            }
        }
    }
    if constexpr ((SX || SU || SV) && MT == 0) {
        // Runtime replica count: blocks of RB replicas, all loads of a block in flight together,
        // then added in ascending m.  The sums start from -0.0f, the one value with
        // (-0.0f) + s == s bit for bit for every s, so the result is the plain ascending sum.
        constexpr int RB = DESLOC_RT_PASS1_BLOCK;
#pragma unroll
        for (int j = 0; j < W; ++j) xbar[j] = ubar[j] = vbar[j] = -0.0f;
        for (int m0 = 0; m0 < M; m0 += RB) {
            float tx[RB][W], tu[RB][W], tv[RB][W];
#pragma unroll
            for (int b = 0; b < RB; ++b) {
                if (m0 + b < M) {
                    if constexpr (SX) ld_f32<W>(tx[b], X(m0 + b));
                    if constexpr (SU) ld_f32<W>(tu[b], U(m0 + b));
                    if constexpr (SV) ld_f32<W>(tv[b], V(m0 + b));
                }
            }
#pragma unroll
            for (int b = 0; b < RB; ++b) {
                if (m0 + b < M) {
#pragma unroll
                    for (int j = 0; j < W; ++j) {
                        if constexpr (SX) xbar[j] = xbar[j] + tx[b][j];
                        if constexpr (SU) ubar[j] = ubar[j] + tu[b][j];
                        if constexpr (SV) vbar[j] = vbar[j] + tv[b][j];
                    }
                }
            }
        }
    }
    if constexpr (SX || SU || SV) {
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
            if (MT != 0 || m < M) {
                ld_grad<W, BF16>(g[b], G(m), e);
                if constexpr (TOUCH_X && !SX) ld_f32<W>(x[b], X(m));
                if constexpr (TOUCH_U && !SU) ld_f32<W>(u[b], U(m));
                if constexpr (READ_V && !SV) ld_f32<W>(v[b], V(m));
                if constexpr (LOCAL_V_NORM && MT == 0) ld_f32<W>(vn[b], V(m));
            }
        }
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const int m = m0 + b;
            if (MT == 0 && m >= M) continue;
            float xo[W], uo[W], vo[W];
#pragma unroll
            for (int j = 0; j < W; ++j) {
                const float xin = SX ? xbar[j] : (TOUCH_X ? x[b][j] : 0.0f);
                const float uin = SU ? ubar[j] : (TOUCH_U ? u[b][j] : 0.0f);
                const float vin = SV ? vbar[j] : (READ_V ? v[b][j] : 0.0f);
                float vnorm = vin;
                if constexpr (LOCAL_V_NORM) vnorm = MT ? vkeep[MT ? m : 0][j] : vn[b][j];
                update_coord<KIND>(g[b][j], P.gs(m), xin, uin, vin, vnorm, sc, xo[j], uo[j], vo[j]);
            }
            if constexpr (TOUCH_X) st_f32<W>(X(m), xo);
            if constexpr (TOUCH_U) st_f32<W>(U(m), uo);
            if constexpr (HAS_V) st_f32<W>(V(m), vo);
        }
    }
}

// Vectors per lane whose loads are issued together on the replica-major (no gate) path.
#ifndef DESLOC_LOCAL_UNROLL
#define DESLOC_LOCAL_UNROLL 2
#endif

// One replica, no gate: VU independent 4-vectors per lane, vstride elements apart, all loads
// before any store.
template <int KIND, bool BF16, int VU>
__device__ __forceinline__ void process_local(float* __restrict__ x, float* __restrict__ u,
                                              float* __restrict__ v, const void* __restrict__ gp,
                                              float gs, uint64_t start, uint32_t off0,
                                              uint32_t vstride, const StepScalars& sc) {
    constexpr bool HAS_V = KIND != KIND_SGDM;
    constexpr bool TOUCH_XU = KIND != KIND_ADOPT_T0;
    constexpr bool READ_V = HAS_V && KIND != KIND_ADOPT_T0;
    float g[VU][VEC], xi[VU][VEC], ui[VU][VEC], vi[VU][VEC];
#pragma unroll
    for (int j = 0; j < VU; ++j) {
        const uint64_t e = start + off0 + static_cast<uint32_t>(j) * vstride;
        ld_grad<VEC, BF16>(g[j], gp, e);
        if constexpr (TOUCH_XU) ld_f32<VEC>(xi[j], x + e);
        if constexpr (TOUCH_XU) ld_f32<VEC>(ui[j], u + e);
        if constexpr (READ_V) ld_f32<VEC>(vi[j], v + e);
    }
#pragma unroll
    for (int j = 0; j < VU; ++j) {
        const uint64_t e = start + off0 + static_cast<uint32_t>(j) * vstride;
        float xo[VEC], uo[VEC], vo[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const float vin = READ_V ? vi[j][k] : 0.0f;
            update_coord<KIND>(g[j][k], gs, TOUCH_XU ? xi[j][k] : 0.0f, TOUCH_XU ? ui[j][k] : 0.0f,
                               vin, vin, sc, xo[k], uo[k], vo[k]);
        }
        if constexpr (TOUCH_XU) st_f32<VEC>(x + e, xo);
        if constexpr (TOUCH_XU) st_f32<VEC>(u + e, uo);
        if constexpr (HAS_V) st_f32<VEC>(v + e, vo);
    }
}

// A workgroup's share of a strided segment.  Lanes run
//   for (off = lane_off; off < len; off += lane_step)   over elements start + off .. + VEC.
// Contiguous chunks: lane_off = 4 * lane, lane_step = one tile.  Paired mapping (see
// PAIR_GROUP_ELEMS): start is the group's first element, len the group size, every lane has
// exactly one full vector (lane_step = len ends the loop after it).
struct Share {
    uint64_t start;
    uint32_t len;
    uint32_t lane_off;
    uint32_t lane_step;
};
static_assert(STEP_WG_THREADS == 64 && TILE_ELEMS == 256, "the paired mapping assumes single-wave workgroups");

__device__ __forceinline__ Share strided_share(const LaunchArgs& a, uint32_t c) {
    Share w;
    if (c < a.pair_blocks) {
        w.start = a.pair_e0 + static_cast<uint64_t>(c >> PAIR_WAVES_LOG2) * PAIR_GROUP_ELEMS;
        w.len = PAIR_GROUP_ELEMS;
        w.lane_off = (threadIdx.x >> 5) * PAIR_HALF_ELEMS + (c & (PAIR_WAVES - 1u)) * (TILE_ELEMS / 2) +
                     (threadIdx.x & 31u) * VEC;
        w.lane_step = PAIR_GROUP_ELEMS;
        return w;
    }
    const uint32_t j = c - a.pair_blocks;
    uint64_t end;
    if (j < a.head_chunks) {
        w.start = static_cast<uint64_t>(j) * a.chunk_elems;
        end = a.pair_e0;
    } else {
        w.start = a.pair_e1 + static_cast<uint64_t>(j - a.head_chunks) * a.chunk_elems;
        end = a.numel0;
    }
    const uint64_t left = end - w.start;
    w.len = left < a.chunk_elems ? static_cast<uint32_t>(left) : a.chunk_elems;
    w.lane_off = threadIdx.x * VEC;
    w.lane_step = TILE_ELEMS;
    return w;
}

// A workgroup's share on table layouts: 2^split_log2 workgroups share one chunk record.  Plain
// records are cut into equal pieces; a paired record (PAIRED_REC_FLAG) holds two wave slots of a
// group: one per workgroup when split (gated steps, Adam / ADOPT steps without a gate), both
// for one workgroup otherwise (SGDM steps without a gate: `second` is then set and the lane's
// second vector lies half a tile further).  Paired records only exist with the default two-tile
// records, for which the host always splits gated launches, so only the launches without a
// gate look at `second`.
struct TableShare {
    Share w;
    uint32_t seg;
    bool empty;
    bool second;
};

__device__ __forceinline__ TableShare table_share(const LaunchArgs& a, uint32_t c) {
    const ChunkRec rec = a.chunks[c >> a.split_log2];
    const uint32_t sub = c & ((1u << a.split_log2) - 1u);
    TableShare t;
    t.seg = rec.seg;
    t.empty = false;
    t.second = false;
    if (rec.len & PAIRED_REC_FLAG) {
        const uint32_t slot = 2u * (rec.len & PAIRED_REC_SLOT_MASK) + sub;
        t.w.start = rec.start;
        t.w.len = PAIR_GROUP_ELEMS;
        t.w.lane_off = (threadIdx.x >> 5) * PAIR_HALF_ELEMS + slot * (TILE_ELEMS / 2) + (threadIdx.x & 31u) * VEC;
        t.w.lane_step = PAIR_GROUP_ELEMS;
        t.second = a.split_log2 == 0;
        return t;
    }
    const uint32_t piece = a.chunk_elems >> a.split_log2;
    const uint32_t first = sub * piece;
    if (first >= rec.len) {  // this share of a short record is empty
        t.empty = true;
        return t;
    }
    t.w.start = rec.start + first;
    t.w.len = rec.len - first < piece ? rec.len - first : piece;
    t.w.lane_off = threadIdx.x * VEC;
    t.w.lane_step = TILE_ELEMS;
    return t;
}

// STRIDED: a single segment whose replica pointers are base[a] + m * rstride[a] (one packed
// buffer per replica, the common case): chunk bounds and every address follow from kernel
// arguments alone, so the first vector load is not behind any dependent table load.
// Otherwise: one 16-byte chunk record, then the segment's pointer row.
// The occupancy limiter keeps at most 14 single-wave workgroups on a compute unit (4 per SIMD),
// so a wave may use up to 128 vector registers.  Saying so matters: without the hint the
// compiler schedules for 8 waves per SIMD (64 registers) and, in the instantiations with the
// most loads in flight, serialises pass 1 into load - wait - add chains, one memory round trip
// per replica and state.
#define DESLOC_STEP_KERNEL_ATTRS __launch_bounds__(STEP_WG_THREADS) __attribute__((amdgpu_waves_per_eu(1, 4)))

template <int KIND, int MASK, int MT, bool BF16, bool STRIDED>
__global__ void DESLOC_STEP_KERNEL_ATTRS step_kernel(LaunchArgs a) {
    const uint32_t c = blockIdx.x;
    uint64_t start;
    uint32_t len;
    const uint64_t* __restrict__ row = nullptr;
    const uint32_t Mrow = static_cast<uint32_t>(a.M);
    uint32_t lane_off = threadIdx.x * VEC, lane_step = TILE_ELEMS;
    bool second = false;  // a paired record's second wave slot is this workgroup's too
    if constexpr (STRIDED) {
        const Share w = strided_share(a, c);
        start = w.start;
        len = w.len;
        lane_off = w.lane_off;
        lane_step = w.lane_step;
    } else {
        const TableShare t = table_share(a, c);
        if (t.empty) return;
        start = t.w.start;
        len = t.w.len;
        lane_off = t.w.lane_off;
        lane_step = t.w.lane_step;
        second = t.second;
        row = a.ptrs + static_cast<uint64_t>(t.seg) * N_ARRAYS * Mrow;
    }

    if constexpr (MASK == 0) {
        // replica-major: blockIdx.y is the replica
#ifdef DESLOC_UNGATED_SLEEP  // A/B switch for measurements only
        if constexpr (STRIDED) __builtin_amdgcn_s_sleep(DESLOC_UNGATED_SLEEP);
#endif
        RegPtrs<1> R;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if constexpr (STRIDED) R.p[k][0] = a.base[k] + blockIdx.y * a.rstride[k];
            else R.p[k][0] = row[k * Mrow + blockIdx.y];
        }
        float* x = reinterpret_cast<float*>(R.p[0][0]);
        float* u = reinterpret_cast<float*>(R.p[1][0]);
        float* v = reinterpret_cast<float*>(R.p[2][0]);
        const void* g = reinterpret_cast<const void*>(R.p[3][0]);
        R.g_scale[0] = a.gscale ? a.gscale[blockIdx.y] : 1.0f;
        const float gs = R.g_scale[0];
        constexpr int VU = DESLOC_LOCAL_UNROLL;
#ifdef DESLOC_PROBE_LOAD  // A/B switch for measurements only: a dependent scalar read ahead of the vector loads
        if constexpr (STRIDED) {
            // the first element this wave will read (paired shares: its slot inside the group)
            const uint64_t e0 = start + (lane_step == PAIR_GROUP_ELEMS && DESLOC_PROBE_LOAD == 2 ? (c & (PAIR_WAVES - 1u)) * (TILE_ELEMS / 2) : 0u);
            const uint32_t* pp = reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(g) + e0 * (BF16 ? 2 : 4));
            uint32_t probe = ld_const(pp);
            asm volatile("s_waitcnt lgkmcnt(0)" ::"s"(probe) : "memory");
        }
#endif
        uint32_t off = lane_off;
        if (lane_step == TILE_ELEMS) {
            for (; off + (VU - 1) * TILE_ELEMS + VEC <= len; off += VU * TILE_ELEMS)
                process_local<KIND, BF16, VU>(x, u, v, g, gs, start, off, TILE_ELEMS, a.sc);
        } else if (second) {
            process_local<KIND, BF16, 2>(x, u, v, g, gs, start, off, TILE_ELEMS / 2, a.sc);
            off += lane_step;
        }
        for (; off < len; off += lane_step) {
            if (off + VEC <= len) {
                process_local<KIND, BF16, 1>(x, u, v, g, gs, start, off, TILE_ELEMS, a.sc);
            } else {
                for (uint32_t k = off; k < len; ++k)
                    process<KIND, 0, 1, BF16, 1>(R, 1, start + k, a.sc);
            }
        }
    } else if constexpr (MT != 0 && STRIDED) {
        // All 4 * MT addresses formed once, in scalar registers.  (Forming each at its use
        // instead, as the table path below does, measured within 0.3 % of this on MI355X.)
        RegPtrs<MT> R;
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int m = 0; m < MT; ++m) R.p[k][m] = a.base[k] + static_cast<uint32_t>(m) * a.rstride[k];
#pragma unroll
        for (int m = 0; m < MT; ++m) R.g_scale[m] = a.gscale ? a.gscale[m] : 1.0f;
        for (uint32_t off = lane_off; off < len; off += lane_step) {
            if (off + VEC <= len) {
                process<KIND, MASK, MT, BF16, VEC>(R, MT, start + off, a.sc);
            } else {
                // ragged tail of the segment: 1..3 elements, one at a time
                for (uint32_t k = off; k < len; ++k)
                    process<KIND, MASK, MT, BF16, 1>(R, MT, start + k, a.sc);
            }
        }
    } else if constexpr (MT != 0) {
        // 4 * MT pointers of 64 bits do not fit the scalar register file next to everything
        // else (MT = 8: the compiler spilled them to vector lanes and serialised the loads
        // behind the reloads; steps that gate one state of 8 separately allocated replicas ran
        // 10 % slower than those that gate all three).  Each use reads its pointer from the row
        // instead, through the scalar cache; making the row opaque once per iteration keeps the
        // compiler from hoisting all 4 * MT reads to the top again.
        for (uint32_t off = lane_off; off < len; off += lane_step) {
            const uint64_t* r = row;
            asm volatile("" : "+s"(r));
            const TablePtrs T{r, MT, a.gscale};
            if (off + VEC <= len) {
                process<KIND, MASK, MT, BF16, VEC>(T, MT, start + off, a.sc);
            } else {
                for (uint32_t k = off; k < len; ++k)
                    process<KIND, MASK, MT, BF16, 1>(T, MT, start + k, a.sc);
            }
        }
    } else {
        // runtime replica count: addresses from the stride (strided layouts) or from the
        // segment's pointer row in the device table
        auto run = [&](const auto& T) {
            for (uint32_t off = lane_off; off < len; off += lane_step) {
                if (off + VEC <= len) {
                    process<KIND, MASK, 0, BF16, VEC>(T, a.M, start + off, a.sc);
                } else {
                    for (uint32_t k = off; k < len; ++k)
                        process<KIND, MASK, 0, BF16, 1>(T, a.M, start + k, a.sc);
                }
            }
        };
        if constexpr (STRIDED) run(StridePtrs{a.base, a.rstride, a.gscale});
        else run(TablePtrs{row, a.M, a.gscale});
    }
}

typedef void (*StepKernelFn)(LaunchArgs);

// Launches fn over the decomposition in `a`.  With resident_out, nothing is launched: the
// runtime is asked how many workgroups of fn one compute unit holds under this launch's
// dynamic-LDS request (the occupancy limiter), and the answer is stored there.
inline hipError_t launch_or_query(StepKernelFn fn, uint32_t mask, const LaunchArgs& a, hipStream_t stream,
                                  uint32_t* resident_out) {
    if (fn == nullptr) return hipErrorInvalidValue;
    if (a.lds_bytes > 65536u) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           static_cast<int>(a.lds_bytes));
        if (e != hipSuccess) return e;
    }
    if (resident_out != nullptr) {
        int blocks = 0;
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, reinterpret_cast<const void*>(fn),
                                                                    STEP_WG_THREADS, a.lds_bytes);
        if (e != hipSuccess) return e;
        *resident_out = blocks < 0 ? 0u : static_cast<uint32_t>(blocks);
        return hipSuccess;
    }
    hipLaunchKernelGGL(fn, dim3(a.n_chunks, mask == 0 ? a.M : 1), dim3(STEP_WG_THREADS), a.lds_bytes, stream, a);
    return hipGetLastError();
}

// Compile-time replica counts; any other M takes the runtime-M instantiation (MT = 0).
template <int KIND, int MT, bool BF16, bool STRIDED>
struct MaskRow {
    static StepKernelFn get(uint32_t mask) {
        switch (mask) {
            case 0: return step_kernel<KIND, 0, 1, BF16, STRIDED>;  // replica-major, any M
            case 1: return step_kernel<KIND, 1, MT, BF16, STRIDED>;
            case 2: return step_kernel<KIND, 2, MT, BF16, STRIDED>;
            case 3: return step_kernel<KIND, 3, MT, BF16, STRIDED>;
            default: break;
        }
        if constexpr (KIND != KIND_SGDM) {
            switch (mask) {
                case 4: return step_kernel<KIND, 4, MT, BF16, STRIDED>;
                case 5: return step_kernel<KIND, 5, MT, BF16, STRIDED>;
                case 6: return step_kernel<KIND, 6, MT, BF16, STRIDED>;
                case 7: return step_kernel<KIND, 7, MT, BF16, STRIDED>;
                default: break;
            }
        }
        return nullptr;
    }
};

template <int KIND, int MT>
StepKernelFn pick_dtype_layout(uint32_t mask, int bf16, int strided) {
    if (bf16) return strided ? MaskRow<KIND, MT, true, true>::get(mask) : MaskRow<KIND, MT, true, false>::get(mask);
    return strided ? MaskRow<KIND, MT, false, true>::get(mask) : MaskRow<KIND, MT, false, false>::get(mask);
}

template <int KIND>
StepKernelFn select_kernel(uint32_t mask, int M, int bf16, int strided) {
#ifndef DESLOC_NO_FIXED_M  // A/B switch for measurements: every M through the runtime loop
    if (M == 4) return pick_dtype_layout<KIND, 4>(mask, bf16, strided);
    if (M == 8) return pick_dtype_layout<KIND, 8>(mask, bf16, strided);
#endif
    return pick_dtype_layout<KIND, 0>(mask, bf16, strided);
}

}  // namespace desloc
