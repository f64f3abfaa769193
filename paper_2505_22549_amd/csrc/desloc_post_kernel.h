// DES-LOC step in the update-then-average ordering: the semantics of the listings the
// paper's proofs use (the SGDM appendix listing and the probabilistic DES-LOC-Adam listing),
// with the deterministic gates t mod K == 0 in place of their coin flips, and with the
// AMSGrad normaliser vt_t = max(v_t, vt_{t-1}) of the latter as an option.
//
//   u'^m = b1 u^m + (1-b1) gh^m          gated: u'^m <- E_m[u'^m]     (same for v with gh^2)
//   vt'^m = max(v'^m, vt^m)              (AMSGrad; per replica, never averaged itself)
//   x'^m = x^m - d(u'^m, v'^m or vt'^m)  gated: x'^m <- E_m[x'^m]
//
// Same mapping as the average-then-update kernel: one lane owns a 128-bit vector of elements
// for all M replicas, E_m[.] is an ascending-m register sum.  With a compile-time replica
// count everything stays in registers and every array is read once and written once.  With a
// runtime replica count the gradient is read twice on steps that gate u or v (first for the
// sums of the locally updated moments, then for the update itself); nothing else is re-read.
#pragma once

#include <type_traits>

#include "desloc_step_kernel.h"

namespace desloc {

template <int KIND>
__device__ __forceinline__ float post_direction(float un, float vsel, const StepScalars& sc) {
    if constexpr (KIND == KIND_SGDM) {
        return sc.lr * un;
    } else if constexpr (KIND == KIND_ADAM_LITERAL) {
        return fdiv(sc.lr, fsqrt(vsel + sc.eps2)) * un;
    } else {
        const float denom = fdiv(fsqrt(vsel), sc.sbc2) + sc.eps;
        return sc.step * fdiv(un, denom);
    }
}

template <int KIND, int MASK, int MT, bool BF16, bool AMS, int W, typename PTRS>
__device__ __forceinline__ void process_post(const PTRS& P, int Mrt, uint64_t e,
                                             const StepScalars& sc) {
    constexpr bool ADAM = KIND != KIND_SGDM;
    constexpr bool SX = (MASK & 1) != 0;
    constexpr bool SU = (MASK & 2) != 0;
    constexpr bool SV = ADAM && (MASK & 4) != 0;
    const int M = MT ? MT : Mrt;

    auto X = [&](int m) { return reinterpret_cast<float*>(P.get(ARR_X, m)) + e; };
    auto U = [&](int m) { return reinterpret_cast<float*>(P.get(ARR_U, m)) + e; };
    auto V = [&](int m) { return reinterpret_cast<float*>(P.get(ARR_V, m)) + e; };
    auto G = [&](int m) { return reinterpret_cast<const void*>(P.get(ARR_G, m)); };
    auto VT = [&](int m) -> float* {
        if constexpr (AMS) return reinterpret_cast<float*>(P.get(ARR_VMAX, m)) + e;
        else return nullptr;
    };

    if constexpr (MT != 0) {
        // ---- everything in registers: one read and one write per array ----
        float g[MT][W], x[MT][W], un[MT][W], vn[MT][W], vt[MT][W];
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            ld_grad<W, BF16>(g[m], G(m), e);
            ld_f32<W>(x[m], X(m));
            ld_f32<W>(un[m], U(m));
            if constexpr (ADAM) ld_f32<W>(vn[m], V(m));
            if constexpr (AMS) ld_f32<W>(vt[m], VT(m));
        }
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int j = 0; j < W; ++j) {
                const float gh = clip_coord(g[m][j] * P.gs(m), sc.rho);
                un[m][j] = sc.b1 * un[m][j] + sc.omb1 * gh;
                if constexpr (ADAM) vn[m][j] = sc.b2 * vn[m][j] + sc.omb2 * (gh * gh);
            }
#pragma unroll
        for (int j = 0; j < W; ++j) {
            if constexpr (SU) {
                float s = un[0][j];
#pragma unroll
                for (int m = 1; m < MT; ++m) s = s + un[m][j];
                s = s / sc.Mf;
#pragma unroll
                for (int m = 0; m < MT; ++m) un[m][j] = s;
            }
            if constexpr (SV) {
                float s = vn[0][j];
#pragma unroll
                for (int m = 1; m < MT; ++m) s = s + vn[m][j];
                s = s / sc.Mf;
#pragma unroll
                for (int m = 0; m < MT; ++m) vn[m][j] = s;
            }
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                float vsel = ADAM ? vn[m][j] : 0.0f;
                if constexpr (AMS) {
                    vsel = vn[m][j] > vt[m][j] ? vn[m][j] : vt[m][j];
                    vt[m][j] = vsel;
                }
                x[m][j] = x[m][j] - post_direction<KIND>(un[m][j], vsel, sc);
            }
            if constexpr (SX) {
                float s = x[0][j];
#pragma unroll
                for (int m = 1; m < MT; ++m) s = s + x[m][j];
                s = s / sc.Mf;
#pragma unroll
                for (int m = 0; m < MT; ++m) x[m][j] = s;
            }
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            st_f32<W>(X(m), x[m]);
            st_f32<W>(U(m), un[m]);
            if constexpr (ADAM) st_f32<W>(V(m), vn[m]);
            if constexpr (AMS) st_f32<W>(VT(m), vt[m]);
        }
    } else {
        // ---- runtime replica count: blocks of replicas, a block's loads in flight together ----
        // Sums start from -0.0f: (-0.0f) + s == s bit for bit, so each is the plain ascending sum.
        constexpr int RA = DESLOC_RT_PASS1_BLOCK, RB = DESLOC_RT_PASS2_BLOCK;
        float ubar[W], vbar[W], xbar[W];
#pragma unroll
        for (int j = 0; j < W; ++j) ubar[j] = vbar[j] = xbar[j] = -0.0f;
        if constexpr (SU || SV) {
            // pass A: ascending-m sums of the locally UPDATED gated moments
            for (int m0 = 0; m0 < M; m0 += RA) {
                float g[RA][W], tu[RA][W], tv[RA][W];
#pragma unroll
                for (int b = 0; b < RA; ++b) {
                    if (m0 + b < M) {
                        ld_grad<W, BF16>(g[b], G(m0 + b), e);
                        if constexpr (SU) ld_f32<W>(tu[b], U(m0 + b));
                        if constexpr (SV) ld_f32<W>(tv[b], V(m0 + b));
                    }
                }
#pragma unroll
                for (int b = 0; b < RA; ++b) {
                    if (m0 + b < M) {
                        const float gs = P.gs(m0 + b);
#pragma unroll
                        for (int j = 0; j < W; ++j) {
                            const float gh = clip_coord(g[b][j] * gs, sc.rho);
                            if constexpr (SU) ubar[j] = ubar[j] + (sc.b1 * tu[b][j] + sc.omb1 * gh);
                            if constexpr (SV) vbar[j] = vbar[j] + (sc.b2 * tv[b][j] + sc.omb2 * (gh * gh));
                        }
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < W; ++j) {
                if constexpr (SU) ubar[j] = ubar[j] / sc.Mf;
                if constexpr (SV) vbar[j] = vbar[j] / sc.Mf;
            }
        }
        // pass B: per replica update; ungated x is final, gated x is summed
        for (int m0 = 0; m0 < M; m0 += RB) {
            float g[RB][W], x[RB][W], u[RB][W], v[RB][W], vt[RB][W];
#pragma unroll
            for (int b = 0; b < RB; ++b) {
                if (m0 + b < M) {
                    const int m = m0 + b;
                    ld_grad<W, BF16>(g[b], G(m), e);
                    ld_f32<W>(x[b], X(m));
                    if constexpr (!SU) ld_f32<W>(u[b], U(m));
                    if constexpr (ADAM && !SV) ld_f32<W>(v[b], V(m));
                    if constexpr (AMS) ld_f32<W>(vt[b], VT(m));
                }
            }
#pragma unroll
            for (int b = 0; b < RB; ++b) {
                const int m = m0 + b;
                if (m >= M) continue;
                const float gs = P.gs(m);
                float uo[W], vo[W], xo[W];
#pragma unroll
                for (int j = 0; j < W; ++j) {
                    const float gh = clip_coord(g[b][j] * gs, sc.rho);
                    uo[j] = SU ? ubar[j] : sc.b1 * u[b][j] + sc.omb1 * gh;
                    vo[j] = !ADAM ? 0.0f : (SV ? vbar[j] : sc.b2 * v[b][j] + sc.omb2 * (gh * gh));
                    float vsel = vo[j];
                    if constexpr (AMS) {
                        vsel = vo[j] > vt[b][j] ? vo[j] : vt[b][j];
                        vt[b][j] = vsel;
                    }
                    xo[j] = x[b][j] - post_direction<KIND>(uo[j], vsel, sc);
                    if constexpr (SX) xbar[j] = xbar[j] + xo[j];
                }
                st_f32<W>(U(m), uo);
                if constexpr (ADAM) st_f32<W>(V(m), vo);
                if constexpr (AMS) st_f32<W>(VT(m), vt[b]);
                if constexpr (!SX) st_f32<W>(X(m), xo);
            }
        }
        if constexpr (SX) {
#pragma unroll
            for (int j = 0; j < W; ++j) xbar[j] = xbar[j] / sc.Mf;
            for (int m = 0; m < M; ++m) st_f32<W>(X(m), xbar);
        }
    }
}

template <int KIND, int MASK, int MT, bool BF16, bool AMS, bool STRIDED>
__global__ void DESLOC_STEP_KERNEL_ATTRS step_post_kernel(LaunchArgs a) {
    constexpr int NA = AMS ? N_ARRAYS : 4;
    const uint32_t c = blockIdx.x;
    uint64_t start;
    uint32_t len;
    const uint64_t* __restrict__ row = nullptr;
    const uint32_t Mrow = static_cast<uint32_t>(a.M);
    uint32_t lane_off = threadIdx.x * VEC, lane_step = TILE_ELEMS;
    bool second = false;
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

    auto run = [&](const auto& P, auto mt_tag) {
        constexpr int MTV = decltype(mt_tag)::value;
        for (uint32_t off = lane_off; off < len; off += lane_step) {
            auto Q = P;
            // pointer rows are read where they are used, not all ahead of the loop (see step_kernel)
            if constexpr (std::is_same<decltype(Q), TablePtrs>::value) asm volatile("" : "+s"(Q.row));
            if (off + VEC <= len) {
                process_post<KIND, MASK, MTV, BF16, AMS, VEC>(Q, a.M, start + off, a.sc);
            } else {
                for (uint32_t k = off; k < len; ++k)
                    process_post<KIND, MASK, MTV, BF16, AMS, 1>(Q, a.M, start + k, a.sc);
            }
        }
        if constexpr (MASK == 0) {
            if (second) process_post<KIND, MASK, MTV, BF16, AMS, VEC>(P, a.M, start + lane_off + TILE_ELEMS / 2, a.sc);
        }
    };

    if constexpr (MASK == 0) {
        // no gate: replicas are independent; replica-major launch (blockIdx.y = replica)
        RegPtrs<1, NA> R;
#pragma unroll
        for (int k = 0; k < NA; ++k) {
            if constexpr (STRIDED) R.p[k][0] = a.base[k] + blockIdx.y * a.rstride[k];
            else R.p[k][0] = row[k * Mrow + blockIdx.y];
        }
        R.g_scale[0] = a.gscale ? a.gscale[blockIdx.y] : 1.0f;
        run(R, std::integral_constant<int, 1>{});
    } else if constexpr (MT != 0 && STRIDED) {
        RegPtrs<MT, NA> R;
#pragma unroll
        for (int k = 0; k < NA; ++k)
#pragma unroll
            for (int m = 0; m < MT; ++m) R.p[k][m] = a.base[k] + static_cast<uint32_t>(m) * a.rstride[k];
#pragma unroll
        for (int m = 0; m < MT; ++m) R.g_scale[m] = a.gscale ? a.gscale[m] : 1.0f;
        run(R, std::integral_constant<int, MT>{});
    } else if constexpr (MT != 0) {
        run(TablePtrs{row, MT, a.gscale}, std::integral_constant<int, MT>{});
    } else {
        if constexpr (STRIDED) run(StridePtrs{a.base, a.rstride, a.gscale}, std::integral_constant<int, 0>{});
        else run(TablePtrs{row, a.M, a.gscale}, std::integral_constant<int, 0>{});
    }
}

template <int KIND, int MT, bool BF16, bool AMS, bool STRIDED>
struct PostMaskRow {
    static StepKernelFn get(uint32_t mask) {
        switch (mask) {
            case 0: return step_post_kernel<KIND, 0, 1, BF16, AMS, STRIDED>;
            case 1: return step_post_kernel<KIND, 1, MT, BF16, AMS, STRIDED>;
            case 2: return step_post_kernel<KIND, 2, MT, BF16, AMS, STRIDED>;
            case 3: return step_post_kernel<KIND, 3, MT, BF16, AMS, STRIDED>;
            default: break;
        }
        if constexpr (KIND != KIND_SGDM) {
            switch (mask) {
                case 4: return step_post_kernel<KIND, 4, MT, BF16, AMS, STRIDED>;
                case 5: return step_post_kernel<KIND, 5, MT, BF16, AMS, STRIDED>;
                case 6: return step_post_kernel<KIND, 6, MT, BF16, AMS, STRIDED>;
                case 7: return step_post_kernel<KIND, 7, MT, BF16, AMS, STRIDED>;
                default: break;
            }
        }
        return nullptr;
    }
};

template <int KIND, bool AMS>
StepKernelFn select_post_kernel(uint32_t mask, int M, int bf16, int strided) {
#define DESLOC_POST_PICK(MTV)                                                                    \
    if (bf16) return strided ? PostMaskRow<KIND, MTV, true, AMS, true>::get(mask)                \
                             : PostMaskRow<KIND, MTV, true, AMS, false>::get(mask);              \
    return strided ? PostMaskRow<KIND, MTV, false, AMS, true>::get(mask)                         \
                   : PostMaskRow<KIND, MTV, false, AMS, false>::get(mask);
    if (M == 4) { DESLOC_POST_PICK(4) }
    if (M == 8) { DESLOC_POST_PICK(8) }
    DESLOC_POST_PICK(0)
#undef DESLOC_POST_PICK
}

inline hipError_t launch_post_fn(StepKernelFn fn, uint32_t mask, const LaunchArgs& a, hipStream_t stream) {
    return launch_or_query(fn, mask, a, stream, nullptr);
}

}  // namespace desloc
