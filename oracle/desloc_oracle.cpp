// DES-LOC CPU oracle  --  TEST INFRASTRUCTURE, NOT PRODUCT CODE.
//
// A plain, single-threaded, element-at-a-time implementation of the DES-LOC
// per-step optimizer update on M worker replicas with one sync period per
// state (paper: Alg. 1 generic method; Alg. 2 DES-LOC-Adam; Alg. 3
// DES-LOC-ADOPT; SGDM as Alg. 1 with a single momentum state whose update
// form is the one shown in the DES-LOC-SGDM listing of the SGDM appendix).
//
// Only tests, the smoke check and the benchmark's cpu_baseline leg may load
// this file's library.  It shares no code, header, table or constant with the
// HIP library: it declares its own config struct and its own ABI below.
//
// Every function here follows the listings in their own order and notation:
//   x  parameters, u first moment (m in the ADOPT listing), v second moment,
//   g  gradient, gh clipped gradient, M workers, t step (0-based),
//   Kx, Ku, Kv sync periods, E_m[.] uniform mean over the M workers.
// There is no blocking, vectorisation, threading or fusion.
//
// Arithmetic type R is float (the parity reference for the fp32 GPU path) or
// double (used by the CPU pins to separate formula errors from rounding).
// Compile WITHOUT fast-math and WITHOUT fp contraction so that every
// operation below is one IEEE-754 rounding in the order written.
//
// Canonical operation order (the paper fixes none; this is the builder's
// reading, listed in the design notes):
//   clip      gh   = copysign(min(|g|, rho), g)                 (Sec. 2.1 clip)
//             norm mode (what the paper's model table says the experiments used, no formula
//             printed; builder's reading = the usual global-norm clip): per worker m,
//             nrm = (R) sqrt( sum_i (double) g_i^2 )  over ALL coordinates, in coordinate order,
//             sc  = nrm > rho ? rho / nrm : 1 ;  gh_i = g_i * sc   (no coordinate clip then)
//   mean      sbar = (((s^0 + s^1) + s^2) + ... + s^{M-1}) / (R)M
//   Adam      u' = b1*uin + (1-b1)*gh ; v' = b2*vin + (1-b2)*(gh*gh)
//             default:  x' = xin - step*(u'/(sqrt(v')/sbc2 + eps))
//                       step = lr/(1-b1^(t+1)), sbc2 = sqrt(1-b2^(t+1))
//                       (bias-corrected Adam as cited by the paper, Eq. (1-2);
//                        the two per-step scalars are formed in double and
//                        rounded once to R)
//             literal:  x' = xin - (lr/sqrt(v' + eps*eps))*u'   (Alg. 2 as printed)
//   ADOPT     nrm = max(sqrt(v_local_prev), eps)   [flag: mean of v when v syncs]
//             v' = b2*vin + (1-b2)*(gh*gh) ; m' = b1*min + (1-b1)*(gh/nrm)
//             x' = xin - lr*m'                                   (Alg. 3)
//             flag init_g0sq, t == 0 only: v' = gh*gh, m' = min, x' = xin
//   SGDM      u' = b*uin + (1-b)*gh ; x' = xin - lr*u'
// where sin = E_m[s_prev] if the state's gate fires at t, else the worker's
// own s_prev (average-then-update, exactly as Alg. 1-3 place the mean).
//
// post_average mode = the ordering of the listings used by the proofs (SGDM appendix listing
// and the probabilistic DES-LOC-Adam listing), with the deterministic gates t mod K == 0 in
// place of their coin flips: every worker first updates locally, then a gated state is
// replaced by the mean of the UPDATED values,
//   u'^m = b1*u^m + (1-b1)*gh^m ;  gated: u'^m <- E_m[u'^m]        (same for v with gh*gh)
//   amsgrad (Adam only): vt'^m = max(v'^m, vt^m), vt_{-1} = v_{-1}; the direction uses vt'
//   d^m from u'^m and v'^m (or vt'^m) by the same direction formulas as above
//   x'^m = x^m - d^m ;  gated: x'^m <- E_m[x'^m]
// so that all workers hold identical bits of a state right after its sync.
//
// Pins (tests/, "not gpu"): sync-count closed forms and the paper's printed
// communication ratios; reduction to torch.optim.Adam / torch.optim.SGD and a
// textbook ADOPT loop for M = 1 and for identical gradients; constant-gradient
// closed forms; replica-mean dynamics from the SGDM and Adam appendices;
// clip bounds of the max-change lemma; brute force from Alg. 1's generic form
// on tiny inputs; planted-mistake checks; norm mode against
// torch.nn.utils.clip_grad_norm_ semantics (scale = rho/norm when norm > rho).
// parity unpinned: the ADOPT literal first step (division by eps because
// v_{-1} = 0) and the local-vs-mean normaliser choice on a v-sync step are
// fixed only by the printed listing and the builder's reading of it.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

extern "C" {

enum { ORACLE_ADAM = 0, ORACLE_ADOPT = 1, ORACLE_SGDM = 2 };

typedef struct oracle_cfg {
    int32_t variant;      // ORACLE_ADAM / ORACLE_ADOPT / ORACLE_SGDM
    int32_t M;            // number of workers (replicas), >= 1
    uint64_t Kx, Ku, Kv;  // sync periods; 0 encodes "never" (K = infinity)
    double lr;            // eta_t for this step
    double beta1, beta2;  // decay factors (beta1 = momentum for SGDM)
    double eps;           // Adam eps / lambda, ADOPT epsilon
    double rho;           // clip radius; +inf disables the clip
    int32_t adam_literal;          // 1: Alg. 2 exactly as printed (no bias correction)
    int32_t adopt_avg_normaliser;  // 1: ADOPT normaliser uses E_m[v] on a v-sync step
    int32_t adopt_init_g0sq;       // 1: at t = 0, v_0 = gh^2 and no parameter move
    int32_t norm_clip;             // 1: global-L2-norm clip per worker instead of the coordinate clip
    int32_t post_average;          // 1: update-then-average ordering (Adam and SGDM only)
    int32_t amsgrad;               // 1: AMSGrad normaliser max(v_t, vt_{t-1}) (post_average Adam only)
} oracle_cfg;

// Gate of Alg. 1: state j is averaged at step t iff t mod K_j == 0.
// bit0 = x, bit1 = u, bit2 = v (never set for SGDM, which has no v).
uint32_t oracle_sync_mask(const oracle_cfg* c, uint64_t t) {
    uint32_t mask = 0;
    if (c->Kx != 0 && t % c->Kx == 0) mask |= 1u;
    if (c->Ku != 0 && t % c->Ku == 0) mask |= 2u;
    if (c->variant != ORACLE_SGDM && c->Kv != 0 && t % c->Kv == 0) mask |= 4u;
    return mask;
}

// Number of steps in [0, T) on which a state with period K is averaged.
uint64_t oracle_sync_count(uint64_t T, uint64_t K) {
    uint64_t n = 0;
    for (uint64_t t = 0; t < T; ++t)
        if (K != 0 && t % K == 0) ++n;
    return n;
}

// bf16 -> fp32 widening of a gradient (exact: bf16 is the top half of fp32).
float oracle_widen_bf16(uint16_t h) {
    uint32_t bits = static_cast<uint32_t>(h) << 16;
    float f;
    std::memcpy(&f, &bits, sizeof f);
    return f;
}

}  // extern "C"

namespace {

// Coordinate-wise clip of Sec. 2.1: sgn(g) * min(|g|, rho).
template <typename R>
R clip_coord(R g, R rho) {
    R a = std::fabs(g);
    R c = a < rho ? a : rho;
    return std::copysign(c, g);
}

// E_m[s]: ascending-m sequential sum, then one division by M.
template <typename R>
R worker_mean(const R* s, uint64_t n, uint64_t i, int M) {
    R sum = s[i];
    for (int m = 1; m < M; ++m) sum = sum + s[static_cast<uint64_t>(m) * n + i];
    return sum / static_cast<R>(M);
}

// Sum of squares of one worker's gradient in double, coordinate order.
template <typename R>
double sum_squares(const R* g, uint64_t n) {
    double ss = 0.0;
    for (uint64_t i = 0; i < n; ++i) ss += static_cast<double>(g[i]) * static_cast<double>(g[i]);
    return ss;
}

// Hyper-parameters and per-step scalars in the arithmetic type R.
template <typename R>
struct Scalars {
    R b1, b2, omb1, omb2, lr, eps, rho;
    R step;  // lr / (1 - b1^(t+1))
    R sbc2;  // sqrt(1 - b2^(t+1))
};

template <typename R>
Scalars<R> make_scalars(const oracle_cfg* c, uint64_t t) {
    Scalars<R> s;
    s.b1 = static_cast<R>(c->beta1);
    s.b2 = static_cast<R>(c->beta2);
    s.omb1 = static_cast<R>(1) - s.b1;
    s.omb2 = static_cast<R>(1) - s.b2;
    s.lr = static_cast<R>(c->lr);
    s.eps = static_cast<R>(c->eps);
    s.rho = static_cast<R>(c->rho);
    // Per-step scalars of bias-corrected Adam, exponent t+1 because the loop
    // is 0-based and the states are seeded at t = -1.
    const double tp1 = static_cast<double>(t) + 1.0;
    const double bc1 = 1.0 - std::pow(static_cast<double>(s.b1), tp1);
    const double bc2 = 1.0 - std::pow(static_cast<double>(s.b2), tp1);
    s.step = static_cast<R>(static_cast<double>(s.lr) / bc1);
    s.sbc2 = static_cast<R>(std::sqrt(bc2));
    return s;
}

// Norm-based clipping: per-worker factor (1 when the mode is off or the norm is within rho).
// sumsq_rest (may be null): per worker, the sum of squares of gradient coordinates that are
// NOT among the n passed here, so that a run on a subset of the coordinates can use the norm
// of the whole gradient.  norms_out (may be null) receives the per-worker norm.
template <typename R>
std::vector<R> norm_clip_factors(const oracle_cfg* c, uint64_t n, const R* g, R rho,
                                 const double* sumsq_rest, R* norms_out) {
    const int M = c->M;
    std::vector<R> gscale(static_cast<size_t>(M), static_cast<R>(1));
    if (c->norm_clip) {
        for (int m = 0; m < M; ++m) {
            double ss = sum_squares(g + static_cast<uint64_t>(m) * n, n);
            if (sumsq_rest) ss += sumsq_rest[m];
            const R nrm = static_cast<R>(std::sqrt(ss));
            gscale[m] = nrm > rho ? rho / nrm : static_cast<R>(1);
            if (norms_out) norms_out[m] = nrm;
        }
    }
    return gscale;
}

// gh^m for coordinate i of every worker: norm mode scales, otherwise the coordinate clip.
template <typename R>
void clipped_gradients(const oracle_cfg* c, uint64_t n, uint64_t i, const R* g,
                       const std::vector<R>& gscale, R rho, std::vector<R>& gh) {
    for (int m = 0; m < c->M; ++m) {
        const R gm = g[static_cast<uint64_t>(m) * n + i];
        gh[m] = c->norm_clip ? gm * gscale[m] : clip_coord(gm, rho);
    }
}

// Adam direction d from the (possibly averaged / maximised) moments.
template <typename R>
R adam_direction(const oracle_cfg* c, const Scalars<R>& s, R un, R vsel) {
    if (c->adam_literal) return (s.lr / std::sqrt(vsel + s.eps * s.eps)) * un;
    const R denom = std::sqrt(vsel) / s.sbc2 + s.eps;
    return s.step * (un / denom);
}

// One DES-LOC step over n coordinates.  Arrays are [M][n], worker-major.
// x, u, v are updated in place; g is read only.  v may be null for SGDM.
// sumsq_rest / norms_out: see norm_clip_factors.
template <typename R>
void step_impl(const oracle_cfg* c, uint64_t t, uint64_t n, R* x, R* u, R* v, const R* g,
               const double* sumsq_rest, R* norms_out) {
    const int M = c->M;
    const uint32_t mask = oracle_sync_mask(c, t);
    const bool sx = mask & 1u, su = mask & 2u, sv = mask & 4u;
    const Scalars<R> s = make_scalars<R>(c, t);
    const R b1 = s.b1, b2 = s.b2, omb1 = s.omb1, omb2 = s.omb2, lr = s.lr, eps = s.eps, rho = s.rho;

    std::vector<R> gh(static_cast<size_t>(M));
    const std::vector<R> gscale = norm_clip_factors(c, n, g, rho, sumsq_rest, norms_out);

    for (uint64_t i = 0; i < n; ++i) {
        clipped_gradients(c, n, i, g, gscale, rho, gh);

        // Means of the PREVIOUS values of every gated state.
        const R xbar = sx ? worker_mean(x, n, i, M) : static_cast<R>(0);
        const R ubar = su ? worker_mean(u, n, i, M) : static_cast<R>(0);
        const R vbar = sv ? worker_mean(v, n, i, M) : static_cast<R>(0);

        for (int m = 0; m < M; ++m) {
            const uint64_t k = static_cast<uint64_t>(m) * n + i;
            const R xin = sx ? xbar : x[k];
            const R uin = su ? ubar : u[k];

            if (c->variant == ORACLE_SGDM) {
                const R un = b1 * uin + omb1 * gh[m];
                u[k] = un;
                x[k] = xin - lr * un;
                continue;
            }

            const R vprev = v[k];
            const R vin = sv ? vbar : vprev;

            if (c->variant == ORACLE_ADAM) {
                const R un = b1 * uin + omb1 * gh[m];
                const R vn = b2 * vin + omb2 * (gh[m] * gh[m]);
                u[k] = un;
                v[k] = vn;
                x[k] = xin - adam_direction(c, s, un, vn);
            } else {  // ORACLE_ADOPT
                if (c->adopt_init_g0sq && t == 0) {
                    v[k] = gh[m] * gh[m];
                    u[k] = uin;
                    x[k] = xin;
                    continue;
                }
                const R vnorm = (c->adopt_avg_normaliser && sv) ? vbar : vprev;
                const R root = std::sqrt(vnorm);
                const R nrm = root > eps ? root : eps;
                const R vn = b2 * vin + omb2 * (gh[m] * gh[m]);
                const R mn = b1 * uin + omb1 * (gh[m] / nrm);
                v[k] = vn;
                u[k] = mn;
                x[k] = xin - lr * mn;
            }
        }
    }
}

// Ascending sequential sum of M values, then one division by M.
template <typename R>
R mean_of(const std::vector<R>& a, int M) {
    R sum = a[0];
    for (int m = 1; m < M; ++m) sum = sum + a[m];
    return sum / static_cast<R>(M);
}

// One DES-LOC step in the update-then-average ordering (see the header comment).
// vmax is the AMSGrad state vt ([M][n]; may be null unless c->amsgrad).
template <typename R>
void step_post_impl(const oracle_cfg* c, uint64_t t, uint64_t n, R* x, R* u, R* v, R* vmax,
                    const R* g, const double* sumsq_rest, R* norms_out) {
    const int M = c->M;
    const uint32_t mask = oracle_sync_mask(c, t);
    const bool sx = mask & 1u, su = mask & 2u, sv = mask & 4u;
    const bool adam = c->variant == ORACLE_ADAM;
    const Scalars<R> s = make_scalars<R>(c, t);
    const R b1 = s.b1, b2 = s.b2, omb1 = s.omb1, omb2 = s.omb2, lr = s.lr, rho = s.rho;
    const std::vector<R> gscale = norm_clip_factors(c, n, g, rho, sumsq_rest, norms_out);

    std::vector<R> gh(M), un(M), vn(M), xl(M);
    for (uint64_t i = 0; i < n; ++i) {
        clipped_gradients(c, n, i, g, gscale, rho, gh);
        // local moment updates, then the mean of the updated values where gated
        for (int m = 0; m < M; ++m) un[m] = b1 * u[static_cast<uint64_t>(m) * n + i] + omb1 * gh[m];
        if (su) {
            const R ubar = mean_of(un, M);
            for (int m = 0; m < M; ++m) un[m] = ubar;
        }
        if (adam) {
            for (int m = 0; m < M; ++m)
                vn[m] = b2 * v[static_cast<uint64_t>(m) * n + i] + omb2 * (gh[m] * gh[m]);
            if (sv) {
                const R vbar = mean_of(vn, M);
                for (int m = 0; m < M; ++m) vn[m] = vbar;
            }
        }
        // direction and local parameter step
        for (int m = 0; m < M; ++m) {
            const uint64_t k = static_cast<uint64_t>(m) * n + i;
            R d;
            if (adam) {
                R vsel = vn[m];
                if (c->amsgrad) {
                    const R prev = vmax[k];
                    vsel = vn[m] > prev ? vn[m] : prev;
                    vmax[k] = vsel;
                }
                d = adam_direction(c, s, un[m], vsel);
                v[k] = vn[m];
            } else {
                d = lr * un[m];
            }
            u[k] = un[m];
            xl[m] = x[k] - d;
        }
        if (sx) {
            const R xbar = mean_of(xl, M);
            for (int m = 0; m < M; ++m) xl[m] = xbar;
        }
        for (int m = 0; m < M; ++m) x[static_cast<uint64_t>(m) * n + i] = xl[m];
    }
}

template <typename R>
void mean_impl(int M, uint64_t n, const R* s, R* out) {
    for (uint64_t i = 0; i < n; ++i) out[i] = worker_mean(s, n, i, M);
}

}  // namespace

extern "C" {

void oracle_step_f32(const oracle_cfg* c, uint64_t t, uint64_t n, float* x, float* u, float* v,
                     const float* g) {
    step_impl<float>(c, t, n, x, u, v, g, nullptr, nullptr);
}

void oracle_step_f64(const oracle_cfg* c, uint64_t t, uint64_t n, double* x, double* u, double* v,
                     const double* g) {
    step_impl<double>(c, t, n, x, u, v, g, nullptr, nullptr);
}

// Norm-clip variants: see step_impl for sumsq_rest / norms_out (either may be null).
void oracle_step_norm_f32(const oracle_cfg* c, uint64_t t, uint64_t n, float* x, float* u, float* v,
                          const float* g, const double* sumsq_rest, float* norms_out) {
    step_impl<float>(c, t, n, x, u, v, g, sumsq_rest, norms_out);
}

void oracle_step_norm_f64(const oracle_cfg* c, uint64_t t, uint64_t n, double* x, double* u,
                          double* v, const double* g, const double* sumsq_rest, double* norms_out) {
    step_impl<double>(c, t, n, x, u, v, g, sumsq_rest, norms_out);
}

// Update-then-average ordering (cfg->post_average must be 1; ADOPT is not defined for it and
// is ignored: nothing is written).  vmax: AMSGrad state, null unless cfg->amsgrad.
void oracle_step_post_f32(const oracle_cfg* c, uint64_t t, uint64_t n, float* x, float* u, float* v,
                          float* vmax, const float* g, const double* sumsq_rest, float* norms_out) {
    if (c->variant == ORACLE_ADOPT) return;
    step_post_impl<float>(c, t, n, x, u, v, vmax, g, sumsq_rest, norms_out);
}

void oracle_step_post_f64(const oracle_cfg* c, uint64_t t, uint64_t n, double* x, double* u,
                          double* v, double* vmax, const double* g, const double* sumsq_rest,
                          double* norms_out) {
    if (c->variant == ORACLE_ADOPT) return;
    step_post_impl<double>(c, t, n, x, u, v, vmax, g, sumsq_rest, norms_out);
}

// Relative rate of change of a state (Sec. 4, "Metrics"): per worker m,
//   change[m] = || s^m - ref^m ||_2   and   base[m] = || ref^m ||_2
// so that change/base = ||s_{t+K} - s_t||_2 / ||s_t||_2 when ref is the state K steps earlier.
// Sums in double, coordinate order, one rounding to float at the end.
void oracle_state_change_f32(int32_t M, uint64_t n, const float* s, const float* ref, float* change,
                             float* base) {
    for (int m = 0; m < M; ++m) {
        double dd = 0.0, rr = 0.0;
        for (uint64_t i = 0; i < n; ++i) {
            const double a = static_cast<double>(s[static_cast<uint64_t>(m) * n + i]);
            const double b = static_cast<double>(ref[static_cast<uint64_t>(m) * n + i]);
            dd += (a - b) * (a - b);
            rr += b * b;
        }
        change[m] = static_cast<float>(std::sqrt(dd));
        base[m] = static_cast<float>(std::sqrt(rr));
    }
}

// The same diagnostic per tensor (the paper's rate-of-change figure is drawn per state from
// per-tensor values): tensor k is the coordinate range [start_k, start_k + numel[k]) with
// start_k the sum of the earlier sizes.  change[k * M + m] = || s^m - ref^m ||_2 over tensor k,
// base[k * M + m] = || ref^m ||_2 over tensor k; a tensor of size 0 gives 0 and 0.
// n is the row length of s and ref (>= the sum of the sizes).
void oracle_state_change_tensors_f32(int32_t M, uint64_t n_tensors, const uint64_t* numel, uint64_t n,
                                     const float* s, const float* ref, float* change, float* base) {
    uint64_t start = 0;
    for (uint64_t k = 0; k < n_tensors; ++k) {
        for (int m = 0; m < M; ++m) {
            double dd = 0.0, rr = 0.0;
            for (uint64_t i = start; i < start + numel[k]; ++i) {
                const double a = static_cast<double>(s[static_cast<uint64_t>(m) * n + i]);
                const double b = static_cast<double>(ref[static_cast<uint64_t>(m) * n + i]);
                dd += (a - b) * (a - b);
                rr += b * b;
            }
            change[k * static_cast<uint64_t>(M) + m] = static_cast<float>(std::sqrt(dd));
            base[k * static_cast<uint64_t>(M) + m] = static_cast<float>(std::sqrt(rr));
        }
        start += numel[k];
    }
}

// The averaged iterate E_m[s^m] used by the paper's analysis.
void oracle_worker_mean_f32(int32_t M, uint64_t n, const float* s, float* out) {
    mean_impl<float>(M, n, s, out);
}

void oracle_worker_mean_f64(int32_t M, uint64_t n, const double* s, double* out) {
    mean_impl<double>(M, n, s, out);
}

}  // extern "C"
