// Internal declarations shared by the host dispatch and the gfx950 kernels of the
// DES-LOC step library.  Not part of the public ABI (that is include/desloc.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace desloc {

// Update rule selected on the host from (variant, flags, t).
enum Kind : int {
    KIND_ADAM = 0,        // bias-corrected Adam direction (Eq. 1-2 + the cited Adam step)
    KIND_ADAM_LITERAL,    // Alg. 2 as printed: eta * u / sqrt(v + lambda^2)
    KIND_ADOPT,           // Alg. 3, normaliser from the worker's own previous v
    KIND_ADOPT_AVGNORM,   // Alg. 3, normaliser from E_m[v] when v is gated
    KIND_ADOPT_T0,        // first step of ADOPT with v_0 = gh^2 and no parameter move
    KIND_SGDM,            // Alg. 1 with one momentum state
    KIND_COUNT
};

// The step kernels run as single-wave workgroups: they never synchronise across waves, and
// one-wave granularity lets the LDS occupancy limiter set the resident waves per CU in steps
// of one (the optimum on MI355X lies between 8 and 14 per CU, by kernel path and kind of step:
// the table beside the limiter constants of the host dispatch; 256-lane workgroups can only
// offer 8, 12, 16 and lose 3-8 % of HBM throughput).
#ifndef DESLOC_WG_THREADS
#define DESLOC_WG_THREADS 64
#endif
enum {
    STEP_WG_THREADS = DESLOC_WG_THREADS,   // step / post-average step kernels
    WG_THREADS = 256,                      // reductions, initialisation, means
    VEC = 4,
    TILE_ELEMS = STEP_WG_THREADS * VEC,    // elements one step workgroup covers per pass
    AUX_TILE_ELEMS = WG_THREADS * VEC
};

// Paired mapping of strided layouts.  When the bases of all fp32 streams (every array, every
// replica) are congruent modulo PAIR_GROUP_BYTES, the elements between the first and the last
// PAIR_GROUP_BYTES boundary are handed out in groups of PAIR_GROUP_ELEMS: wave w of a group
// covers two runs of 128 elements (512 bytes) that lie PAIR_HALF_ELEMS apart, lanes 0-31 the
// first and lanes 32-63 the second, so that the two halves of every 1 KiB vector access differ
// in address bit 15 only.  Measured on MI355X (M = 8 replicas, 56 concurrently swept streams):
// gated steps 5.65 -> 6.6 TB/s, ungated steps +1 %; pairs that differ in any other single bit
// (4 KiB ... 512 MiB apart) or that also differ in bit 16 (groups not aligned) are slower than
// plain contiguous 1 KiB accesses, so this is a property of this chip's address interleaving
// and the mapping is only used when the alignment condition holds.
enum : uint32_t {
    PAIR_WAVES_LOG2 = 6,
    PAIR_WAVES = 1u << PAIR_WAVES_LOG2,            // waves (workgroups) per group
    PAIR_HALF_ELEMS = 8192,                        // 32 KiB of fp32
    PAIR_GROUP_ELEMS = 2 * PAIR_HALF_ELEMS,        // 64 KiB of fp32
    PAIR_GROUP_BYTES = PAIR_GROUP_ELEMS * 4,
    // Table layouts: a chunk record whose len has this bit set covers the wave slots 2j and 2j + 1
    // (j = len & PAIRED_REC_SLOT_MASK) of the group that starts at element `start` of its segment:
    // 512 elements as two runs of 256, PAIR_HALF_ELEMS apart.
    PAIRED_REC_FLAG = 0x80000000u,
    PAIRED_REC_SLOT_MASK = 0xffffu
};

// Arrays per replica, in pointer-table order: x, u, v, g, vmax (AMSGrad state, optional).
enum { ARR_X = 0, ARR_U = 1, ARR_V = 2, ARR_G = 3, ARR_VMAX = 4, N_ARRAYS = 5 };

// One workgroup's share of a segment, in device memory (multi-segment layouts only).
// Pointers live in a separate table ptrs[segment][array (N_ARRAYS of them)][replica].
struct ChunkRec {
    uint64_t start;  // first element within the segment
    uint32_t seg;    // segment index
    uint32_t len;    // elements in this chunk (<= chunk_elems), or PAIRED_REC_FLAG | slot pair
};

// Scalars of one step, formed on the host (bias terms in double, rounded once).
struct StepScalars {
    float b1, omb1;   // beta1, 1 - beta1
    float b2, omb2;   // beta2, 1 - beta2
    float lr;         // eta_t
    float eps;        // eps / lambda / epsilon
    float eps2;       // eps * eps (Alg. 2 literal)
    float rho;        // clip radius (+inf = off)
    float step;       // eta_t / (1 - beta1^(t+1))
    float sbc2;       // sqrt(1 - beta2^(t+1))
    float Mf;         // (float) M
};

struct LaunchArgs {
    const ChunkRec* chunks;  // [n_chunks]; null when strided
    const uint64_t* ptrs;
    uint32_t n_chunks;       // workgroups along x: chunks (strided) or chunk records << split_log2
    uint32_t chunk_elems;
    // Table layouts: 2^split_log2 workgroups share one chunk record, each taking
    // chunk_elems >> split_log2 of its elements (gated steps run best with one 256-element
    // tile per workgroup, ungated ones with two: one table serves both).
    uint32_t split_log2;
    int M;
    uint32_t lds_bytes;  // dynamic LDS requested per workgroup: an occupancy limiter, never accessed
    // Fast path: one segment whose replica pointers are base[a] + m * rstride[a] (bytes).
    int strided;
    uint64_t numel0;
    // Strided layouts: workgroups [0, pair_blocks) take the paired mapping over the elements
    // [pair_e0, pair_e1) (whole groups); the remaining workgroups take contiguous chunks of
    // chunk_elems, first head_chunks of them over [0, pair_e0), then the rest over
    // [pair_e1, numel0).  pair_blocks == 0 (then pair_e0 == pair_e1 == head_chunks == 0) is the
    // plain contiguous decomposition.
    uint32_t pair_blocks;
    uint32_t pair_e0;
    uint32_t head_chunks;
    uint64_t pair_e1;
    uint64_t base[N_ARRAYS];
    uint64_t rstride[N_ARRAYS];
    // Norm-based clipping: per-replica factor the gradient is multiplied by (device, [M]);
    // null = coordinate-wise clipping (factor 1).
    const float* gscale;
    StepScalars sc;
};

// Launches the step kernel for (kind, mask, M, gradient dtype) on `stream`.
// Returns hipErrorInvalidValue when the combination does not exist.
// With resident_out nothing is launched: *resident_out receives the workgroups of that kernel
// one compute unit holds under a.lds_bytes of dynamic LDS, as the runtime computes it.
hipError_t launch_step(int kind, uint32_t mask, int grad_bf16, const LaunchArgs& a,
                       hipStream_t stream, uint32_t* resident_out = nullptr);

// Update-then-average ordering (the listings the paper's proofs use) for kind in
// {KIND_ADAM, KIND_ADAM_LITERAL, KIND_SGDM}; amsgrad adds the vmax state (Adam kinds only).
hipError_t launch_step_post(int kind, uint32_t mask, int amsgrad, int grad_bf16, const LaunchArgs& a,
                            hipStream_t stream);

// u = v = 0 (v skipped when has_v == 0; vmax too when present) and, when broadcast != 0, x^m = x^0 for m >= 1,
// for every segment (d_ptrs: the device pointer table, seg_numel: host array).
hipError_t launch_init_states(const uint64_t* d_ptrs, int M, const uint64_t* seg_numel,
                              uint64_t n_segs, int has_v, int has_vmax, int broadcast,
                              hipStream_t stream);

// Norm-based clipping, first half: ||g^m||_2 over every element of replica m into
// d_norms[m], and d_gscale[m] = norm > rho ? rho / norm : 1.  One workgroup and one partial sum
// per replica and run of elements: a.n_chunks runs, either chunks of a.chunk_elems elements
// (strided layouts, runs == nullptr) or the entries of `runs` (device memory; table layouts:
// segment-aligned, never crossing a segment).  d_partials needs a.M * a.n_chunks doubles.
// Deterministic (no atomics).
struct DiagChunk;
hipError_t launch_grad_norms(const LaunchArgs& a, const DiagChunk* runs, int grad_bf16, float rho,
                             double* d_partials, float* d_norms, float* d_gscale, hipStream_t stream);

// Relative-rate-of-change diagnostic.  For each of n_ranges element ranges (segment
// row_index[k], elements [offsets[k], offsets[k] + numels[k])) accumulates, per replica,
// sum (s - ref)^2 and sum ref^2; then d_out[m] = sqrt of the first, d_out[M + m] = sqrt of the
// second.  d_s_rows points at the state's row of segment 0 in the pointer table (array already
// selected); d_r_rows is a [n_segments][M] table of reference base pointers.  P = total
// partials per replica = sum over ranges of ceil(numel / chunk); d_part holds 2 * M * P doubles.
// vec_ok: every state and reference base is 16-byte aligned (128-bit loads), else scalar loads.
hipError_t launch_state_change(const uint64_t* d_s_rows, const uint64_t* d_r_rows, uint32_t M,
                               uint32_t n_ranges, const uint64_t* row_index, const uint64_t* offsets,
                               const uint64_t* numels, uint32_t chunk, int vec_ok, double* d_part, uint32_t P,
                               float* d_out, hipStream_t stream);

// Batched, per-tensor form of the diagnostic.  One record per run of at most DIAG_CHUNK_ELEMS
// elements of one tensor (records never cross tensor boundaries); tensor k owns the records
// [first[k], first[k] + count[k]).
struct DiagChunk {
    uint64_t start;  // first element within the segment
    uint32_t seg;    // segment index
    uint32_t len;    // elements (<= DIAG_CHUNK_ELEMS)
};
enum : uint32_t { DIAG_CHUNK_ELEMS = 16384 };

// For every record and replica: partial sums of (s - ref)^2 and ref^2 into part[0 .. M*P) and
// part[M*P .. 2*M*P); then per tensor and replica the square roots of their sums into
// change[k * M + m] and base[k * M + m] (device memory).  d_ptrs: the context's pointer table,
// which: array index; d_ref: [n_segments][M] reference base pointers.  vec_ok: every state and
// reference segment base is 16-byte aligned (128-bit loads), else scalar loads.  Enqueues two
// kernels on `stream`; nothing else.
hipError_t launch_state_change_tensors(const uint64_t* d_ptrs, int which, const uint64_t* d_ref, uint32_t M,
                                       const DiagChunk* d_chunks, uint32_t P, const uint32_t* d_first,
                                       const uint32_t* d_count, uint64_t n_tensors, int vec_ok, double* d_part,
                                       float* d_change, float* d_base, hipStream_t stream);

// dst^m = s^m for every record and replica (the snapshot), one launch.  numel: elements per replica
// covered by the P records (chooses between the kernel for long and the one for short records).
hipError_t launch_snapshot_copy(const uint64_t* d_ptrs, int which, const uint64_t* d_dst, uint32_t M,
                                const DiagChunk* d_chunks, uint32_t P, uint64_t numel, int vec_ok, hipStream_t stream);

// out[i] = (((s^0[i] + s^1[i]) + ...) + s^{M-1}[i]) / M for i in [0, numel) of one tensor
// that starts `offset` elements into a segment whose replica pointers are row[0..M-1].
hipError_t launch_replica_mean(const uint64_t* row, int M, int is_bf16, uint64_t offset,
                               uint64_t numel, float* out, hipStream_t stream);

}  // namespace desloc
