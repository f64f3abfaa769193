/*
 * desloc.h -- C ABI of the MI355X (gfx950) DES-LOC optimizer-step library.
 *
 * DES-LOC (Desynced Low Communication adaptive optimizers) runs a base optimizer
 * (Adam, ADOPT or SGD with momentum) on M worker replicas and averages each piece
 * of state across the workers on its own period: parameters x every Kx steps,
 * first moment u every Ku steps, second moment v every Kv steps (paper: Alg. 1,
 * the generic method; Alg. 2, DES-LOC-Adam; Alg. 3, DES-LOC-ADOPT; the SGDM
 * appendix for the momentum form).  In this library all M replicas live in one
 * GPU's HBM, so every "average across workers" E_m[.] is an in-register,
 * ascending-m sum inside the same elementwise kernel that applies the update.
 *
 * Conventions
 *   - Every pointer named *device* points to GPU global memory owned by the
 *     caller (e.g. PyTorch allocations).  The library never frees, reallocates
 *     or keeps host copies of it.  Host pointers are only read during the call.
 *   - All state (x, u, v) is fp32.  Gradients are fp32 or bf16 (widened exactly).
 *   - Tensor k of replica m of array a is the device pointer a[m * n_tensors + k]
 *     and holds numel[k] contiguous elements.
 *   - Tensors that are adjacent in memory in every array and every replica are
 *     merged into one segment at init; each segment base must be 16-byte aligned
 *     (8-byte for bf16 gradients), else DESLOC_ERR_ALIGN.  A packed flat buffer
 *     of many small tensors therefore becomes a single segment.
 *   - Functions return DESLOC_OK (0) or a negative desloc_status.  They never
 *     throw and never abort.  On error no output argument is written.
 *   - Work is enqueued on the HIP stream given at init and is asynchronous with
 *     respect to the host unless stated otherwise.  Calls on one context are not
 *     thread-safe; different contexts are independent.
 *
 * Fast layout.  Results never depend on the layout, the speed does.  The fastest path needs
 * (a) one segment (every replica one packed buffer), (b) the same distance between
 * consecutive replicas within every array, and (c) every fp32 array of every replica
 * starting at the same offset modulo 65536 bytes (e.g. 64 KiB-aligned allocations and a
 * replica stride that is a multiple of 16384 elements).  With (a) and (b) every address is
 * formed from kernel arguments; with (c) as well, the elements between the first and the last
 * 64 KiB boundary are handed out so that the two halves of each 1 KiB vector access lie
 * exactly 32 KiB apart, which this GPU's memory system serves markedly faster when many
 * replica streams are swept at once (gated steps).  desloc_plan_info reports what applies.
 * Segments of separately allocated tensors that satisfy (c) get the same mapping.
 * Where to put the arrays: keep close together what a launch sweeps at one time.  A step
 * without a gate sweeps one replica's g, x, u, v at the same element position, a gated step
 * all M replicas' at once, and streams that are swept together run 3-8 % faster on this GPU
 * when they lie within a few GiB of each other than when each array is a block of its own
 * tens of GiB away.  Fastest measured: the tensor list cut into groups of consecutive tensors
 * of about 128 MiB per array and replica, and inside a group replica 0's x, u, v, g, then
 * replica 1's, ..., each starting on a 64 KiB boundary (one segment per group; every tensor
 * stays contiguous).  Several segments are no handicap: every workgroup of a launch without a
 * gate reads a 16-byte chunk record first, also on a one-segment layout, because so paced the
 * launch runs 2 % faster than with all addresses formed from kernel arguments.
 *
 * The library reads no environment variables.  (A build with -DDESLOC_TUNING, used only for
 * launch-shape sweeps, reads DESLOC_LDS_BYTES, DESLOC_LDS_BYTES_GATED, DESLOC_GATED_CHUNK,
 * DESLOC_NO_STRIDED, DESLOC_NO_PAIRING and DESLOC_STRIDED_UNGATED at desloc_init and
 * DESLOC_UNGATED_SPLIT at desloc_step; the values in effect show up in desloc_plan_info.)
 */
#ifndef DESLOC_H
#define DESLOC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DESLOC_VERSION 100 /* major*10000 + minor*100 + patch */

typedef enum desloc_status {
    DESLOC_OK = 0,
    DESLOC_ERR_NULL = -1,    /* a required pointer is NULL */
    DESLOC_ERR_BAD_ARG = -2, /* value out of range, struct_size mismatch, buffer too small */
    DESLOC_ERR_ALIGN = -3,   /* a segment base pointer is not sufficiently aligned */
    DESLOC_ERR_OOM = -4,     /* host or device allocation of the library's own tables failed */
    DESLOC_ERR_HIP = -5,     /* a HIP runtime call failed; see desloc_last_hip_error */
    DESLOC_ERR_VARIANT = -6, /* flag or array not valid for the chosen variant */
    DESLOC_ERR_TOO_LARGE = -7 /* input exceeds the fixed scratch of desloc_state_change_static */
} desloc_status;

/* Base optimizer. */
typedef enum desloc_variant {
    DESLOC_ADAM = 0,  /* Alg. 2: states u, v */
    DESLOC_ADOPT = 1, /* Alg. 3: states m (stored in u), v */
    DESLOC_SGDM = 2   /* Alg. 1 with one state u: u = beta u + (1-beta) g, x = x - eta u */
} desloc_variant;

typedef enum desloc_dtype { DESLOC_F32 = 0, DESLOC_BF16 = 1 } desloc_dtype;

/* Readings of the listings that the paper leaves open; default (0) is listed first. */
enum {
    /* Adam direction.  Default: bias-corrected Adam as cited by the paper,
     *   d = eta/(1-b1^(t+1)) * u / (sqrt(v)/sqrt(1-b2^(t+1)) + eps).
     * With this flag: Alg. 2 exactly as printed, d = eta * u / sqrt(v + eps^2). */
    DESLOC_FLAG_ADAM_LITERAL = 1u << 0,
    /* ADOPT normaliser max(sqrt(v_prev), eps).  Default: the worker's own previous v,
     * as printed in Alg. 3.  With this flag: E_m[v_prev] on steps where v is averaged. */
    DESLOC_FLAG_ADOPT_AVG_NORMALISER = 1u << 1,
    /* ADOPT first step.  Default: Alg. 3 as printed (v_{-1} = 0, so t = 0 divides by eps).
     * With this flag, at t = 0 only: v_0 = clip(g)^2, m and x keep their (possibly
     * averaged) incoming value, as in the base ADOPT algorithm. */
    DESLOC_FLAG_ADOPT_INIT_G0SQ = 1u << 2,
    /* Which clip.  Default: the coordinate-wise clip of the listings (Sec. 2.1).
     * With this flag: norm-based clipping, which the paper's model table says its experiments
     * used (no formula printed; taken as the usual global-norm clip): per replica m,
     *   gh = g * (||g^m||_2 > rho ? rho / ||g^m||_2 : 1),   norm over all tensors of replica m,
     * and no coordinate clip.  Each step then reads the gradients twice (norm pass, then the
     * update pass); the norm is a deterministic two-level fp64 reduction. */
    DESLOC_FLAG_NORM_CLIP = 1u << 3,
    /* Ordering of update and average.  Default: Alg. 1-3, the previous state is averaged, then
     * updated locally.  With this flag: the ordering of the listings used by the paper's proofs
     * (SGDM appendix listing; DES-LOC-Adam with probabilistic synchronization), with the
     * deterministic gates t mod K == 0 in place of their coin flips: every replica updates
     * locally first and a gated state is then replaced by the mean of the UPDATED values,
     *   u^m = E_m[b1 u^m + (1-b1) gh^m],  x^m = E_m[x^m - d^m],
     * so all replicas hold identical bits of a state right after its sync.  Adam and SGDM only. */
    DESLOC_FLAG_POST_AVERAGE = 1u << 4,
    /* AMSGrad normaliser of the probabilistic DES-LOC-Adam listing: vt = max(v_t, vt_prev) per
     * replica (never averaged itself), used in place of v_t in the direction.  Needs
     * DESLOC_FLAG_POST_AVERAGE, the Adam variant and the vmax pointer table. */
    DESLOC_FLAG_AMSGRAD = 1u << 5
};

/* What desloc_init does to the caller's buffers (Alg. 1, local-init line). */
typedef enum desloc_init_mode {
    DESLOC_INIT_AS_IS = 0,             /* use x, u, v as they are (resume / custom seeds) */
    DESLOC_INIT_ZERO_STATES = 1,       /* u = v (= vmax) = 0 on every replica; x untouched */
    DESLOC_INIT_BROADCAST_REPLICA0 = 2 /* u = v (= vmax) = 0 and x^m = x^0 for every replica m */
} desloc_init_mode;

/* Which array desloc_read_state reads. */
typedef enum desloc_array {
    DESLOC_X = 0, DESLOC_U = 1, DESLOC_V = 2, DESLOC_G = 3,
    DESLOC_VMAX = 4 /* AMSGrad state; only with DESLOC_FLAG_AMSGRAD */
} desloc_array;

/* replica argument of desloc_read_state: the ascending-m mean E_m[s^m] (the averaged
 * iterate of the paper's analysis) instead of one replica. */
#define DESLOC_REPLICA_MEAN (-1)
/* tensor argument of desloc_read_state: all tensors, concatenated without padding. */
#define DESLOC_ALL_TENSORS (-1)

/* Sync-mask bits returned by desloc_sync_mask. */
#define DESLOC_SYNC_X 1u
#define DESLOC_SYNC_U 2u
#define DESLOC_SYNC_V 4u

#define DESLOC_MAX_REPLICAS 1024

typedef struct desloc_config {
    uint32_t struct_size; /* sizeof(desloc_config), for ABI checking */
    uint32_t variant;     /* desloc_variant */
    uint32_t M;           /* worker replicas, 1 .. DESLOC_MAX_REPLICAS */
    uint32_t grad_dtype;  /* desloc_dtype of the g arrays */
    uint64_t n_tensors;   /* >= 1 */
    const uint64_t* numel; /* host, [n_tensors]; zero-sized tensors are allowed and skipped */
    uint64_t Kx, Ku, Kv;  /* sync periods in steps; 0 = never (K = infinity); Kv ignored for SGDM */
    float lr;             /* eta; change between steps with desloc_set_lr */
    float beta1;          /* in [0,1); the momentum decay for SGDM */
    float beta2;          /* in [0,1); ignored for SGDM */
    float eps;            /* > 0: Adam eps (lambda when ADAM_LITERAL), ADOPT epsilon */
    float rho;            /* > 0: coordinate-wise clip radius; INFINITY disables the clip */
    uint32_t flags;       /* DESLOC_FLAG_* */
    uint32_t init_mode;   /* desloc_init_mode */
    void* const* x;       /* host array [M * n_tensors] of device pointers to fp32 */
    void* const* u;       /* same shape */
    void* const* v;       /* same shape; must be NULL for SGDM */
    void* const* g;       /* same shape; element type grad_dtype */
    void* const* vmax;    /* same shape, fp32: AMSGrad state; NULL unless DESLOC_FLAG_AMSGRAD */
    void* stream;         /* hipStream_t to enqueue on; NULL = the default stream */
    uint32_t chunk_elems; /* elements one workgroup processes; 0 = library default;
                             otherwise a multiple of 256 in [256, 1048576] */
    uint32_t reserved;    /* must be 0 */
} desloc_config;

typedef struct desloc_ctx desloc_ctx; /* opaque */

/* Work decomposition computed at init (host logic only, no GPU needed). */
typedef struct desloc_plan_info {
    uint64_t n_segments;  /* after merging adjacent tensors */
    uint64_t n_chunks;    /* strided layouts: workgroups of a gated step; other layouts: 16-byte chunk
                             records (a launch uses one or two workgroups per record and, on steps
                             without a gate, per replica) */
    uint64_t total_numel; /* sum of numel, per replica */
    uint32_t chunk_elems; /* the value in effect */
    uint32_t strided;     /* 1: single segment with uniform replica strides (conditions (a), (b)):
                             gated steps form every address from kernel arguments */
    uint64_t paired_numel; /* elements per replica that take the 32 KiB-paired mapping
                              (condition (c)); 0 when the layout is not eligible */
    /* The step kernels run as 64-lane workgroups and cap the workgroups resident per compute
     * unit with a dynamic-LDS request that is never accessed.  Index 0: steps without a gate,
     * index 1: steps with a gate. */
    uint32_t lds_limiter_bytes[2];   /* the request per workgroup */
    uint32_t intended_workgroups[2]; /* floor(160 KiB / request): what the request aims at */
    uint32_t resident_workgroups[2]; /* what the HIP runtime reports for the kernel that step t = 1
                                        (index 0) / the first gated step after 0 (index 1) would
                                        launch; 0 = not queried (desloc_plan, no such step, or a
                                        context with DESLOC_FLAG_POST_AVERAGE) */
    uint32_t gated_chunk_elems;      /* elements per workgroup on gated steps */
    uint32_t reserved;
} desloc_plan_info;

/* Library version (DESLOC_VERSION of the build). */
uint32_t desloc_version(void);

/* Static, NUL-terminated description of a status code. */
const char* desloc_strerror(int status);

/* hipError_t value of the last failing HIP call made for this context (0 if none),
 * for DESLOC_ERR_HIP.  ctx may be NULL: then the last error of a failed desloc_init
 * on the calling thread. */
int desloc_last_hip_error(const desloc_ctx* ctx);

/* Gate of Alg. 1 without a context: bit0 = (Kx != 0 && t mod Kx == 0), bit1 likewise
 * for Ku, bit2 for Kv.  Pure integer function; every gate fires at t = 0. */
uint32_t desloc_sync_mask_k(uint64_t t, uint64_t Kx, uint64_t Ku, uint64_t Kv);

/* Validates cfg and computes the segment / chunk decomposition exactly as desloc_init
 * would, without touching the GPU (pointer values are only compared, never
 * dereferenced).  Returns the same status desloc_init would return for argument
 * errors.  out must be non-NULL. */
int desloc_plan(const desloc_config* cfg, desloc_plan_info* out);

/* Creates a context from the inputs of Alg. 1 (its Require line: the initial parameters x_0
 * and states s_{-1} are the contents of the caller's arrays, plus rho, eta, M, Kx and the
 * per-state periods): validates cfg, merges adjacent tensors into segments, uploads the
 * segment and chunk tables, applies init_mode (Alg. 1's local-init line; asynchronously, on
 * cfg->stream).  A packed layout with more than 2^26 - 1 workgroups per launch (2^34 elements
 * per replica at the default chunk size) is rejected with DESLOC_ERR_BAD_ARG; pass a larger
 * chunk_elems for such sizes.
 * The pointer tables and numel are copied; cfg may be freed after the call.
 * The tensor memory itself stays owned by the caller and must outlive the context. */
int desloc_init(const desloc_config* cfg, desloc_ctx** out);

/* Which states are averaged at step t for this context (Alg. 1 gates; Alg. 2 / Alg. 3
 * for the three states).  bit0 = x, bit1 = u, bit2 = v; bit2 is never set for SGDM.
 * Pure integer function, no device work.  NULL ctx returns 0. */
uint32_t desloc_sync_mask(const desloc_ctx* ctx, uint64_t t);

/* Sets the learning rate eta_t used by subsequent steps (Alg. 1 takes a schedule). */
int desloc_set_lr(desloc_ctx* ctx, float lr);

/* One DES-LOC step t (0-based) over every tensor and every replica, in place, using
 * the gradients currently in the g arrays:
 *   gh = clip(g, rho); for each state gated at t the previous values are replaced by
 *   their ascending-m mean over replicas; then the base optimizer's state and
 *   parameter updates are applied per replica (Alg. 1 main loop; Alg. 2 / Alg. 3).
 * One kernel launch on the context's stream (with DESLOC_FLAG_NORM_CLIP two more before it, for
 * the norms); a sync step reads and writes each array once, like any other step.  t need not be consecutive between calls: both
 * the gates and Adam's bias correction are functions of the t passed here.
 * The caller must not touch the arrays until the stream has been synchronised.
 * The call only enqueues kernels (no allocation, synchronisation or memset), so it may
 * run under HIP stream capture; a captured step keeps the t it was captured with. */
int desloc_step(desloc_ctx* ctx, uint64_t t);

/* The outputs of Alg. 1 (its Ensure line: x_T and the states s_{T-1}; the listing prints no
 * worker index, so both the per-worker values and their mean are offered).
 * Copies state to the host as fp32 (bf16 gradients are widened).  Synchronises the
 * context's stream first.  which: desloc_array.  replica: 0..M-1, or
 * DESLOC_REPLICA_MEAN for E_m[.] computed on the device in ascending-m order.
 * tensor: 0..n_tensors-1, or DESLOC_ALL_TENSORS for all tensors concatenated in index
 * order without padding.  dst_bytes must be at least 4 * (number of elements
 * returned), else DESLOC_ERR_BAD_ARG.  Reading DESLOC_V of an SGDM context is
 * DESLOC_ERR_VARIANT. */
int desloc_read_state(desloc_ctx* ctx, int which, int replica, int64_t tensor, void* host_dst,
                      size_t dst_bytes);

/* Norm-based clipping only (DESLOC_FLAG_NORM_CLIP, else DESLOC_ERR_VARIANT): the gradient
 * norms ||g^m||_2, m = 0..M-1, computed by the most recent desloc_step, as fp32 into
 * host_dst (count >= M floats, else DESLOC_ERR_BAD_ARG).  Synchronises the stream. */
int desloc_read_grad_norms(desloc_ctx* ctx, float* host_dst, size_t count);

/* Relative rate of change of a state, the paper's diagnostic ||s_{t+K} - s_t||_2 / ||s_t||_2
 * (Sec. 4, "Metrics").  ref is a host array [M * n_tensors] of device pointers to fp32
 * reference copies of array `which` (DESLOC_X, _U, _V or _VMAX), e.g. a snapshot taken K steps
 * earlier with desloc_snapshot_state; wherever two tensors of the state are adjacent in memory
 * their reference copies must be adjacent too (else DESLOC_ERR_BAD_ARG).  For every replica m:
 *     change_out[m] = || s^m - ref^m ||_2 ,   base_out[m] = || ref^m ||_2
 * over tensor `tensor` or, with DESLOC_ALL_TENSORS, over all tensors; the ratio is the
 * paper's measure.  fp64 accumulation in a fixed order (same bits on every run), rounded to
 * fp32.  count >= M floats each.  Synchronises the stream.  Scratch is kept in the context and
 * grown when a call needs more than any earlier one (the only case in which it allocates). */
int desloc_state_change(desloc_ctx* ctx, int which, int64_t tensor, void* const* ref,
                        float* change_out, float* base_out, size_t count);

/* For callers that must not allocate (code under HIP graph capture nearby, tight serving
 * loops, harnesses that forbid hipMalloc): desloc_state_change with the same arguments,
 * results and errors, except that it allocates nothing, neither on the device nor on the host.
 * Its partial sums, its copy of the reference base table and its results live in one fixed
 * array of DESLOC_STATIC_SCRATCH_BYTES that the library holds on every GPU it runs on until the
 * process ends.  Partial sums cover 16384 elements each, or the next power-of-two multiple for
 * which they fit (so the last bits of the fp64 sums, not of the fp32 results in practice, can
 * differ from desloc_state_change); an input whose tables and partial sums still do not fit
 * (2 * M * ceil(numel / 4194304) doubles per tensor range, plus 8 * n_segments * M bytes) is
 * refused with DESLOC_ERR_TOO_LARGE and nothing is computed.  All calls on one GPU, from any
 * context, share that array: calls that overlap in time race, so serialise them. */
#define DESLOC_STATIC_SCRATCH_BYTES (4u << 20)
int desloc_state_change_static(desloc_ctx* ctx, int which, int64_t tensor, void* const* ref,
                               float* change_out, float* base_out, size_t count);

/* Copies array `which` of every replica and tensor into dst (same shape and rules as ref
 * above), with one kernel launch on the context's stream: the snapshot s_t of the diagnostic.
 * dst also becomes the bound reference of desloc_state_change_tensors (see desloc_bind_reference:
 * the first call, and any call with a different dst, allocates and synchronises). */
int desloc_snapshot_state(desloc_ctx* ctx, int which, void* const* dst);

/* Binds the reference copy that desloc_state_change_tensors compares against: ref as for
 * desloc_state_change.  Validates the layout, uploads the table of its segment bases and, on
 * the first call for a context, builds the per-tensor work tables: it allocates and
 * synchronises the stream, so call it outside loops.  Binding the table already bound is free. */
int desloc_bind_reference(desloc_ctx* ctx, void* const* ref);

/* The paper's diagnostic per tensor and per state, as the rate-of-change figure of its Sec. 4
 * ("Metrics") draws it, for all tensors in one pass: for every tensor k and replica m
 *     change_dev[k * M + m] = || s^m_k - ref^m_k ||_2 ,   base_dev[k * M + m] = || ref^m_k ||_2
 * with s = array `which` (DESLOC_X, _U, _V or _VMAX) and ref the bound reference (the last
 * desloc_snapshot_state destination or desloc_bind_reference table; none bound:
 * DESLOC_ERR_BAD_ARG).  change_dev and base_dev are DEVICE buffers of n_tensors * M floats each,
 * owned by the caller.  The call enqueues two kernels on the context's stream and returns: no
 * synchronisation, no allocation, no host copy, so it can sit inside a training loop or a
 * captured graph; read the buffers after synchronising.  fp64 accumulation in a fixed order
 * (16384-element partial sums per tensor, then one sum per tensor and replica), rounded to fp32;
 * a tensor of size 0 gives 0 and 0.  Reads each of the two arrays once. */
int desloc_state_change_tensors(desloc_ctx* ctx, int which, float* change_dev, float* base_dev);

/* The decomposition in effect for a context. */
int desloc_get_plan(const desloc_ctx* ctx, desloc_plan_info* out);

/* Waits for all work enqueued by this context. */
int desloc_synchronize(desloc_ctx* ctx);

/* Frees the library's own tables.  The tensor memory is not touched.  NULL is a no-op. */
int desloc_destroy(desloc_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* DESLOC_H */
