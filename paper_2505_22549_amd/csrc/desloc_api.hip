// C ABI of the DES-LOC step library (declared in include/desloc.h): argument
// validation, segment / chunk planning, per-step scalars and kernel selection.
// Every step of the method itself runs in the gfx950 kernels; the host only decides
// which instantiation to launch (the sync mask of Alg. 1 is uniform over a step).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/desloc.h"
#include "desloc_internal.h"

using namespace desloc;

// Scratch of desloc_state_change_static, the entry point for callers that must not allocate:
// one array per GPU, held until the process ends.  In host code the name below is only a
// stand-in; the device address is looked up once per device (desloc_init, with that device
// current) and only that address is ever handed to kernels and copies.
static __device__ __align__(256) unsigned char scratch[DESLOC_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[MAX_DEVICES] = {};  // device address of `scratch` on each GPU

// The device address of this GPU's scratch array (device = the current device).
hipError_t static_scratch_for(int device, unsigned char** out) {
    *out = nullptr;
    if (device < 0 || device >= MAX_DEVICES) return hipSuccess;  // the static entry point reports it
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device] == nullptr) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[device] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

// Measured on MI355X over the five benchmark workloads: single-wave workgroups of 256
// elements (one 4-vector per lane and replica) and a cap on the workgroups resident per CU.
// The dynamic-LDS requests below are never touched by the kernels: they only cap how many
// workgroups the 160 KiB of a CU admit.  More resident waves widen the address window the chip
// sweeps at any instant and lower HBM efficiency; fewer leave the memory pipeline short of
// requests.  Strided path (addresses from kernel arguments): about 10 on steps without a gate
// (9-11 are equivalent; SGDM with its three read streams prefers 13-14) and 9 on gated steps
// (8-10 within 2 % for M = 4 and M = 8; 5 or fewer fall off a cliff).  With the default chunking
// only gated launches take this path; the table path has limiters of its own, below.
constexpr uint32_t DEFAULT_CHUNK_ELEMS = 256;                // strided layouts
constexpr uint32_t DEFAULT_TABLE_CHUNK_ELEMS = 512;          // table layouts: two tiles per chunk record
constexpr uint32_t DEFAULT_GATED_CHUNK_ELEMS = 256;          // strided layouts only (no chunk table)
constexpr uint32_t DEFAULT_LDS_LIMITER_BYTES = 15500;        // Adam / ADOPT without a gate
constexpr uint32_t DEFAULT_SGDM_LDS_LIMITER_BYTES = 11500;   // SGDM without a gate
constexpr uint32_t DEFAULT_GATED_LDS_LIMITER_BYTES = 17500;  // any gated step
// Table layouts, steps without a gate: 13 per CU, one wave slot (one 4-vector per lane) per
// workgroup for Adam / ADOPT, one two-slot record per workgroup for SGDM.  A workgroup of the
// table path reads its chunk record and its pointer row before its first vector load, and
// with that start-up the optimum sits at 13-14 resident workgroups, where the launch runs
// 2 % faster than the strided path does at its own optimum of 10-11 (measured on the same
// arrays, configs 2, 3 and 5; 9 or 16 resident are 5-15 % slower, so this one is a sharp peak).
constexpr uint32_t DEFAULT_TABLE_LDS_LIMITER_BYTES = 12500;
// The same with the AMSGrad state (five read and four write streams per replica): 10 per CU
// (1.7B workload over a whole run: 6.86 TB/s at 10, 6.83 at 11 with a wider spread, 6.74 at 12, 6.60 at 13).
constexpr uint32_t DEFAULT_TABLE_AMSGRAD_LDS_LIMITER_BYTES = 16000;
// Table layouts, gated steps: 8 per CU for Adam / ADOPT (M = 4 and M = 8; 8 and 9 are equivalent, 7 is
// 1 % faster when only x is gated and 1 % slower when more is; 6 or fewer fall off a cliff),
// 11 for SGDM (10-14 are equivalent).
constexpr uint32_t DEFAULT_TABLE_GATED_LDS_LIMITER_BYTES = 20000;
constexpr uint32_t DEFAULT_TABLE_SGDM_GATED_LDS_LIMITER_BYTES = 14800;
constexpr uint64_t CLOSE_SPAN_BYTES = 8ull << 30;
// Any other replica count runs the runtime loop, one replica's loads in flight at a time in its
// second pass, and wants more waves: 10 per CU (M = 3, 5, 6, 12, 16, 32: 8-10 equivalent, 7 is
// 7-10 % slower), 12 for M = 2 (7: -25 %).
constexpr uint32_t DEFAULT_TABLE_RUNTIME_M_GATED_LDS_LIMITER_BYTES = 16000;
constexpr uint32_t DEFAULT_TABLE_RUNTIME_M2_GATED_LDS_LIMITER_BYTES = 13000;
// Strided layouts: elements per norm workgroup.  65536 keeps the second level short (config 5:
// 26 k partial sums per replica, 0.02 ms) at the same read rate as smaller chunks.
constexpr uint32_t NORM_CHUNK_ELEMS = 65536;
constexpr uint32_t MAX_CHUNK_ELEMS = 1u << 20;

struct Segment {
    uint64_t numel;
    uint64_t chunk0;
    uint64_t first_tensor;
    // table layouts: the segment's fp32 streams are congruent modulo PAIR_GROUP_BYTES, so the
    // elements [pair_e0, pair_e0 + pair_groups * PAIR_GROUP_ELEMS) get paired chunk records
    bool pair_ok = false;
    uint32_t pair_e0 = 0;
    uint64_t pair_groups = 0;
};

// Chunk records a segment of a table layout gets: head, paired groups, tail.
struct SegmentRecords {
    uint64_t head = 0, paired = 0, tail = 0;
    uint64_t total() const { return head + paired + tail; }
};

SegmentRecords segment_records(const Segment& s, uint32_t chunk) {
    SegmentRecords r;
    const uint64_t e1 = s.pair_e0 + s.pair_groups * PAIR_GROUP_ELEMS;
    if (s.pair_groups != 0) {
        r.head = (s.pair_e0 + chunk - 1) / chunk;
        r.paired = s.pair_groups * (PAIR_GROUP_ELEMS / (2 * TILE_ELEMS));
        r.tail = (s.numel - e1 + chunk - 1) / chunk;
    } else {
        r.tail = (s.numel + chunk - 1) / chunk;
    }
    return r;
}

struct Plan {
    std::vector<Segment> segs;
    std::vector<uint64_t> tensor_seg;   // segment of tensor k (unused for numel == 0)
    std::vector<uint64_t> tensor_off;   // element offset of tensor k in its segment
    uint64_t n_chunks = 0;
    uint64_t total_numel = 0;
    uint32_t chunk_elems = DEFAULT_CHUNK_ELEMS;
    // Single segment whose replica pointers are base[a] + m * rstride[a] in every array:
    // addresses can then be formed from kernel arguments alone (no tables on the device).
    bool strided = false;
    uint64_t base[N_ARRAYS] = {0, 0, 0, 0, 0};
    uint64_t rstride[N_ARRAYS] = {0, 0, 0, 0, 0};
    // Strided layouts whose fp32 streams are all congruent modulo PAIR_GROUP_BYTES can take the
    // paired mapping; pair_e0 is the first element on a PAIR_GROUP_BYTES boundary.
    bool pair_ok = false;
    uint32_t pair_e0 = 0;
    uint64_t max_span_bytes = 0;  // widest segment, over all its arrays and replicas (see make_plan)
    // Chunk records of the table decomposition (Segment::chunk0 indexes into them).  Strided layouts
    // with the default chunking have them too: their launches without a gate take the table path,
    // which is the faster one (see DEFAULT_TABLE_LDS_LIMITER_BYTES), their gated launches stay strided.
    uint64_t table_chunks = 0;
    uint32_t table_chunk_elems = 0;
    bool ungated_table = false;
};

// Workgroups and their decomposition for a launch over a strided segment with `chunk` elements
// per contiguous workgroup: whole aligned groups take the paired mapping when the layout allows
// it and a workgroup is exactly one tile, everything else is cut into contiguous chunks.
struct StridedGrid {
    uint64_t n_blocks = 0;
    uint32_t pair_blocks = 0, pair_e0 = 0, head_chunks = 0;
    uint64_t pair_e1 = 0;
};

StridedGrid strided_grid(const Plan& p, uint32_t chunk) {
    StridedGrid g;
    const uint64_t n = p.segs.empty() ? 0 : p.segs[0].numel;
    if (p.pair_ok && chunk == TILE_ELEMS && n >= static_cast<uint64_t>(p.pair_e0) + PAIR_GROUP_ELEMS) {
        const uint64_t groups = (n - p.pair_e0) / PAIR_GROUP_ELEMS;
        if (groups * PAIR_WAVES <= 0xffffffffull) {
            g.pair_e0 = p.pair_e0;
            g.pair_e1 = p.pair_e0 + groups * PAIR_GROUP_ELEMS;
            g.pair_blocks = static_cast<uint32_t>(groups * PAIR_WAVES);
            g.head_chunks = (p.pair_e0 + chunk - 1) / chunk;
        }
    }
    g.n_blocks = static_cast<uint64_t>(g.pair_blocks) + g.head_chunks + (n - g.pair_e1 + chunk - 1) / chunk;
    return g;
}

// A launch dimension holds fewer than 2^32 work-items: with 64-lane workgroups, 2^26 - 1 of them.
constexpr uint64_t MAX_BLOCKS_X = (1ull << 26) - 1;

thread_local int g_init_hip_error = 0;

inline size_t grad_elem_size(uint32_t dt) { return dt == DESLOC_BF16 ? 2u : 4u; }

int validate(const desloc_config* c) {
    if (c == nullptr) return DESLOC_ERR_NULL;
    if (c->struct_size != sizeof(desloc_config)) return DESLOC_ERR_BAD_ARG;
    if (c->variant > DESLOC_SGDM) return DESLOC_ERR_BAD_ARG;
    if (c->M < 1 || c->M > DESLOC_MAX_REPLICAS) return DESLOC_ERR_BAD_ARG;
    if (c->grad_dtype > DESLOC_BF16) return DESLOC_ERR_BAD_ARG;
    if (c->n_tensors < 1) return DESLOC_ERR_BAD_ARG;
    if (c->numel == nullptr || c->x == nullptr || c->u == nullptr || c->g == nullptr)
        return DESLOC_ERR_NULL;
    if (c->variant == DESLOC_SGDM) {
        if (c->v != nullptr) return DESLOC_ERR_VARIANT;
    } else if (c->v == nullptr) {
        return DESLOC_ERR_NULL;
    }
    const uint32_t known = DESLOC_FLAG_ADAM_LITERAL | DESLOC_FLAG_ADOPT_AVG_NORMALISER |
                           DESLOC_FLAG_ADOPT_INIT_G0SQ | DESLOC_FLAG_NORM_CLIP |
                           DESLOC_FLAG_POST_AVERAGE | DESLOC_FLAG_AMSGRAD;
    if (c->flags & ~known) return DESLOC_ERR_BAD_ARG;
    if ((c->flags & DESLOC_FLAG_ADAM_LITERAL) && c->variant != DESLOC_ADAM) return DESLOC_ERR_VARIANT;
    if ((c->flags & (DESLOC_FLAG_ADOPT_AVG_NORMALISER | DESLOC_FLAG_ADOPT_INIT_G0SQ)) &&
        c->variant != DESLOC_ADOPT)
        return DESLOC_ERR_VARIANT;
    if ((c->flags & DESLOC_FLAG_POST_AVERAGE) && c->variant == DESLOC_ADOPT) return DESLOC_ERR_VARIANT;
    if (c->flags & DESLOC_FLAG_AMSGRAD) {
        if (!(c->flags & DESLOC_FLAG_POST_AVERAGE) || c->variant != DESLOC_ADAM) return DESLOC_ERR_VARIANT;
        if (c->vmax == nullptr) return DESLOC_ERR_NULL;
    } else if (c->vmax != nullptr) {
        return DESLOC_ERR_VARIANT;
    }
    if (c->init_mode > DESLOC_INIT_BROADCAST_REPLICA0) return DESLOC_ERR_BAD_ARG;
    if (!std::isfinite(c->lr)) return DESLOC_ERR_BAD_ARG;
    if (!(c->beta1 >= 0.0f && c->beta1 < 1.0f)) return DESLOC_ERR_BAD_ARG;
    if (c->variant != DESLOC_SGDM && !(c->beta2 >= 0.0f && c->beta2 < 1.0f)) return DESLOC_ERR_BAD_ARG;
    if (!(c->eps > 0.0f) || !std::isfinite(c->eps)) return DESLOC_ERR_BAD_ARG;
    if (!(c->rho > 0.0f)) return DESLOC_ERR_BAD_ARG;  // +inf allowed, NaN rejected
    if (c->reserved != 0) return DESLOC_ERR_BAD_ARG;
    if (c->chunk_elems != 0 &&
        (c->chunk_elems % TILE_ELEMS != 0 || c->chunk_elems > MAX_CHUNK_ELEMS))
        return DESLOC_ERR_BAD_ARG;
    return DESLOC_OK;
}

// Merges tensors that are adjacent in every array of every replica into segments and
// cuts the segments into chunks.  Pointer values are compared, never dereferenced.
int make_plan(const desloc_config* c, Plan& p) {
    const uint64_t nt = c->n_tensors;
    const uint32_t M = c->M;
    const bool has_v = c->variant != DESLOC_SGDM;
    const bool has_vmax = c->vmax != nullptr;
    const size_t gsz = grad_elem_size(c->grad_dtype);
    p.tensor_seg.assign(nt, 0);
    p.tensor_off.assign(nt, 0);

    auto ptr = [&](void* const* tab, uint32_t m, uint64_t k) {
        return reinterpret_cast<uintptr_t>(tab[static_cast<uint64_t>(m) * nt + k]);
    };

    bool have_prev = false;
    uint64_t prev = 0;
    for (uint64_t k = 0; k < nt; ++k) {
        const uint64_t n = c->numel[k];
        if (n == 0) continue;
        for (uint32_t m = 0; m < M; ++m) {
            if (!ptr(c->x, m, k) || !ptr(c->u, m, k) || !ptr(c->g, m, k) ||
                (has_v && !ptr(c->v, m, k)) || (has_vmax && !ptr(c->vmax, m, k)))
                return DESLOC_ERR_NULL;
        }
        bool adjacent = have_prev;
        if (adjacent) {
            const uint64_t pn = c->numel[prev];
            for (uint32_t m = 0; m < M && adjacent; ++m) {
                adjacent = ptr(c->x, m, k) == ptr(c->x, m, prev) + pn * 4u &&
                           ptr(c->u, m, k) == ptr(c->u, m, prev) + pn * 4u &&
                           ptr(c->g, m, k) == ptr(c->g, m, prev) + pn * gsz &&
                           (!has_v || ptr(c->v, m, k) == ptr(c->v, m, prev) + pn * 4u) &&
                           (!has_vmax || ptr(c->vmax, m, k) == ptr(c->vmax, m, prev) + pn * 4u);
            }
        }
        if (!adjacent) {
            for (uint32_t m = 0; m < M; ++m) {
                if (ptr(c->x, m, k) % 16u || ptr(c->u, m, k) % 16u ||
                    (has_v && ptr(c->v, m, k) % 16u) || (has_vmax && ptr(c->vmax, m, k) % 16u) ||
                    ptr(c->g, m, k) % (4u * gsz))
                    return DESLOC_ERR_ALIGN;
            }
            Segment seg;
            seg.numel = 0;
            seg.chunk0 = 0;
            seg.first_tensor = k;
            // every fp32 stream of the segment congruent modulo PAIR_GROUP_BYTES (bf16 gradients exempt)
            const uint64_t phase = ptr(c->x, 0, k) % PAIR_GROUP_BYTES;
            bool ok = true;
            for (uint32_t m = 0; m < M && ok; ++m) {
                ok = ptr(c->x, m, k) % PAIR_GROUP_BYTES == phase && ptr(c->u, m, k) % PAIR_GROUP_BYTES == phase &&
                     (!has_v || ptr(c->v, m, k) % PAIR_GROUP_BYTES == phase) &&
                     (!has_vmax || ptr(c->vmax, m, k) % PAIR_GROUP_BYTES == phase) &&
                     (gsz != 4u || ptr(c->g, m, k) % PAIR_GROUP_BYTES == phase);
            }
            seg.pair_ok = ok;
            seg.pair_e0 = static_cast<uint32_t>(((PAIR_GROUP_BYTES - phase) % PAIR_GROUP_BYTES) / 4u);
            p.segs.push_back(seg);
        }
        Segment& s = p.segs.back();
        p.tensor_seg[k] = p.segs.size() - 1;
        p.tensor_off[k] = s.numel;
        s.numel += n;
        p.total_numel += n;
        prev = k;
        have_prev = true;
    }
    // How far apart the streams lie that a gated launch sweeps at one time: per segment, from the
    // lowest base of any array and replica to the highest end.
    for (const Segment& sg : p.segs) {
        void* const* all[N_ARRAYS] = {c->x, c->u, has_v ? c->v : nullptr, c->g, c->vmax};
        uint64_t lo = ~0ull, hi = 0;
        for (int a = 0; a < N_ARRAYS; ++a) {
            if (all[a] == nullptr) continue;
            const uint64_t es = a == ARR_G ? gsz : 4u;
            for (uint32_t m = 0; m < M; ++m) {
                const uint64_t b = ptr(all[a], m, sg.first_tensor);
                lo = b < lo ? b : lo;
                hi = b + sg.numel * es > hi ? b + sg.numel * es : hi;
            }
        }
        if (hi > lo && hi - lo > p.max_span_bytes) p.max_span_bytes = hi - lo;
    }
    if (p.segs.size() == 1) {
        const uint64_t k = p.segs[0].first_tensor;
        void* const* tabs[N_ARRAYS] = {c->x, c->u, has_v ? c->v : nullptr, c->g, c->vmax};
        bool uniform = true;
        for (int a = 0; a < N_ARRAYS && uniform; ++a) {
            if (tabs[a] == nullptr) continue;
            const uint64_t p0 = ptr(tabs[a], 0, k);
            const uint64_t st = M > 1 ? ptr(tabs[a], 1, k) - p0 : 0;
            for (uint32_t m = 0; m < M; ++m) uniform = uniform && ptr(tabs[a], m, k) == p0 + m * st;
            p.base[a] = p0;
            p.rstride[a] = st;
        }
        p.strided = uniform;
#ifdef DESLOC_TUNING
        if (const char* env = std::getenv("DESLOC_NO_STRIDED")) if (std::atoi(env)) p.strided = false;
#endif
        if (p.strided) {
            // every fp32 stream (array, replica) congruent modulo PAIR_GROUP_BYTES; bf16 gradients
            // are exempt (their halves are 16 KiB apart whatever their base)
            const uint64_t phase = p.base[ARR_X] % PAIR_GROUP_BYTES;
            bool ok = true;
            for (int a = 0; a < N_ARRAYS && ok; ++a) {
                if (tabs[a] == nullptr) continue;
                if (a == ARR_G && c->grad_dtype == DESLOC_BF16) continue;
                ok = p.base[a] % PAIR_GROUP_BYTES == phase && (M == 1 || p.rstride[a] % PAIR_GROUP_BYTES == 0);
            }
#ifdef DESLOC_TUNING
            if (const char* env = std::getenv("DESLOC_NO_PAIRING")) if (std::atoi(env)) ok = false;
#endif
            p.pair_ok = ok;
            p.pair_e0 = static_cast<uint32_t>(((PAIR_GROUP_BYTES - phase) % PAIR_GROUP_BYTES) / 4u);
        }
    }
    p.chunk_elems = c->chunk_elems ? c->chunk_elems
                                   : (p.strided ? DEFAULT_CHUNK_ELEMS : DEFAULT_TABLE_CHUNK_ELEMS);
    const bool default_chunks = c->chunk_elems == 0;
    bool table_pairing = default_chunks;  // records of two tiles, as the paired ones
#ifdef DESLOC_TUNING
    if (const char* env = std::getenv("DESLOC_NO_PAIRING")) if (std::atoi(env)) table_pairing = false;
#endif
    p.table_chunk_elems = default_chunks ? DEFAULT_TABLE_CHUNK_ELEMS : p.chunk_elems;
    uint64_t tchunks = 0;
    for (Segment& s : p.segs) {
        s.chunk0 = tchunks;
        s.pair_groups = 0;
        if (table_pairing && s.pair_ok && s.numel >= static_cast<uint64_t>(s.pair_e0) + PAIR_GROUP_ELEMS)
            s.pair_groups = (s.numel - s.pair_e0) / PAIR_GROUP_ELEMS;
        tchunks += segment_records(s, p.table_chunk_elems).total();
    }
    p.table_chunks = tchunks;
    p.ungated_table = p.strided && default_chunks;
#ifdef DESLOC_TUNING
    if (const char* env = std::getenv("DESLOC_STRIDED_UNGATED")) if (std::atoi(env)) p.ungated_table = false;
#endif
    const uint64_t chunks = p.strided ? strided_grid(p, p.chunk_elems).n_blocks : tchunks;
    // table-path launches use up to two workgroups per chunk record
    const bool table_used = !p.strided || p.ungated_table;
    if (chunks > MAX_BLOCKS_X || (table_used && 2 * tchunks > MAX_BLOCKS_X) || p.segs.size() > 0xffffffffull)
        return DESLOC_ERR_BAD_ARG;
    p.n_chunks = chunks;
    return DESLOC_OK;
}

constexpr uint32_t LDS_PER_CU_BYTES = 160u * 1024u;

uint32_t ungated_limiter(uint32_t variant, bool strided, uint32_t flags) {
    if (!strided) return (flags & DESLOC_FLAG_AMSGRAD) ? DEFAULT_TABLE_AMSGRAD_LDS_LIMITER_BYTES : DEFAULT_TABLE_LDS_LIMITER_BYTES;
    return variant == DESLOC_SGDM ? DEFAULT_SGDM_LDS_LIMITER_BYTES : DEFAULT_LDS_LIMITER_BYTES;
}

uint32_t gated_limiter(uint32_t variant, const Plan& p, uint32_t M) {
    if (p.strided) return DEFAULT_GATED_LDS_LIMITER_BYTES;
    const bool fixed_m = M == 4 || M == 8;  // compile-time replica counts: four replicas' loads in flight per wave
    if (variant == DESLOC_SGDM) return fixed_m ? DEFAULT_TABLE_SGDM_GATED_LDS_LIMITER_BYTES : DEFAULT_TABLE_RUNTIME_M2_GATED_LDS_LIMITER_BYTES;
    // 8 per CU when everything a launch sweeps at one time lies close together (grouped layouts:
    // a few GiB); replicas allocated tens of GiB apart run better with 9
    if (fixed_m) return p.max_span_bytes <= CLOSE_SPAN_BYTES ? DEFAULT_TABLE_GATED_LDS_LIMITER_BYTES : DEFAULT_GATED_LDS_LIMITER_BYTES;
    return M == 2 ? DEFAULT_TABLE_RUNTIME_M2_GATED_LDS_LIMITER_BYTES : DEFAULT_TABLE_RUNTIME_M_GATED_LDS_LIMITER_BYTES;
}

void fill_info(const Plan& p, uint32_t variant, uint32_t flags, uint32_t M, bool user_chunk, desloc_plan_info* out) {
    std::memset(out, 0, sizeof *out);
    out->n_segments = p.segs.size();
    out->n_chunks = p.n_chunks;
    out->total_numel = p.total_numel;
    out->chunk_elems = p.chunk_elems;
    out->strided = p.strided ? 1u : 0u;
    if (p.strided) {
        const StridedGrid g = strided_grid(p, p.chunk_elems);
        out->paired_numel = g.pair_e1 - g.pair_e0;
    } else {
        for (const Segment& sg : p.segs) out->paired_numel += sg.pair_groups * PAIR_GROUP_ELEMS;
    }
    out->lds_limiter_bytes[0] = ungated_limiter(variant, p.strided && !p.ungated_table, flags);
    out->lds_limiter_bytes[1] = gated_limiter(variant, p, M);
    for (int k = 0; k < 2; ++k)
        out->intended_workgroups[k] = out->lds_limiter_bytes[k] ? LDS_PER_CU_BYTES / out->lds_limiter_bytes[k] : 0u;
    out->gated_chunk_elems = !p.strided ? TILE_ELEMS : (user_chunk ? p.chunk_elems : DEFAULT_GATED_CHUNK_ELEMS);
}

}  // namespace

struct desloc_ctx {
    uint32_t variant = 0, M = 0, grad_dtype = 0, flags = 0;
    uint64_t n_tensors = 0;
    uint64_t Kx = 0, Ku = 0, Kv = 0;
    float lr = 0, beta1 = 0, beta2 = 0, eps = 0, rho = 0;
    std::vector<uint64_t> numel;
    std::vector<void*> tab[N_ARRAYS];  // host copies of the x, u, v, g, vmax pointer tables
    Plan plan;
    ChunkRec* d_chunks = nullptr;  // only for layouts that are not a single strided segment
    uint64_t* d_ptrs = nullptr;
    // norm-based clipping (DESLOC_FLAG_NORM_CLIP): partial sums, norms and factors
    double* d_partials = nullptr;
    float* d_norms = nullptr;   // [2 * M]: norms, then factors
    uint32_t norm_chunk_elems = 0;
    // rate-of-change diagnostic: scratch kept between calls, grown on demand
    void* d_diag[3] = {nullptr, nullptr, nullptr};  // reference bases, partial sums, results
    size_t diag_cap[3] = {0, 0, 0};
    // batched per-tensor diagnostic: the bound reference and the tensor-aligned records
    uint64_t* d_refbase = nullptr;       // [n_segments][M] reference base pointers
    std::vector<uint64_t> bound_bases;   // host copy of what d_refbase holds
    bool ref_bound = false;
    int ref_vec_ok = 0;                  // every reference segment base is 16-byte aligned
    DiagChunk* d_diag_chunks = nullptr;  // [diag_P]
    uint32_t* d_diag_first = nullptr;    // [n_tensors]
    uint32_t* d_diag_count = nullptr;    // [n_tensors]
    double* d_diag_part = nullptr;       // [2][M][diag_P]
    uint32_t diag_P = 0;
    bool diag_tables = false;
    // host staging of the diagnostic, sized once at init so that the calls never allocate
    std::vector<uint64_t> h_bases, h_row_index, h_offsets, h_numels;
    std::vector<float> h_out;
    unsigned char* static_scratch = nullptr;  // this GPU's `scratch` array (device address)
    float* d_mean = nullptr;                  // temporary of desloc_read_state(DESLOC_REPLICA_MEAN)
    size_t mean_cap = 0;
    uint32_t norm_chunks = 0;   // partials per replica
    DiagChunk* d_norm_runs = nullptr;  // table layouts: the runs the norm pass sums, one partial each
    hipStream_t stream = nullptr;
    int device = 0;
    uint32_t lds_bytes = DEFAULT_LDS_LIMITER_BYTES;              // steps without a gate
    uint32_t lds_bytes_gated = DEFAULT_GATED_LDS_LIMITER_BYTES;  // steps with a gate
    uint32_t gated_chunk_elems = DEFAULT_GATED_CHUNK_ELEMS;
    bool user_chunk = false;
    int strided = 0;  // single segment with uniformly strided replicas
    uint64_t base[N_ARRAYS] = {0, 0, 0, 0, 0};
    uint64_t rstride[N_ARRAYS] = {0, 0, 0, 0, 0};
    int last_hip_error = 0;
};

namespace {

int hip_fail(desloc_ctx* ctx, hipError_t e) {
    if (ctx) ctx->last_hip_error = static_cast<int>(e);
    g_init_hip_error = static_cast<int>(e);
    return DESLOC_ERR_HIP;
}

void free_tables(desloc_ctx* ctx) {
    if (ctx->d_chunks) (void)hipFree(ctx->d_chunks);
    if (ctx->d_ptrs) (void)hipFree(ctx->d_ptrs);
    if (ctx->d_partials) (void)hipFree(ctx->d_partials);
    if (ctx->d_norm_runs) (void)hipFree(ctx->d_norm_runs);
    if (ctx->d_norms) (void)hipFree(ctx->d_norms);
    for (int k = 0; k < 3; ++k) {
        if (ctx->d_diag[k]) (void)hipFree(ctx->d_diag[k]);
        ctx->d_diag[k] = nullptr;
        ctx->diag_cap[k] = 0;
    }
    void* more[] = {ctx->d_refbase, ctx->d_diag_chunks, ctx->d_diag_first, ctx->d_diag_count, ctx->d_diag_part,
                    ctx->d_mean};
    ctx->d_mean = nullptr;
    ctx->mean_cap = 0;
    for (void* q : more)
        if (q) (void)hipFree(q);
    ctx->d_refbase = nullptr;
    ctx->d_diag_chunks = nullptr;
    ctx->d_diag_first = ctx->d_diag_count = nullptr;
    ctx->d_diag_part = nullptr;
    ctx->ref_bound = ctx->diag_tables = false;
    ctx->d_chunks = nullptr;
    ctx->d_ptrs = nullptr;
    ctx->d_partials = nullptr;
    ctx->d_norm_runs = nullptr;
    ctx->d_norms = nullptr;
}

void set_strided_grid(const Plan& p, LaunchArgs& a, uint32_t chunk) {
    const StridedGrid g = strided_grid(p, chunk);
    a.chunk_elems = chunk;
    a.n_chunks = static_cast<uint32_t>(g.n_blocks);
    a.pair_blocks = g.pair_blocks;
    a.pair_e0 = g.pair_e0;
    a.pair_e1 = g.pair_e1;
    a.head_chunks = g.head_chunks;
}

LaunchArgs base_args(const desloc_ctx* ctx) {
    LaunchArgs a;
    std::memset(&a, 0, sizeof a);
    a.chunks = ctx->d_chunks;
    a.ptrs = ctx->d_ptrs;
    a.n_chunks = static_cast<uint32_t>(ctx->plan.n_chunks);
    a.chunk_elems = ctx->plan.chunk_elems;
    a.M = static_cast<int>(ctx->M);
    a.lds_bytes = ctx->lds_bytes;
    a.strided = ctx->strided;
    a.numel0 = ctx->plan.segs.empty() ? 0 : ctx->plan.segs[0].numel;
    for (int k = 0; k < N_ARRAYS; ++k) {
        a.base[k] = ctx->base[k];
        a.rstride[k] = ctx->rstride[k];
    }
    if (ctx->strided) set_strided_grid(ctx->plan, a, ctx->plan.chunk_elems);
    return a;
}

}  // namespace

extern "C" {

uint32_t desloc_version(void) { return DESLOC_VERSION; }

const char* desloc_strerror(int status) {
    switch (status) {
        case DESLOC_OK: return "ok";
        case DESLOC_ERR_NULL: return "a required pointer is NULL";
        case DESLOC_ERR_BAD_ARG: return "argument out of range, struct size mismatch or buffer too small";
        case DESLOC_ERR_ALIGN: return "a segment base pointer is not 16-byte aligned (8-byte for bf16 gradients)";
        case DESLOC_ERR_OOM: return "allocation of the library's tables failed";
        case DESLOC_ERR_HIP: return "a HIP runtime call failed (see desloc_last_hip_error)";
        case DESLOC_ERR_VARIANT: return "flag or array not valid for the chosen optimizer variant";
        case DESLOC_ERR_TOO_LARGE: return "input exceeds the fixed scratch of the allocation-free entry point";
        default: return "unknown status";
    }
}

int desloc_last_hip_error(const desloc_ctx* ctx) {
    return ctx ? ctx->last_hip_error : g_init_hip_error;
}

uint32_t desloc_sync_mask_k(uint64_t t, uint64_t Kx, uint64_t Ku, uint64_t Kv) {
    uint32_t mask = 0;
    if (Kx != 0 && t % Kx == 0) mask |= DESLOC_SYNC_X;
    if (Ku != 0 && t % Ku == 0) mask |= DESLOC_SYNC_U;
    if (Kv != 0 && t % Kv == 0) mask |= DESLOC_SYNC_V;
    return mask;
}

int desloc_plan(const desloc_config* cfg, desloc_plan_info* out) {
    if (out == nullptr) return DESLOC_ERR_NULL;
    int rc = validate(cfg);
    if (rc != DESLOC_OK) return rc;
    try {
        Plan p;
        rc = make_plan(cfg, p);
        if (rc != DESLOC_OK) return rc;
        fill_info(p, cfg->variant, cfg->flags, cfg->M, cfg->chunk_elems != 0, out);
    } catch (const std::bad_alloc&) {
        return DESLOC_ERR_OOM;
    }
    return DESLOC_OK;
}

int desloc_init(const desloc_config* cfg, desloc_ctx** out) {
    if (out == nullptr) return DESLOC_ERR_NULL;
    int rc = validate(cfg);
    if (rc != DESLOC_OK) return rc;
    desloc_ctx* ctx = nullptr;
    try {
        ctx = new desloc_ctx();
        rc = make_plan(cfg, ctx->plan);
        if (rc != DESLOC_OK) {
            delete ctx;
            return rc;
        }
        ctx->variant = cfg->variant;
        ctx->M = cfg->M;
        ctx->grad_dtype = cfg->grad_dtype;
        ctx->flags = cfg->flags;
        ctx->n_tensors = cfg->n_tensors;
        ctx->Kx = cfg->Kx;
        ctx->Ku = cfg->Ku;
        ctx->Kv = cfg->variant == DESLOC_SGDM ? 0 : cfg->Kv;
        ctx->lr = cfg->lr;
        ctx->beta1 = cfg->beta1;
        ctx->beta2 = cfg->beta2;
        ctx->eps = cfg->eps;
        ctx->rho = cfg->rho;
        ctx->stream = static_cast<hipStream_t>(cfg->stream);
        ctx->user_chunk = cfg->chunk_elems != 0;
        ctx->lds_bytes = ungated_limiter(cfg->variant, ctx->plan.strided && !ctx->plan.ungated_table, cfg->flags);
        ctx->lds_bytes_gated = gated_limiter(cfg->variant, ctx->plan, cfg->M);
#ifdef DESLOC_TUNING
        // Knobs for launch-shape sweeps, compiled in only with -DDESLOC_TUNING (a production
        // build never reads the environment); out-of-range values are ignored.
        if (const char* env = std::getenv("DESLOC_LDS_BYTES")) {
            const long v = std::atol(env);
            if (v >= 0 && v <= 160 * 1024) ctx->lds_bytes = static_cast<uint32_t>(v);
        }
        if (const char* env = std::getenv("DESLOC_LDS_BYTES_GATED")) {
            const long v = std::atol(env);
            if (v >= 0 && v <= 160 * 1024) ctx->lds_bytes_gated = static_cast<uint32_t>(v);
        }
        if (const char* env = std::getenv("DESLOC_GATED_CHUNK")) {
            const long v = std::atol(env);
            if (v > 0 && v % TILE_ELEMS == 0 && v <= static_cast<long>(MAX_CHUNK_ELEMS))
                ctx->gated_chunk_elems = static_cast<uint32_t>(v);
        }
#endif
        ctx->numel.assign(cfg->numel, cfg->numel + cfg->n_tensors);
        const uint64_t cells = static_cast<uint64_t>(cfg->M) * cfg->n_tensors;
        void* const* src[N_ARRAYS] = {cfg->x, cfg->u, cfg->v, cfg->g, cfg->vmax};
        for (int a = 0; a < N_ARRAYS; ++a)
            if (src[a]) ctx->tab[a].assign(src[a], src[a] + cells);

        const Plan& p = ctx->plan;
        const uint64_t ns = p.segs.size();
        const uint32_t M = cfg->M;
        std::vector<uint64_t> h_ptrs(ns * N_ARRAYS * M, 0);
        for (uint64_t s = 0; s < ns; ++s) {
            const uint64_t k = p.segs[s].first_tensor;
            for (int a = 0; a < N_ARRAYS; ++a) {
                if (ctx->tab[a].empty()) continue;
                for (uint32_t m = 0; m < M; ++m)
                    h_ptrs[(s * N_ARRAYS + a) * M + m] =
                        reinterpret_cast<uint64_t>(ctx->tab[a][static_cast<uint64_t>(m) * cfg->n_tensors + k]);
            }
        }

        ctx->strided = p.strided ? 1 : 0;
        for (int a = 0; a < N_ARRAYS; ++a) {
            ctx->base[a] = p.base[a];
            ctx->rstride[a] = p.rstride[a];
        }

        hipError_t e = hipGetDevice(&ctx->device);
        if (e == hipSuccess) e = static_scratch_for(ctx->device, &ctx->static_scratch);
        if (e != hipSuccess) { rc = hip_fail(ctx, e); delete ctx; return rc; }
        ctx->h_bases.reserve(ns * cfg->M);
        ctx->h_row_index.reserve(ns + 1);
        ctx->h_offsets.reserve(ns + 1);
        ctx->h_numels.reserve(ns + 1);
        ctx->h_out.resize(2u * cfg->M);
        if (ns > 0) {
            auto upload = [&](void** dptr, const void* h, size_t bytes) -> hipError_t {
                hipError_t err = hipMalloc(dptr, bytes);
                if (err != hipSuccess) return err;
                return hipMemcpy(*dptr, h, bytes, hipMemcpyHostToDevice);
            };
            e = upload(reinterpret_cast<void**>(&ctx->d_ptrs), h_ptrs.data(), h_ptrs.size() * 8u);
            if (e == hipSuccess && (!ctx->strided || p.ungated_table)) {
                const uint32_t tchunk = p.table_chunk_elems;
                std::vector<ChunkRec> h_chunks(p.table_chunks);
                for (uint64_t s = 0; s < ns; ++s) {
                    const Segment& sg = p.segs[s];
                    const SegmentRecords nr = segment_records(sg, tchunk);
                    ChunkRec* r = h_chunks.data() + sg.chunk0;
                    // contiguous records over [from, to)
                    auto plain = [&](uint64_t from, uint64_t to) {
                        for (uint64_t at = from; at < to; at += tchunk, ++r) {
                            r->start = at;
                            r->seg = static_cast<uint32_t>(s);
                            r->len = to - at < tchunk ? static_cast<uint32_t>(to - at) : tchunk;
                        }
                    };
                    const uint64_t e1 = sg.pair_e0 + sg.pair_groups * PAIR_GROUP_ELEMS;
                    if (sg.pair_groups != 0) {
                        plain(0, sg.pair_e0);
                        for (uint64_t grp = 0; grp < sg.pair_groups; ++grp)
                            for (uint32_t j = 0; j < PAIR_GROUP_ELEMS / (2 * TILE_ELEMS); ++j, ++r) {
                                r->start = sg.pair_e0 + grp * PAIR_GROUP_ELEMS;
                                r->seg = static_cast<uint32_t>(s);
                                r->len = PAIRED_REC_FLAG | j;
                            }
                        plain(e1, sg.numel);
                    } else {
                        plain(0, sg.numel);
                    }
                    if (static_cast<uint64_t>(r - (h_chunks.data() + sg.chunk0)) != nr.total()) {
                        free_tables(ctx);
                        delete ctx;
                        return DESLOC_ERR_BAD_ARG;  // cannot happen: the plan and the records disagree
                    }
                }
                e = upload(reinterpret_cast<void**>(&ctx->d_chunks), h_chunks.data(),
                           h_chunks.size() * sizeof(ChunkRec));
            }
            if (e == hipSuccess && (cfg->flags & DESLOC_FLAG_NORM_CLIP)) {
                if (ctx->strided && !ctx->user_chunk) {
                    ctx->norm_chunk_elems = NORM_CHUNK_ELEMS;
                    ctx->norm_chunks = static_cast<uint32_t>(
                        (p.segs[0].numel + NORM_CHUNK_ELEMS - 1) / NORM_CHUNK_ELEMS);
                } else if (ctx->strided) {
                    ctx->norm_chunk_elems = p.chunk_elems;  // the caller's chunk size
                    ctx->norm_chunks = static_cast<uint32_t>(p.n_chunks);
                } else {
                    // table layouts: runs of up to NORM_CHUNK_ELEMS elements, segment by segment
                    std::vector<DiagChunk> runs;
                    for (uint64_t s = 0; s < ns; ++s)
                        for (uint64_t at = 0; at < p.segs[s].numel; at += NORM_CHUNK_ELEMS) {
                            const uint64_t left = p.segs[s].numel - at;
                            runs.push_back(DiagChunk{at, static_cast<uint32_t>(s),
                                                     static_cast<uint32_t>(left < NORM_CHUNK_ELEMS ? left : NORM_CHUNK_ELEMS)});
                        }
                    if (runs.size() > 0x7fffffffull) e = hipErrorInvalidValue;
                    ctx->norm_chunk_elems = NORM_CHUNK_ELEMS;
                    ctx->norm_chunks = static_cast<uint32_t>(runs.size());
                    if (e == hipSuccess && !runs.empty())
                        e = upload(reinterpret_cast<void**>(&ctx->d_norm_runs), runs.data(), runs.size() * sizeof(DiagChunk));
                }
                if (e == hipSuccess)
                    e = hipMalloc(reinterpret_cast<void**>(&ctx->d_partials),
                                  sizeof(double) * static_cast<size_t>(M) * (ctx->norm_chunks ? ctx->norm_chunks : 1u));
                if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&ctx->d_norms), sizeof(float) * 2u * M);
            }
            if (e != hipSuccess) {
                rc = (e == hipErrorOutOfMemory) ? DESLOC_ERR_OOM : hip_fail(ctx, e);
                free_tables(ctx);
                delete ctx;
                return rc;
            }
        }
        if (cfg->init_mode != DESLOC_INIT_AS_IS) {
            std::vector<uint64_t> seg_numel(ns);
            for (uint64_t s = 0; s < ns; ++s) seg_numel[s] = p.segs[s].numel;
            e = launch_init_states(ctx->d_ptrs, static_cast<int>(M), seg_numel.data(), ns,
                                   ctx->variant != DESLOC_SGDM, cfg->vmax != nullptr,
                                   cfg->init_mode == DESLOC_INIT_BROADCAST_REPLICA0, ctx->stream);
            if (e != hipSuccess) {
                rc = hip_fail(ctx, e);
                free_tables(ctx);
                delete ctx;
                return rc;
            }
        }
    } catch (const std::bad_alloc&) {
        if (ctx) {
            free_tables(ctx);
            delete ctx;
        }
        return DESLOC_ERR_OOM;
    }
    *out = ctx;
    return DESLOC_OK;
}

uint32_t desloc_sync_mask(const desloc_ctx* ctx, uint64_t t) {
    if (ctx == nullptr) return 0;
    return desloc_sync_mask_k(t, ctx->Kx, ctx->Ku, ctx->Kv);
}

int desloc_set_lr(desloc_ctx* ctx, float lr) {
    if (ctx == nullptr) return DESLOC_ERR_NULL;
    if (!std::isfinite(lr)) return DESLOC_ERR_BAD_ARG;
    ctx->lr = lr;
    return DESLOC_OK;
}

namespace {

// Update rule of step t (the first step of ADOPT can differ from the others).
int kind_for(const desloc_ctx* ctx, uint64_t t) {
    if (ctx->variant == DESLOC_ADAM) return (ctx->flags & DESLOC_FLAG_ADAM_LITERAL) ? KIND_ADAM_LITERAL : KIND_ADAM;
    if (ctx->variant == DESLOC_ADOPT) {
        if ((ctx->flags & DESLOC_FLAG_ADOPT_INIT_G0SQ) && t == 0) return KIND_ADOPT_T0;
        return (ctx->flags & DESLOC_FLAG_ADOPT_AVG_NORMALISER) ? KIND_ADOPT_AVGNORM : KIND_ADOPT;
    }
    return KIND_SGDM;
}

// Decomposition and occupancy limiter of a launch with sync mask `mask`.
LaunchArgs shaped_args(const desloc_ctx* ctx, uint32_t mask) {
    LaunchArgs a = base_args(ctx);
    if (mask != 0) a.lds_bytes = ctx->lds_bytes_gated;
    if (mask == 0 && ctx->strided && ctx->plan.ungated_table && a.numel0 != 0) {
        // a strided layout's launches without a gate take the table path over its single segment
        a.strided = 0;
        a.n_chunks = static_cast<uint32_t>(ctx->plan.table_chunks);
        a.chunk_elems = ctx->plan.table_chunk_elems;
    }
    if (mask != 0 && ctx->strided && !ctx->user_chunk && a.numel0 != 0)
        set_strided_grid(ctx->plan, a, ctx->gated_chunk_elems);
    // table layouts: the records hold two tiles (two wave slots of a paired group); gated steps
    // and the Adam / ADOPT steps without a gate give each a workgroup of its own, SGDM steps
    // without a gate (three read streams only) run best with the whole record in one workgroup
    bool split = mask != 0 || ctx->variant != DESLOC_SGDM;
#ifdef DESLOC_TUNING
    if (const char* env = std::getenv("DESLOC_UNGATED_SPLIT")) if (mask == 0) split = std::atoi(env) != 0;
#endif
    if (split && !a.strided && !ctx->user_chunk && a.chunk_elems == 2 * TILE_ELEMS) {
        a.split_log2 = 1;
        a.n_chunks *= 2;
    }
    return a;
}

}  // namespace

int desloc_step(desloc_ctx* ctx, uint64_t t) {
    if (ctx == nullptr) return DESLOC_ERR_NULL;
    // With a single replica the mean of a gated state is the state itself, bit for bit
    // (s / 1.0f == s): every step then takes the instantiations without a gate.
    const uint32_t mask = ctx->M == 1 ? 0u : desloc_sync_mask(ctx, t);
    const int kind = kind_for(ctx, t);
    LaunchArgs a = shaped_args(ctx, mask);
    StepScalars& sc = a.sc;
    sc.b1 = ctx->beta1;
    sc.omb1 = 1.0f - ctx->beta1;
    sc.b2 = ctx->beta2;
    sc.omb2 = 1.0f - ctx->beta2;
    sc.lr = ctx->lr;
    sc.eps = ctx->eps;
    sc.eps2 = ctx->eps * ctx->eps;
    sc.rho = ctx->rho;
    // Bias terms of the cited Adam step with exponent t + 1 (0-based loop, states seeded
    // at t = -1): formed in double, rounded once to fp32.
    const double tp1 = static_cast<double>(t) + 1.0;
    const double bc1 = 1.0 - std::pow(static_cast<double>(ctx->beta1), tp1);
    const double bc2 = 1.0 - std::pow(static_cast<double>(ctx->beta2), tp1);
    sc.step = static_cast<float>(static_cast<double>(ctx->lr) / bc1);
    sc.sbc2 = static_cast<float>(std::sqrt(bc2));
    sc.Mf = static_cast<float>(ctx->M);

    hipError_t e = hipSuccess;
    if ((ctx->flags & DESLOC_FLAG_NORM_CLIP) && ctx->d_norms != nullptr) {
        // pass 1 over the gradients: per-replica norms and factors, then the update pass
        // multiplies by the factor instead of clipping coordinates
        LaunchArgs na = base_args(ctx);
        na.chunk_elems = ctx->norm_chunk_elems;
        na.n_chunks = ctx->norm_chunks;
        e = launch_grad_norms(na, ctx->d_norm_runs, ctx->grad_dtype == DESLOC_BF16, ctx->rho, ctx->d_partials,
                              ctx->d_norms, ctx->d_norms + ctx->M, ctx->stream);
        if (e != hipSuccess) return hip_fail(ctx, e);
        a.gscale = ctx->d_norms + ctx->M;
        sc.rho = INFINITY;
    }
    const bool ams = (ctx->flags & DESLOC_FLAG_AMSGRAD) != 0;
    if ((ctx->flags & DESLOC_FLAG_POST_AVERAGE) && (mask != 0 || ams)) {
        // update-then-average; a step without any gate and without the AMSGrad state is the
        // same arithmetic in both orderings and takes the ordinary kernel below
        e = launch_step_post(kind, mask, ams, ctx->grad_dtype == DESLOC_BF16, a, ctx->stream);
    } else {
        e = launch_step(kind, mask, ctx->grad_dtype == DESLOC_BF16, a, ctx->stream);
    }
    if (e != hipSuccess) return hip_fail(ctx, e);
    return DESLOC_OK;
}

int desloc_read_grad_norms(desloc_ctx* ctx, float* host_dst, size_t count) {
    if (ctx == nullptr || host_dst == nullptr) return DESLOC_ERR_NULL;
    if (!(ctx->flags & DESLOC_FLAG_NORM_CLIP)) return DESLOC_ERR_VARIANT;
    if (count < ctx->M) return DESLOC_ERR_BAD_ARG;
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e);
    if (ctx->d_norms == nullptr) {  // no elements at all: every norm is 0
        for (uint32_t m = 0; m < ctx->M; ++m) host_dst[m] = 0.0f;
        return DESLOC_OK;
    }
    e = hipMemcpy(host_dst, ctx->d_norms, sizeof(float) * ctx->M, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(ctx, e);
    return DESLOC_OK;
}

namespace {

// Per-segment, per-replica base pointers of a caller table laid out like the state arrays;
// checks that tensors merged into one segment are adjacent in the caller's table too.
int segment_bases(const desloc_ctx* ctx, void* const* tab, std::vector<uint64_t>& bases) {
    const uint64_t nt = ctx->n_tensors;
    const uint32_t M = ctx->M;
    bases.assign(ctx->plan.segs.size() * M, 0);
    for (uint64_t k = 0; k < nt; ++k) {
        if (ctx->numel[k] == 0) continue;
        const uint64_t s = ctx->plan.tensor_seg[k];
        for (uint32_t m = 0; m < M; ++m) {
            const uint64_t p = reinterpret_cast<uint64_t>(tab[static_cast<uint64_t>(m) * nt + k]);
            if (p == 0) return DESLOC_ERR_NULL;
            if (p % 4u) return DESLOC_ERR_ALIGN;
            if (ctx->plan.tensor_off[k] == 0) bases[s * M + m] = p;
            else if (p != bases[s * M + m] + ctx->plan.tensor_off[k] * 4u) return DESLOC_ERR_BAD_ARG;
        }
    }
    return DESLOC_OK;
}

int check_state_array(const desloc_ctx* ctx, int which) {
    if (which != DESLOC_X && which != DESLOC_U && which != DESLOC_V && which != DESLOC_VMAX)
        return DESLOC_ERR_BAD_ARG;
    if (which == DESLOC_V && ctx->variant == DESLOC_SGDM) return DESLOC_ERR_VARIANT;
    if (which == DESLOC_VMAX && !(ctx->flags & DESLOC_FLAG_AMSGRAD)) return DESLOC_ERR_VARIANT;
    return DESLOC_OK;
}

}  // namespace

namespace {

// Builds, once per context, the tensor-aligned records of the batched diagnostic and of the
// snapshot copy, and their partial-sum scratch.
int ensure_diag_tables(desloc_ctx* ctx) {
    if (ctx->diag_tables) return DESLOC_OK;
    const uint64_t nt = ctx->n_tensors;
    if (nt > 0x7fffffffull) return DESLOC_ERR_BAD_ARG;
    std::vector<DiagChunk> recs;
    std::vector<uint32_t> first(nt, 0), count(nt, 0);
    for (uint64_t k = 0; k < nt; ++k) {
        const uint64_t n = ctx->numel[k];
        first[k] = static_cast<uint32_t>(recs.size());
        if (n == 0) continue;
        const uint64_t pieces = (n + DIAG_CHUNK_ELEMS - 1) / DIAG_CHUNK_ELEMS;
        if (recs.size() + pieces > 0x7fffffffull) return DESLOC_ERR_BAD_ARG;
        for (uint64_t q = 0; q < pieces; ++q) {
            const uint64_t off = q * DIAG_CHUNK_ELEMS;
            recs.push_back(DiagChunk{ctx->plan.tensor_off[k] + off, static_cast<uint32_t>(ctx->plan.tensor_seg[k]),
                                     static_cast<uint32_t>(n - off < DIAG_CHUNK_ELEMS ? n - off : DIAG_CHUNK_ELEMS)});
        }
        count[k] = static_cast<uint32_t>(pieces);
    }
    const uint32_t P = static_cast<uint32_t>(recs.size());
    auto upload = [&](void** d, const void* h, size_t bytes) -> hipError_t {
        hipError_t e = hipMalloc(d, bytes ? bytes : 16u);
        if (e == hipSuccess && bytes) e = hipMemcpy(*d, h, bytes, hipMemcpyHostToDevice);
        return e;
    };
    hipError_t e = upload(reinterpret_cast<void**>(&ctx->d_diag_chunks), recs.data(), recs.size() * sizeof(DiagChunk));
    if (e == hipSuccess) e = upload(reinterpret_cast<void**>(&ctx->d_diag_first), first.data(), nt * 4u);
    if (e == hipSuccess) e = upload(reinterpret_cast<void**>(&ctx->d_diag_count), count.data(), nt * 4u);
    if (e == hipSuccess)
        e = hipMalloc(reinterpret_cast<void**>(&ctx->d_diag_part), sizeof(double) * 2u * ctx->M * (P ? P : 1u));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&ctx->d_refbase),
                                       8u * (ctx->plan.segs.size() * ctx->M + 1u));
    if (e != hipSuccess) {
        // a later call starts over: give back what this one got
        void** got[] = {reinterpret_cast<void**>(&ctx->d_diag_chunks), reinterpret_cast<void**>(&ctx->d_diag_first),
                        reinterpret_cast<void**>(&ctx->d_diag_count), reinterpret_cast<void**>(&ctx->d_diag_part),
                        reinterpret_cast<void**>(&ctx->d_refbase)};
        for (void** q : got) {
            if (*q) (void)hipFree(*q);
            *q = nullptr;
        }
        return e == hipErrorOutOfMemory ? DESLOC_ERR_OOM : hip_fail(ctx, e);
    }
    ctx->diag_P = P;
    ctx->diag_tables = true;
    return DESLOC_OK;
}

// Makes `ref` the bound reference: validates its layout, uploads its segment base table (only
// when it differs from the one already bound).
int bind_reference(desloc_ctx* ctx, void* const* ref) {
    int rc = ensure_diag_tables(ctx);
    if (rc != DESLOC_OK) return rc;
    std::vector<uint64_t> bases;
    rc = segment_bases(ctx, ref, bases);
    if (rc != DESLOC_OK) return rc;
    if (ctx->ref_bound && bases == ctx->bound_bases) return DESLOC_OK;
    int vec_ok = 1;
    for (uint64_t b : bases) vec_ok &= (b % 16u == 0);
    // earlier work on the stream may still read the old table
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e == hipSuccess && !bases.empty())
        e = hipMemcpy(ctx->d_refbase, bases.data(), bases.size() * 8u, hipMemcpyHostToDevice);
    if (e != hipSuccess) return hip_fail(ctx, e);
    ctx->bound_bases.swap(bases);
    ctx->ref_vec_ok = vec_ok;
    ctx->ref_bound = true;
    return DESLOC_OK;
}

}  // namespace

int desloc_bind_reference(desloc_ctx* ctx, void* const* ref) {
    if (ctx == nullptr || ref == nullptr) return DESLOC_ERR_NULL;
    try {
        return bind_reference(ctx, ref);
    } catch (const std::bad_alloc&) {
        return DESLOC_ERR_OOM;
    }
}

int desloc_snapshot_state(desloc_ctx* ctx, int which, void* const* dst) {
    if (ctx == nullptr || dst == nullptr) return DESLOC_ERR_NULL;
    int rc = check_state_array(ctx, which);
    if (rc != DESLOC_OK) return rc;
    try {
        rc = bind_reference(ctx, dst);
    } catch (const std::bad_alloc&) {
        return DESLOC_ERR_OOM;
    }
    if (rc != DESLOC_OK) return rc;
    hipError_t e = launch_snapshot_copy(ctx->d_ptrs, which, ctx->d_refbase, ctx->M, ctx->d_diag_chunks, ctx->diag_P,
                                        ctx->plan.total_numel, ctx->ref_vec_ok, ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e);
    return DESLOC_OK;
}

int desloc_state_change_tensors(desloc_ctx* ctx, int which, float* change_dev, float* base_dev) {
    if (ctx == nullptr || change_dev == nullptr || base_dev == nullptr) return DESLOC_ERR_NULL;
    int rc = check_state_array(ctx, which);
    if (rc != DESLOC_OK) return rc;
    if (!ctx->ref_bound) return DESLOC_ERR_BAD_ARG;
    hipError_t e = launch_state_change_tensors(ctx->d_ptrs, which, ctx->d_refbase, ctx->M, ctx->d_diag_chunks,
                                               ctx->diag_P, ctx->d_diag_first, ctx->d_diag_count, ctx->n_tensors,
                                               ctx->ref_vec_ok, ctx->d_diag_part, change_dev, base_dev, ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e);
    return DESLOC_OK;
}

namespace {

constexpr uint32_t DIAG_MAX_CHUNK_ELEMS = 1u << 22;
constexpr size_t STATIC_OUT_BYTES = 8192;          // results: 2 * M floats, M <= 1024

inline size_t round_up_256(size_t v) { return (v + 255u) / 256u * 256u; }

// Shared body of desloc_state_change and desloc_state_change_static.  use_static: every device
// buffer is carved out of this GPU's static scratch array and nothing is allocated, on the
// device or on the host (the staging vectors were sized at init).
int state_change_impl(desloc_ctx* ctx, int which, int64_t tensor, void* const* ref, float* change_out,
                      float* base_out, size_t count, bool use_static) {
    if (ctx == nullptr || ref == nullptr || change_out == nullptr || base_out == nullptr)
        return DESLOC_ERR_NULL;
    int rc = check_state_array(ctx, which);
    if (rc != DESLOC_OK) return rc;
    if (count < ctx->M) return DESLOC_ERR_BAD_ARG;
    if (tensor != DESLOC_ALL_TENSORS && (tensor < 0 || static_cast<uint64_t>(tensor) >= ctx->n_tensors))
        return DESLOC_ERR_BAD_ARG;
    if (use_static && ctx->static_scratch == nullptr) return DESLOC_ERR_TOO_LARGE;  // device index beyond the table
    const uint32_t M = ctx->M;
    std::vector<uint64_t>&bases = ctx->h_bases, &row_index = ctx->h_row_index, &offsets = ctx->h_offsets,
                         &numels = ctx->h_numels;
    row_index.clear();
    offsets.clear();
    numels.clear();
    rc = segment_bases(ctx, ref, bases);  // within the capacity reserved at init
    if (rc != DESLOC_OK) return rc;
    int vec_ok = 1;  // the state's segment bases are 16-byte aligned (checked at init); the reference's may not be
    for (uint64_t b : bases) vec_ok &= (b % 16u == 0);
    if (tensor == DESLOC_ALL_TENSORS) {
        for (uint64_t s = 0; s < ctx->plan.segs.size(); ++s) {
            row_index.push_back(s);
            offsets.push_back(0);
            numels.push_back(ctx->plan.segs[s].numel);
        }
    } else if (ctx->numel[tensor] != 0) {
        row_index.push_back(ctx->plan.tensor_seg[tensor]);
        offsets.push_back(ctx->plan.tensor_off[tensor]);
        numels.push_back(ctx->numel[tensor]);
    }
    uint32_t chunk = DIAG_CHUNK_ELEMS;
    auto partials = [&](uint32_t c) {
        uint64_t P = 0;
        for (uint64_t n : numels) P += (n + c - 1) / c;
        return P;
    };
    uint64_t P = partials(chunk);
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e);
    if (P == 0) {
        for (uint32_t m = 0; m < M; ++m) change_out[m] = base_out[m] = 0.0f;
        return DESLOC_OK;
    }
    uint64_t* d_ref = nullptr;
    double* d_part = nullptr;
    float* d_out = nullptr;
    if (use_static) {
        // [results | reference bases | partial sums]; larger chunks until the partial sums fit
        const size_t ref_off = STATIC_OUT_BYTES;
        const size_t part_off = ref_off + round_up_256(bases.size() * 8u);
        if (part_off >= DESLOC_STATIC_SCRATCH_BYTES) return DESLOC_ERR_TOO_LARGE;
        const size_t room = DESLOC_STATIC_SCRATCH_BYTES - part_off;
        while (sizeof(double) * 2u * M * P > room) {
            if (chunk >= DIAG_MAX_CHUNK_ELEMS) return DESLOC_ERR_TOO_LARGE;
            chunk *= 2;
            P = partials(chunk);
        }
        d_out = reinterpret_cast<float*>(ctx->static_scratch);
        d_ref = reinterpret_cast<uint64_t*>(ctx->static_scratch + ref_off);
        d_part = reinterpret_cast<double*>(ctx->static_scratch + part_off);
    } else {
        if (P > 0x7fffffffull) return DESLOC_ERR_BAD_ARG;
        const size_t need[3] = {bases.size() * 8u, sizeof(double) * 2u * M * P, sizeof(float) * 2u * M};
        for (int k = 0; k < 3 && e == hipSuccess; ++k) {
            if (ctx->diag_cap[k] >= need[k]) continue;
            if (ctx->d_diag[k]) (void)hipFree(ctx->d_diag[k]);
            ctx->d_diag[k] = nullptr;
            ctx->diag_cap[k] = 0;
            e = hipMalloc(&ctx->d_diag[k], need[k]);
            if (e == hipSuccess) ctx->diag_cap[k] = need[k];
        }
        d_ref = static_cast<uint64_t*>(ctx->d_diag[0]);
        d_part = static_cast<double*>(ctx->d_diag[1]);
        d_out = static_cast<float*>(ctx->d_diag[2]);
    }
    if (e == hipSuccess) e = hipMemcpy(d_ref, bases.data(), bases.size() * 8u, hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = launch_state_change(ctx->d_ptrs + static_cast<uint64_t>(which) * M, d_ref, M,
                                static_cast<uint32_t>(numels.size()), row_index.data(), offsets.data(),
                                numels.data(), chunk, vec_ok, d_part, static_cast<uint32_t>(P), d_out, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e == hipSuccess) e = hipMemcpy(ctx->h_out.data(), d_out, sizeof(float) * 2u * M, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return e == hipErrorOutOfMemory ? DESLOC_ERR_OOM : hip_fail(ctx, e);
    for (uint32_t m = 0; m < M; ++m) {
        change_out[m] = ctx->h_out[m];
        base_out[m] = ctx->h_out[M + m];
    }
    return DESLOC_OK;
}

}  // namespace

int desloc_state_change(desloc_ctx* ctx, int which, int64_t tensor, void* const* ref, float* change_out,
                        float* base_out, size_t count) {
    return state_change_impl(ctx, which, tensor, ref, change_out, base_out, count, false);
}

int desloc_state_change_static(desloc_ctx* ctx, int which, int64_t tensor, void* const* ref,
                               float* change_out, float* base_out, size_t count) {
    return state_change_impl(ctx, which, tensor, ref, change_out, base_out, count, true);
}

int desloc_get_plan(const desloc_ctx* ctx, desloc_plan_info* out) {
    if (ctx == nullptr || out == nullptr) return DESLOC_ERR_NULL;
    desloc_plan_info info;
    fill_info(ctx->plan, ctx->variant, ctx->flags, ctx->M, ctx->user_chunk, &info);
    info.lds_limiter_bytes[0] = ctx->lds_bytes;
    info.lds_limiter_bytes[1] = ctx->lds_bytes_gated;
    for (int k = 0; k < 2; ++k)
        info.intended_workgroups[k] = info.lds_limiter_bytes[k] ? LDS_PER_CU_BYTES / info.lds_limiter_bytes[k] : 0u;
    if (ctx->strided && !ctx->user_chunk) info.gated_chunk_elems = ctx->gated_chunk_elems;
    // What the runtime grants: asked for the kernels an ordinary step (t = 1) and the first
    // gated step after t = 0 launch.  Host-side query, nothing is enqueued.
    const bool post = (ctx->flags & DESLOC_FLAG_POST_AVERAGE) != 0;
    if (!post && ctx->plan.total_numel != 0) {
        uint64_t tg = 0;
        for (uint64_t K : {ctx->Kx, ctx->Ku, ctx->Kv})
            if (K != 0 && (tg == 0 || K < tg)) tg = K;
        const uint64_t steps[2] = {1, ctx->M > 1 ? tg : 0};
        for (int k = 0; k < 2; ++k) {
            if (k == 1 && steps[k] == 0) continue;
            const uint32_t mask = k == 0 ? 0u : desloc_sync_mask(ctx, steps[k]);
            if (k == 0 && ctx->M > 1 && desloc_sync_mask(ctx, 1) != 0) continue;  // every step is gated
            const LaunchArgs a = shaped_args(ctx, mask);
            uint32_t resident = 0;
            hipError_t e = launch_step(kind_for(ctx, steps[k]), mask, ctx->grad_dtype == DESLOC_BF16, a,
                                       ctx->stream, &resident);
            if (e != hipSuccess) {
                (void)hipGetLastError();
                continue;  // reported as "not queried"
            }
            info.resident_workgroups[k] = resident;
        }
    }
    *out = info;
    return DESLOC_OK;
}

int desloc_synchronize(desloc_ctx* ctx) {
    if (ctx == nullptr) return DESLOC_ERR_NULL;
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e);
    return DESLOC_OK;
}

int desloc_read_state(desloc_ctx* ctx, int which, int replica, int64_t tensor, void* host_dst,
                      size_t dst_bytes) {
    if (ctx == nullptr || host_dst == nullptr) return DESLOC_ERR_NULL;
    if (which < DESLOC_X || which > DESLOC_VMAX) return DESLOC_ERR_BAD_ARG;
    if (which == DESLOC_V && ctx->variant == DESLOC_SGDM) return DESLOC_ERR_VARIANT;
    if (which == DESLOC_VMAX && !(ctx->flags & DESLOC_FLAG_AMSGRAD)) return DESLOC_ERR_VARIANT;
    if (replica != DESLOC_REPLICA_MEAN && (replica < 0 || replica >= static_cast<int>(ctx->M)))
        return DESLOC_ERR_BAD_ARG;
    if (tensor != DESLOC_ALL_TENSORS && (tensor < 0 || static_cast<uint64_t>(tensor) >= ctx->n_tensors))
        return DESLOC_ERR_BAD_ARG;
    // Ranges to copy, as (segment, element offset, count): one tensor, or every segment in order
    // (segments are formed in tensor order and are contiguous, so their concatenation is the
    // concatenation of all tensors without padding).  Large ranges are cut into pieces so that
    // the temporaries stay bounded.
    struct Range { uint64_t seg, off, n; };
    constexpr uint64_t PIECE = 1ull << 26;
    std::vector<Range> ranges;
    uint64_t count = 0;
    try {
        auto add = [&](uint64_t seg, uint64_t off, uint64_t n) {
            count += n;
            for (uint64_t done = 0; done < n; done += PIECE)
                ranges.push_back(Range{seg, off + done, n - done < PIECE ? n - done : PIECE});
        };
        if (tensor == DESLOC_ALL_TENSORS) {
            for (uint64_t s = 0; s < ctx->plan.segs.size(); ++s) add(s, 0, ctx->plan.segs[s].numel);
        } else if (ctx->numel[tensor] != 0) {
            add(ctx->plan.tensor_seg[tensor], ctx->plan.tensor_off[tensor], ctx->numel[tensor]);
        }
    } catch (const std::bad_alloc&) {
        return DESLOC_ERR_OOM;
    }
    if (dst_bytes / 4u < count) return DESLOC_ERR_BAD_ARG;
    uint64_t largest = 0;
    for (const Range& r : ranges) largest = r.n > largest ? r.n : largest;

    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e);
    if (count == 0) return DESLOC_OK;

    const bool bf16 = which == DESLOC_G && ctx->grad_dtype == DESLOC_BF16;
    const size_t esz = bf16 ? 2u : 4u;
    float* dst = static_cast<float*>(host_dst);
    std::vector<uint16_t> h_half;
    try {
        if (bf16 && replica != DESLOC_REPLICA_MEAN) h_half.resize(largest);
    } catch (const std::bad_alloc&) {
        return DESLOC_ERR_OOM;
    }
    float* d_tmp = nullptr;
    if (replica == DESLOC_REPLICA_MEAN) {
        // the temporary for the device-side mean is kept in the context and only grows
        if (ctx->mean_cap < largest * 4u) {
            if (ctx->d_mean) (void)hipFree(ctx->d_mean);
            ctx->d_mean = nullptr;
            ctx->mean_cap = 0;
            e = hipMalloc(reinterpret_cast<void**>(&ctx->d_mean), largest * 4u);
            if (e != hipSuccess) return e == hipErrorOutOfMemory ? DESLOC_ERR_OOM : hip_fail(ctx, e);
            ctx->mean_cap = largest * 4u;
        }
        d_tmp = ctx->d_mean;
    }
    int rc = DESLOC_OK;
    for (size_t q = 0; q < ranges.size() && rc == DESLOC_OK; ++q) {
        const Range& r = ranges[q];
        if (replica == DESLOC_REPLICA_MEAN) {
            const uint64_t* row = ctx->d_ptrs + (r.seg * N_ARRAYS + static_cast<uint64_t>(which)) * ctx->M;
            e = launch_replica_mean(row, static_cast<int>(ctx->M), bf16, r.off, r.n, d_tmp, ctx->stream);
            if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
            if (e == hipSuccess) e = hipMemcpy(dst, d_tmp, r.n * 4u, hipMemcpyDeviceToHost);
        } else {
            const uint64_t k = ctx->plan.segs[r.seg].first_tensor;
            const char* src = static_cast<const char*>(
                                  ctx->tab[which][static_cast<uint64_t>(replica) * ctx->n_tensors + k]) +
                              r.off * esz;
            if (bf16) {
                e = hipMemcpy(h_half.data(), src, r.n * 2u, hipMemcpyDeviceToHost);
                if (e == hipSuccess) {
                    for (uint64_t i = 0; i < r.n; ++i) {
                        const uint32_t bits = static_cast<uint32_t>(h_half[i]) << 16;
                        std::memcpy(&dst[i], &bits, 4);
                    }
                }
            } else {
                e = hipMemcpy(dst, src, r.n * 4u, hipMemcpyDeviceToHost);
            }
        }
        if (e != hipSuccess) rc = hip_fail(ctx, e);
        dst += r.n;
    }
    return rc;
}

int desloc_destroy(desloc_ctx* ctx) {
    if (ctx == nullptr) return DESLOC_OK;
    (void)hipStreamSynchronize(ctx->stream);
    free_tables(ctx);
    delete ctx;
    return DESLOC_OK;
}

}  // extern "C"
