// C-ABI entry points declared in include/tperm.h and include/tperm_tuning.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/tperm_tuning.h"
#include "kernels.hpp"
#include "plan.hpp"
#include "verify.hpp"

using tperm::Plan;

// One executable plan plus the launch geometry resolved for it on first use.
struct PlanSlot {
    Plan* p = nullptr;
    // (device ordinal + 1) << 32 | resident workgroups of this plan's kernel on that whole
    // device; 0 = not resolved yet.  Resolved again when the current device is another one.
    std::atomic<uint64_t> geometry{0};
};

struct tperm_plan_s {
    PlanSlot base;  // the problem as given
    // Optional twin for 4-byte problems whose canonical stride-1 dimension stays in front
    // and has an even extent: the same bytes described as 8-byte elements with that extent
    // halved.  Half the memory instructions per byte; needs 8-byte aligned pointers.
    PlanSlot wide;
    std::atomic<uint64_t> cu_count{0};  // (device ordinal + 1) << 32 | compute units, for the copy class
    ~tperm_plan_s() {
        delete base.p;
        delete wide.p;
    }
};

namespace {

tperm_status_t device_cu_count(int* num_cu) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return TPERM_ERR_HIP;
    }
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
        (void)hipGetLastError();
        return TPERM_ERR_HIP;
    }
    *num_cu = n;
    return TPERM_OK;
}

// Compute units of the current device, remembered per plan for the device it was asked on.
tperm_status_t cached_cu_count(tperm_plan_s* handle, int* num_cu) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return TPERM_ERR_HIP;
    }
    const uint64_t seen = handle->cu_count.load(std::memory_order_acquire);
    if ((seen >> 32) == (uint64_t)dev + 1u) {
        *num_cu = (int)(seen & 0xFFFFFFFFu);
        return TPERM_OK;
    }
    tperm_status_t st = device_cu_count(num_cu);
    if (st != TPERM_OK) return st;
    handle->cu_count.store((((uint64_t)dev + 1u) << 32) | (uint64_t)*num_cu, std::memory_order_release);
    return TPERM_OK;
}

// Number of workgroups to launch for a tile plan: as many as the current device keeps resident.
tperm_status_t resolve_grid(PlanSlot* h, int* grid) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return TPERM_ERR_HIP;
    }
    const uint64_t seen = h->geometry.load(std::memory_order_acquire);
    int mb = 0;
    if ((seen >> 32) == (uint64_t)dev + 1u) {
        mb = (int)(seen & 0xFFFFFFFFu);
    } else {
        int num_cu = 0;
        tperm_status_t st = device_cu_count(&num_cu);
        if (st != TPERM_OK) return st;
        int per_cu = 0;
        if (tperm::tile_blocks_per_cu(*h->p, &per_cu) != hipSuccess || per_cu < 1) {
            (void)hipGetLastError();
            return TPERM_ERR_HIP;
        }
        if (h->p->blocks_per_cu > 0 && per_cu > h->p->blocks_per_cu) per_cu = h->p->blocks_per_cu;
        mb = per_cu * num_cu;
        h->geometry.store((((uint64_t)dev + 1u) << 32) | (uint64_t)mb, std::memory_order_release);
    }
    int64_t g = h->p->tile.num_tiles;
    if (g > mb) g = mb;
    if (h->p->tile.grid_mode != 0u) {
        g = (g + 7) / 8 * 8;  // whole rounds over the 8 XCDs
    }
    *grid = (int)g;
    return TPERM_OK;
}

tperm_status_t wrap(Plan* p, tperm_plan_t* out) {
    tperm_plan_s* h = new (std::nothrow) tperm_plan_s();
    if (h == nullptr) {
        delete p;
        return TPERM_ERR_NOMEM;
    }
    h->base.p = p;
    *out = h;
    return TPERM_OK;
}

// True when the canonical problem can be described in 8-byte units: 4-byte elements, the
// stride-1 dimension first on both sides, an even extent there.  (A canonical rank of 1
// is the plain copy, which already moves 16 bytes per lane.)
bool pairable(const tperm::Canonical& c, size_t elem) {
    return elem == 4 && c.rank >= 2 && c.perm[0] == 0 && (c.dims[0] % 2) == 0;
}

// The paired problem: canonical dims with the leading extent halved, elements of 8 bytes.
void paired_problem(const tperm::Canonical& c, int64_t* dims, int* perm) {
    for (int z = 0; z < c.rank; ++z) {
        dims[z] = c.dims[z];
        perm[z] = c.perm[z];
    }
    dims[0] /= 2;
}

}  // namespace

extern "C" {

tperm_status_t tperm_plan_create_ex(tperm_plan_t* plan, int rank, const int64_t* dims,
                                    const int* perm, size_t elem_size,
                                    const tperm_plan_opts_t* opts) {
    if (plan == nullptr) return TPERM_ERR_NULL;
    *plan = nullptr;
    Plan* p = nullptr;
    tperm_status_t st = tperm::create_plan(&p, rank, dims, perm, elem_size, opts);
    if (st != TPERM_OK) return st;
    st = wrap(p, plan);
    if (st != TPERM_OK) return st;
    const bool forced = opts != nullptr && (opts->kernel_class != TPERM_KERNEL_AUTO ||
                                            opts->m > 0 || opts->k > 0);
    const int pair = opts ? opts->pair_elems : 0;
    const int vec2 = opts ? opts->vec2 : 0;
    if (vec2 == 0 && !forced && !pairable(p->c, elem_size) &&
        (p->kclass == TPERM_KERNEL_TILED || p->kclass == TPERM_KERNEL_PACKED)) {
        // twin that moves the elements in pairs, for pointers aligned to two elements
        tperm_plan_opts_t o;
        std::memset(&o, 0, sizeof(o));
        o.lds_pad = -1;
        if (opts) o = *opts;
        o.vec2 = 2;
        Plan* w = nullptr;
        // without options the twin reuses the candidate already chosen (no second search)
        const tperm_status_t ws =
            opts == nullptr
                ? tperm::create_plan_with_candidate(&w, rank, dims, perm, elem_size, p->cand, true)
                : tperm::create_plan(&w, rank, dims, perm, elem_size, &o);
        if (ws == TPERM_OK) {
            if (w->vec2) (*plan)->wide.p = w;
            else delete w;
        }
    }
    if ((pair == 2 || (pair == 0 && !forced)) && pairable(p->c, elem_size)) {
        int64_t wdims[TPERM_MAX_RANK];
        int wperm[TPERM_MAX_RANK];
        paired_problem(p->c, wdims, wperm);
        Plan* w = nullptr;
        // a twin that cannot be built (forced options that do not fit it) is simply left out
        if (tperm::create_plan(&w, p->c.rank, wdims, wperm, 8, opts) == TPERM_OK)
            (*plan)->wide.p = w;
    }
    return TPERM_OK;
}

tperm_status_t tperm_plan_create(tperm_plan_t* plan, int rank, const int64_t* dims,
                                 const int* perm, size_t elem_size) {
    return tperm_plan_create_ex(plan, rank, dims, perm, elem_size, nullptr);
}

tperm_status_t tperm_plan_create_forced(tperm_plan_t* plan, int rank, const int64_t* dims,
                                        const int* perm, size_t elem_size, int kernel_class) {
    tperm_plan_opts_t o;
    std::memset(&o, 0, sizeof(o));
    o.lds_pad = -1;
    o.kernel_class = kernel_class;
    return tperm_plan_create_ex(plan, rank, dims, perm, elem_size, &o);
}

tperm_status_t tperm_plan_destroy(tperm_plan_t plan) {
    if (plan == nullptr) return TPERM_ERR_NULL;
    delete plan;
    return TPERM_OK;
}

static tperm_status_t execute_impl(tperm_plan_t plan, const void* in, void* out, void* hip_stream,
                                   bool accumulate) {
    if (plan == nullptr || in == nullptr || out == nullptr) return TPERM_ERR_NULL;
    if (in == out) return TPERM_ERR_ALIAS;
    const uintptr_t a = (uintptr_t)in, b = (uintptr_t)out;
    const uintptr_t elem = (uintptr_t)plan->base.p->elem;
    if ((a % elem) != 0 || (b % elem) != 0) return TPERM_ERR_ALIGN;
    PlanSlot* slot = &plan->base;
    const uintptr_t pair_mask = 2u * elem - 1u;  // the twin moves two elements per access
    // pairs inside line-aligned windows are formed on absolute addresses (written pairs) or
    // read with element alignment (read pairs): no demand on the pointers
    const auto any_alignment = [](const Plan* q) { return q->vec2 && q->align_out; };
    if (plan->wide.p != nullptr && !accumulate &&
        (((a | b) & pair_mask) == 0 || any_alignment(plan->wide.p)))
        slot = &plan->wide;
    const Plan& p = *slot->p;
    // a plan that moves pairs by itself (forced through the options) has no plain twin
    if (p.vec2 && (accumulate || (((a | b) & pair_mask) != 0 && !any_alignment(&p))))
        return accumulate ? TPERM_ERR_KERNEL : TPERM_ERR_ALIGN;
    const size_t nbytes = (size_t)p.c.volume * (size_t)p.elem;
    if ((a < b && a + nbytes > b) || (b < a && b + nbytes > a)) return TPERM_ERR_ALIAS;
    // accumulating kernels exist for the default workgroup size only
    if (accumulate && p.threads != 256 && p.kclass != TPERM_KERNEL_COPY && p.kclass != TPERM_KERNEL_NAIVE)
        return TPERM_ERR_KERNEL;
    hipStream_t stream = (hipStream_t)hip_stream;
    hipError_t err = hipSuccess;
    switch (p.kclass) {
        case TPERM_KERNEL_COPY: {
            int num_cu = 0;
            tperm_status_t st = cached_cu_count(plan, &num_cu);
            if (st != TPERM_OK) return st;
            err = accumulate ? tperm::launch_accumulate_copy(in, out, nbytes, p.elem, num_cu, stream)
                             : tperm::launch_copy(in, out, nbytes, p.elem, num_cu, stream);
            break;
        }
        case TPERM_KERNEL_NAIVE:
            err = tperm::launch_naive(p, in, out, stream, accumulate);
            break;
        case TPERM_KERNEL_ROWCOPY:
        case TPERM_KERNEL_TILED:
        case TPERM_KERNEL_PACKED: {
            if (!tperm::tile_kernel_exists(p, accumulate)) return TPERM_ERR_KERNEL;
            int grid = 0;
            tperm_status_t st = resolve_grid(slot, &grid);
            if (st != TPERM_OK) return st;
            err = tperm::launch_tile(p, in, out, stream, grid, accumulate);
            break;
        }
        default:
            return TPERM_ERR_INTERNAL;
    }
    if (err != hipSuccess) {
        (void)hipGetLastError();
        return TPERM_ERR_HIP;
    }
    return TPERM_OK;
}

tperm_status_t tperm_execute(tperm_plan_t plan, const void* in, void* out, void* hip_stream) {
    return execute_impl(plan, in, out, hip_stream, false);
}

tperm_status_t tperm_execute_accumulate(tperm_plan_t plan, const void* in, void* out,
                                        void* hip_stream) {
    return execute_impl(plan, in, out, hip_stream, true);
}

// Argument rules shared by the checking entry points: the verdict word and the scratch are
// device pointers aligned to 8 bytes, and the scratch is large enough and apart from the data.
static tperm_status_t check_verify_args(const void* a, const void* b, size_t nbytes, const uint64_t* verdict,
                                        const void* scratch, size_t scratch_bytes, size_t needed) {
    if (verdict == nullptr || scratch == nullptr) return TPERM_ERR_NULL;
    if (((reinterpret_cast<uintptr_t>(verdict) | reinterpret_cast<uintptr_t>(scratch)) & 7u) != 0) return TPERM_ERR_ALIGN;
    if (scratch_bytes < needed) return TPERM_ERR_TOO_LARGE;
    const uintptr_t s0 = reinterpret_cast<uintptr_t>(scratch), s1 = s0 + needed;
    const uintptr_t v0 = reinterpret_cast<uintptr_t>(verdict), v1 = v0 + 8;
    if (s0 < v1 && v0 < s1) return TPERM_ERR_ALIAS;
    for (const void* t : {a, b}) {
        const uintptr_t t0 = reinterpret_cast<uintptr_t>(t), t1 = t0 + nbytes;
        if ((s0 < t1 && t0 < s1) || (v0 < t1 && t0 < v1)) return TPERM_ERR_ALIAS;
    }
    return TPERM_OK;
}

tperm_status_t tperm_execute_verified(tperm_plan_t plan, const void* in, void* out, void* hip_stream,
                                      uint64_t* verdict, void* workspace, size_t workspace_bytes) {
    if (plan == nullptr || in == nullptr || out == nullptr) return TPERM_ERR_NULL;
    const Plan& p = *plan->base.p;
    const uint64_t vol = (uint64_t)p.c.volume;
    tperm_status_t st = check_verify_args(in, out, (size_t)vol * (size_t)p.elem, verdict, workspace, workspace_bytes,
                                          tperm::verify_scratch_bytes(vol));
    if (st != TPERM_OK) return st;
    st = execute_impl(plan, in, out, hip_stream, false);
    if (st != TPERM_OK) return st;
    if (tperm::launch_multiset_compare(in, out, vol, p.elem, workspace, verdict, (hipStream_t)hip_stream) != hipSuccess) {
        (void)hipGetLastError();
        return TPERM_ERR_HIP;
    }
    return TPERM_OK;
}

tperm_status_t tperm_execute_verified_static(tperm_plan_t plan, const void* in, void* out,
                                             void* hip_stream, uint64_t* verdict) {
    if (plan == nullptr || in == nullptr || out == nullptr || verdict == nullptr) return TPERM_ERR_NULL;
    // the library's own scratch holds the partial results of tensors up to this size only
    if ((uint64_t)plan->base.p->c.volume > tperm::kVerifyStaticMaxElems) return TPERM_ERR_TOO_LARGE;
    void* scratch = nullptr;
    if (tperm::verify_static_scratch(&scratch) != hipSuccess) {
        (void)hipGetLastError();
        return TPERM_ERR_HIP;
    }
    return tperm_execute_verified(plan, in, out, hip_stream, verdict, scratch, tperm::kVerifyStaticBytes);
}

tperm_status_t tperm_multiset_compare(const void* a, const void* b, int64_t count, size_t elem_size,
                                      uint64_t* verdict, void* workspace, size_t workspace_bytes,
                                      void* hip_stream) {
    if (a == nullptr || b == nullptr) return TPERM_ERR_NULL;
    if (elem_size != 4 && elem_size != 8) return TPERM_ERR_ELEM_SIZE;
    if (count < 1) return TPERM_ERR_DIMS;
    if (count >= ((int64_t)1 << 31)) return TPERM_ERR_TOO_LARGE;
    if (((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) % elem_size) != 0) return TPERM_ERR_ALIGN;
    tperm_status_t st = check_verify_args(a, b, (size_t)count * elem_size, verdict, workspace, workspace_bytes,
                                          tperm::verify_scratch_bytes((uint64_t)count));
    if (st != TPERM_OK) return st;
    if (tperm::launch_multiset_compare(a, b, (uint64_t)count, (int)elem_size, workspace, verdict,
                                       (hipStream_t)hip_stream) != hipSuccess) {
        (void)hipGetLastError();
        return TPERM_ERR_HIP;
    }
    return TPERM_OK;
}

tperm_status_t tperm_plan_describe(tperm_plan_t plan, tperm_plan_info_t* info) {
    if (plan == nullptr || info == nullptr) return TPERM_ERR_NULL;
    const Plan& p = plan->wide.p ? *plan->wide.p : *plan->base.p;
    std::memset(info, 0, sizeof(*info));
    info->paired = (plan->wide.p && !plan->wide.p->vec2) ? 1 : 0;
    info->kernel_class = p.kclass;
    info->elem_size = p.elem;
    info->rank = plan->base.p->rank;
    info->canon_rank = p.c.rank;
    for (int z = 0; z < p.c.rank; ++z) {
        info->canon_dims[z] = p.c.dims[z];
        info->canon_perm[z] = p.c.perm[z];
        info->tile_extent[z] = 1;
    }
    info->volume = p.c.volume;
    const bool tiled = p.kclass == TPERM_KERNEL_ROWCOPY || p.kclass == TPERM_KERNEL_TILED ||
                       p.kclass == TPERM_KERNEL_PACKED;
    if (tiled) {
        for (int z = 0; z < p.c.rank; ++z) info->tile_extent[z] = p.cand.t[z];
        info->tile_volume = p.cand.tile_vol;
        info->run_in = p.cand.run_in;
        info->run_out = p.cand.run_out;
        info->num_tiles = p.cand.num_tiles;
        info->m = p.cand.m;
        info->k = p.cand.k;
        info->nreg = p.nreg;
        info->threads = p.threads;
        info->lds_bytes = p.lds_bytes;
        info->lds_pad = p.lds_pad;
        info->score = p.cand.score;
        info->blocks_per_cu = p.blocks_per_cu;
        info->cache_policy = tperm::tile_launch_policy(p, false, true);
        info->align_out = p.align_out ? 1 : 0;
        info->loads_first = p.loads_first ? 1 : 0;
        info->vec2 = p.vec2 ? 1 : 0;
        info->large = p.big ? 1 : 0;
    } else {
        info->large = (p.kclass == TPERM_KERNEL_NAIVE && p.big) ? 1 : 0;
        info->threads = 256;
    }
    return TPERM_OK;
}

tperm_status_t tperm_device_memory_info(int* bus_width_bits, int* memory_clock_khz, int* compute_units) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return TPERM_ERR_HIP;
    }
    const struct {
        int* out;
        hipDeviceAttribute_t attr;
    } want[] = {{bus_width_bits, hipDeviceAttributeMemoryBusWidth},
                {memory_clock_khz, hipDeviceAttributeMemoryClockRate},
                {compute_units, hipDeviceAttributeMultiprocessorCount}};
    for (const auto& w : want) {
        if (w.out == nullptr) continue;
        if (hipDeviceGetAttribute(w.out, w.attr, dev) != hipSuccess) {
            (void)hipGetLastError();
            return TPERM_ERR_HIP;
        }
    }
    return TPERM_OK;
}

tperm_status_t tperm_plan_model(tperm_plan_t plan, tperm_model_t* model) {
    if (plan == nullptr || model == nullptr) return TPERM_ERR_NULL;
    // the plan that runs on suitably aligned pointers, as tperm_plan_describe reports it
    return tperm::model_plan(plan->wide.p ? *plan->wide.p : *plan->base.p, model);
}

tperm_status_t tperm_plan_index_map(tperm_plan_t plan, int64_t* out_to_in) {
    if (plan == nullptr || out_to_in == nullptr) return TPERM_ERR_NULL;
    if (plan->wide.p == nullptr) return tperm::index_map(*plan->base.p, out_to_in);
    if (plan->wide.p->vec2) return tperm::index_map(*plan->wide.p, out_to_in);
    // The paired twin is the plan that runs: evaluate its map over pairs, then spell it out
    // per 4-byte element (pair q holds elements 2q and 2q+1 on both sides).
    const int64_t pairs = plan->wide.p->c.volume;
    std::vector<int64_t> m((size_t)pairs);
    tperm_status_t st = tperm::index_map(*plan->wide.p, m.data());
    if (st != TPERM_OK) return st;
    for (int64_t q = 0; q < pairs; ++q) {
        out_to_in[2 * q] = m[(size_t)q] < 0 ? -1 : 2 * m[(size_t)q];
        out_to_in[2 * q + 1] = m[(size_t)q] < 0 ? -1 : 2 * m[(size_t)q] + 1;
    }
    return TPERM_OK;
}

tperm_status_t tperm_plan_candidate_count(int rank, const int64_t* dims, const int* perm,
                                          size_t elem_size, int* count) {
    if (count == nullptr) return TPERM_ERR_NULL;
    *count = 0;
    tperm_status_t st = tperm::validate(rank, dims, perm, elem_size);
    if (st != TPERM_OK) return st;
    tperm::Canonical c;
    tperm::canonicalise(rank, dims, perm, &c);
    *count = (int)tperm::enumerate_candidates(c, (int)elem_size).size();
    return TPERM_OK;
}

tperm_status_t tperm_plan_create_candidate(tperm_plan_t* plan, int rank, const int64_t* dims,
                                           const int* perm, size_t elem_size, int index) {
    if (plan == nullptr) return TPERM_ERR_NULL;
    *plan = nullptr;
    tperm_status_t st = tperm::validate(rank, dims, perm, elem_size);
    if (st != TPERM_OK) return st;
    tperm::Canonical c;
    tperm::canonicalise(rank, dims, perm, &c);
    const std::vector<tperm::Candidate> cands = tperm::enumerate_candidates(c, (int)elem_size);
    if (index < 0 || index >= (int)cands.size()) return TPERM_ERR_KERNEL;
    Plan* p = nullptr;
    st = tperm::create_plan_with_candidate(&p, rank, dims, perm, elem_size, cands[index]);
    if (st != TPERM_OK) return st;
    st = wrap(p, plan);
    if (st != TPERM_OK) return st;
    {
        // the same candidate moving pairs, for suitably aligned pointers (as tperm_plan_create)
        Plan* w = nullptr;
        if (tperm::create_plan_with_candidate(&w, rank, dims, perm, elem_size, cands[index], true) ==
            TPERM_OK) {
            if (w->vec2) (*plan)->wide.p = w;
            else delete w;
        }
    }
    return TPERM_OK;
}

// Caller-supplied device memory that measurement runs sweep between timed executions, so that
// a tensor small enough to stay in the last-level cache is timed as it would arrive from HBM.
struct Scratch {
    void* p = nullptr;
    size_t bytes = 0;
};

// Times every candidate plan of (rank, dims, perm, elem) on (in, out) and hands back the
// fastest as a bare Plan.  With scratch, every timed execution is preceded by a copy of one
// half of the scratch onto the other (outside the timed interval).
static tperm_status_t measure_best(int rank, const int64_t* dims, const int* perm, size_t elem,
                                   const std::vector<tperm::Candidate>& cands, const void* in,
                                   void* out, void* hip_stream, Plan** winner, bool vec2,
                                   const Scratch& scratch) {
    *winner = nullptr;
    hipStream_t stream = (hipStream_t)hip_stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return TPERM_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return TPERM_ERR_HIP;
    }
    int num_cu = 0;
    const size_t half = scratch.p != nullptr ? (scratch.bytes / 2) & ~(size_t)255 : 0;
    if (half > 0 && device_cu_count(&num_cu) != TPERM_OK) {
        (void)hipEventDestroy(e0);
        (void)hipEventDestroy(e1);
        return TPERM_ERR_HIP;
    }
    tperm_plan_t best = nullptr;
    float best_ms = 0.f;
    tperm_status_t result = TPERM_OK;
    for (const auto& cd : cands) {
        Plan* p = nullptr;
        if (tperm::create_plan_with_candidate(&p, rank, dims, perm, elem, cd, vec2) != TPERM_OK) continue;
        tperm_plan_t h = nullptr;
        if (wrap(p, &h) != TPERM_OK) continue;
        float ms = 0.f;
        // warm-up; its status tells whether this candidate can run at all
        tperm_status_t est = tperm_execute(h, in, out, hip_stream);
        if (est == TPERM_ERR_KERNEL) {  // no kernel variant for this candidate: not a failure
            tperm_plan_destroy(h);
            continue;
        }
        bool ok = est == TPERM_OK;
        auto run = [&]() {
            est = tperm_execute(h, in, out, hip_stream);
            return est == TPERM_OK;
        };
        if (ok && half == 0) {
            ok = hipEventRecord(e0, stream) == hipSuccess;
            for (int rep = 0; ok && rep < 3; ++rep) ok = run();
            ok = ok && hipEventRecord(e1, stream) == hipSuccess;
            ok = ok && hipEventSynchronize(e1) == hipSuccess;
            ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
        } else if (ok) {
            ms = 1e30f;  // the fastest of five: single short launches are noisy
            for (int rep = 0; ok && rep < 5; ++rep) {
                float one = 0.f;
                ok = tperm::launch_copy(scratch.p, static_cast<char*>(scratch.p) + half, half, 4, num_cu,
                                        stream) == hipSuccess;
                ok = ok && hipEventRecord(e0, stream) == hipSuccess;
                ok = ok && run();
                ok = ok && hipEventRecord(e1, stream) == hipSuccess;
                ok = ok && hipEventSynchronize(e1) == hipSuccess;
                ok = ok && hipEventElapsedTime(&one, e0, e1) == hipSuccess;
                ms = std::min(ms, one);
            }
        }
        if (!ok) {
            (void)hipGetLastError();
            tperm_plan_destroy(h);
            // the status tperm_execute gave (aliasing, alignment, ...) if that is what failed
            result = est != TPERM_OK ? est : TPERM_ERR_HIP;
            break;
        }
        if (best == nullptr || ms < best_ms) {
            if (best) tperm_plan_destroy(best);
            best = h;
            best_ms = ms;
        } else {
            tperm_plan_destroy(h);
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (result != TPERM_OK) {
        if (best) tperm_plan_destroy(best);
        return result;
    }
    if (best == nullptr) return TPERM_ERR_KERNEL;
    *winner = best->base.p;
    best->base.p = nullptr;
    tperm_plan_destroy(best);
    return TPERM_OK;
}

tperm_status_t tperm_plan_create_measured(tperm_plan_t* plan, int rank, const int64_t* dims,
                                          const int* perm, size_t elem_size, const void* in,
                                          void* out, void* hip_stream, int max_candidates) {
    return tperm_plan_create_measured_cold(plan, rank, dims, perm, elem_size, in, out, hip_stream,
                                           max_candidates, nullptr, 0);
}

tperm_status_t tperm_plan_create_measured_cold(tperm_plan_t* plan, int rank, const int64_t* dims,
                                               const int* perm, size_t elem_size, const void* in,
                                               void* out, void* hip_stream, int max_candidates,
                                               void* scratch, size_t scratch_bytes) {
    if (plan == nullptr) return TPERM_ERR_NULL;
    *plan = nullptr;
    if (in == nullptr || out == nullptr) return TPERM_ERR_NULL;
    if (in == out) return TPERM_ERR_ALIAS;
    Scratch sweep;
    if (scratch != nullptr && scratch_bytes >= 512) {
        if ((reinterpret_cast<uintptr_t>(scratch) & 15u) != 0) return TPERM_ERR_ALIGN;
        sweep.p = scratch;
        sweep.bytes = scratch_bytes;
    }
    const tperm_status_t vst = tperm::validate(rank, dims, perm, elem_size);
    if (vst != TPERM_OK) return vst;
    size_t nbytes = elem_size;
    for (int z = 0; z < rank; ++z) nbytes *= (size_t)dims[z];
    {
        // the two tensors must not overlap (the same rule as tperm_execute)
        const uintptr_t i0 = reinterpret_cast<uintptr_t>(in), o0 = reinterpret_cast<uintptr_t>(out);
        if (i0 < o0 + nbytes && o0 < i0 + nbytes) return TPERM_ERR_ALIAS;
    }
    if (sweep.p != nullptr) {
        // the scratch must not touch the tensors it is meant to push out of the caches
        const uintptr_t s0 = reinterpret_cast<uintptr_t>(scratch), s1 = s0 + scratch_bytes;
        for (const void* t : {in, (const void*)out}) {
            const uintptr_t t0 = reinterpret_cast<uintptr_t>(t), t1 = t0 + nbytes;
            if (s0 < t1 && t0 < s1) return TPERM_ERR_ALIAS;
        }
    }
    tperm_status_t st = TPERM_OK;
    const uintptr_t a = (uintptr_t)in, b = (uintptr_t)out;
    if ((a % elem_size) != 0 || (b % elem_size) != 0) return TPERM_ERR_ALIGN;
    tperm::Canonical c;
    tperm::canonicalise(rank, dims, perm, &c);
    if (c.rank < 2) return tperm_plan_create(plan, rank, dims, perm, elem_size);
    auto trimmed = [&](std::vector<tperm::Candidate> v) {
        if (max_candidates > 0 && (int)v.size() > max_candidates) v.resize(max_candidates);
        return v;
    };
    if (pairable(c, elem_size) && ((a | b) & 7u) == 0) {
        // The paired description is what runs on these pointers: measure its candidates and
        // keep the heuristic plan of the problem as given for unaligned pointers.
        int64_t wdims[TPERM_MAX_RANK];
        int wperm[TPERM_MAX_RANK];
        paired_problem(c, wdims, wperm);
        tperm::Canonical wc;
        tperm::canonicalise(c.rank, wdims, wperm, &wc);
        const auto cands = trimmed(tperm::enumerate_candidates(wc, 8));
        if (!cands.empty()) {
            tperm_plan_opts_t off;
            std::memset(&off, 0, sizeof(off));
            off.lds_pad = -1;
            off.pair_elems = 1;
            st = tperm_plan_create_ex(plan, rank, dims, perm, elem_size, &off);
            if (st != TPERM_OK) return st;
            Plan* w = nullptr;
            st = measure_best(c.rank, wdims, wperm, 8, cands, in, out, hip_stream, &w, false, sweep);
            if (st != TPERM_OK) {
                tperm_plan_destroy(*plan);
                *plan = nullptr;
                return st;
            }
            (*plan)->wide.p = w;
            return TPERM_OK;
        }
    }
    const auto cands = trimmed(tperm::enumerate_candidates(c, (int)elem_size));
    if (cands.empty()) return TPERM_ERR_KERNEL;
    const bool try_vec2 = ((a | b) & (2u * (uintptr_t)elem_size - 1u)) == 0;
    Plan* p = nullptr;
    st = measure_best(rank, dims, perm, elem_size, cands, in, out, hip_stream, &p, try_vec2, sweep);
    if (st != TPERM_OK) return st;
    if (!p->vec2) return wrap(p, plan);
    // the winner moves pairs: keep it for aligned pointers beside a plain heuristic plan
    tperm_plan_opts_t off;
    std::memset(&off, 0, sizeof(off));
    off.lds_pad = -1;
    off.vec2 = 1;
    st = tperm_plan_create_ex(plan, rank, dims, perm, elem_size, &off);
    if (st != TPERM_OK) {
        delete p;
        return st;
    }
    (*plan)->wide.p = p;
    return TPERM_OK;
}

tperm_status_t tperm_copy_bytes(const void* in, void* out, size_t nbytes, void* hip_stream) {
    if (in == nullptr || out == nullptr) return TPERM_ERR_NULL;
    if (in == out) return TPERM_ERR_ALIAS;
    if ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)nbytes) & 3u) != 0) return TPERM_ERR_ALIGN;
    int num_cu = 0;
    tperm_status_t st = device_cu_count(&num_cu);
    if (st != TPERM_OK) return st;
    if (tperm::launch_copy(in, out, nbytes, 4, num_cu, (hipStream_t)hip_stream) != hipSuccess) {
        (void)hipGetLastError();
        return TPERM_ERR_HIP;
    }
    return TPERM_OK;
}

const char* tperm_status_string(tperm_status_t s) {
    switch (s) {
        case TPERM_OK: return "ok";
        case TPERM_ERR_NULL: return "null pointer argument";
        case TPERM_ERR_RANK: return "rank out of range";
        case TPERM_ERR_DIMS: return "extent < 1";
        case TPERM_ERR_PERM: return "not a permutation";
        case TPERM_ERR_ELEM_SIZE: return "element size must be 4 or 8";
        case TPERM_ERR_TOO_LARGE: return "tensor too large";
        case TPERM_ERR_ALIAS: return "input and output overlap";
        case TPERM_ERR_ALIGN: return "pointer not aligned to the element size";
        case TPERM_ERR_HIP: return "HIP call failed";
        case TPERM_ERR_NOMEM: return "out of host memory";
        case TPERM_ERR_KERNEL: return "kernel class or options cannot run this problem";
        case TPERM_ERR_INTERNAL: return "plan self-check failed";
    }
    return "unknown status";
}

}  // extern "C"
