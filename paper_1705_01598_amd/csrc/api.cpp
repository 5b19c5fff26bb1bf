// C-ABI entry points declared in include/tperm.h.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/tperm.h"
#include "kernels.hpp"
#include "plan.hpp"

using tperm::Plan;

struct tperm_plan_s {
    Plan* p;
    std::atomic<int> max_blocks{0};  // resident workgroups on the whole device; 0 = unknown
    std::atomic<int> num_cu{0};
};

namespace {

tperm_status_t device_cu_count(int* num_cu) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return TPERM_ERR_HIP;
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
        return TPERM_ERR_HIP;
    *num_cu = n;
    return TPERM_OK;
}

// Number of workgroups to launch for a tile plan: as many as the device keeps resident.
tperm_status_t resolve_grid(tperm_plan_s* h, int* grid) {
    int mb = h->max_blocks.load(std::memory_order_acquire);
    if (mb == 0) {
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
        h->num_cu.store(num_cu, std::memory_order_release);
        h->max_blocks.store(mb, std::memory_order_release);
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
    h->p = p;
    *out = h;
    return TPERM_OK;
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
    return wrap(p, plan);
}

tperm_status_t tperm_plan_create(tperm_plan_t* plan, int rank, const int64_t* dims,
                                 const int* perm, size_t elem_size) {
    return tperm_plan_create_ex(plan, rank, dims, perm, elem_size, nullptr);
}

tperm_status_t tperm_plan_destroy(tperm_plan_t plan) {
    if (plan == nullptr) return TPERM_ERR_NULL;
    delete plan->p;
    delete plan;
    return TPERM_OK;
}

static tperm_status_t execute_impl(tperm_plan_t plan, const void* in, void* out, void* hip_stream,
                                   bool accumulate) {
    if (plan == nullptr || in == nullptr || out == nullptr) return TPERM_ERR_NULL;
    if (in == out) return TPERM_ERR_ALIAS;
    const Plan& p = *plan->p;
    const uintptr_t a = (uintptr_t)in, b = (uintptr_t)out;
    if ((a % (uintptr_t)p.elem) != 0 || (b % (uintptr_t)p.elem) != 0) return TPERM_ERR_ALIGN;
    const size_t nbytes = (size_t)p.c.volume * (size_t)p.elem;
    if ((a < b && a + nbytes > b) || (b < a && b + nbytes > a)) return TPERM_ERR_ALIAS;
    // accumulating kernels exist for the default workgroup size and store mode only
    if (accumulate && (p.align_out || (p.threads != 256 && p.kclass != TPERM_KERNEL_COPY &&
                                       p.kclass != TPERM_KERNEL_NAIVE)))
        return TPERM_ERR_KERNEL;
    hipStream_t stream = (hipStream_t)hip_stream;
    hipError_t err = hipSuccess;
    switch (p.kclass) {
        case TPERM_KERNEL_COPY: {
            int num_cu = plan->num_cu.load(std::memory_order_acquire);
            if (num_cu == 0) {
                tperm_status_t st = device_cu_count(&num_cu);
                if (st != TPERM_OK) return st;
                plan->num_cu.store(num_cu, std::memory_order_release);
            }
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
            int grid = 0;
            tperm_status_t st = resolve_grid(plan, &grid);
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

tperm_status_t tperm_plan_describe(tperm_plan_t plan, tperm_plan_info_t* info) {
    if (plan == nullptr || info == nullptr) return TPERM_ERR_NULL;
    const Plan& p = *plan->p;
    std::memset(info, 0, sizeof(*info));
    info->kernel_class = p.kclass;
    info->elem_size = p.elem;
    info->rank = p.rank;
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
        info->cache_policy = p.cache_policy;
        info->align_out = p.align_out ? 1 : 0;
    } else {
        info->threads = 256;
    }
    return TPERM_OK;
}

tperm_status_t tperm_plan_index_map(tperm_plan_t plan, int64_t* out_to_in) {
    if (plan == nullptr || out_to_in == nullptr) return TPERM_ERR_NULL;
    return tperm::index_map(*plan->p, out_to_in);
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
    return wrap(p, plan);
}

tperm_status_t tperm_plan_create_measured(tperm_plan_t* plan, int rank, const int64_t* dims,
                                          const int* perm, size_t elem_size, const void* in,
                                          void* out, void* hip_stream, int max_candidates) {
    if (plan == nullptr) return TPERM_ERR_NULL;
    *plan = nullptr;
    if (in == nullptr || out == nullptr) return TPERM_ERR_NULL;
    if (in == out) return TPERM_ERR_ALIAS;
    tperm_status_t st = tperm::validate(rank, dims, perm, elem_size);
    if (st != TPERM_OK) return st;
    tperm::Canonical c;
    tperm::canonicalise(rank, dims, perm, &c);
    if (c.rank < 2) return tperm_plan_create(plan, rank, dims, perm, elem_size);
    std::vector<tperm::Candidate> cands = tperm::enumerate_candidates(c, (int)elem_size);
    if (cands.empty()) return TPERM_ERR_KERNEL;
    if (max_candidates > 0 && (int)cands.size() > max_candidates) cands.resize(max_candidates);
    hipStream_t stream = (hipStream_t)hip_stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return TPERM_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return TPERM_ERR_HIP;
    }
    tperm_plan_t best = nullptr;
    float best_ms = 0.f;
    tperm_status_t result = TPERM_OK;
    for (const auto& cd : cands) {
        Plan* p = nullptr;
        if (tperm::create_plan_with_candidate(&p, rank, dims, perm, elem_size, cd) != TPERM_OK)
            continue;
        tperm_plan_t h = nullptr;
        if (wrap(p, &h) != TPERM_OK) continue;
        float ms = 0.f;
        bool ok = tperm_execute(h, in, out, hip_stream) == TPERM_OK;  // warm-up
        ok = ok && hipEventRecord(e0, stream) == hipSuccess;
        for (int rep = 0; ok && rep < 3; ++rep) ok = tperm_execute(h, in, out, hip_stream) == TPERM_OK;
        ok = ok && hipEventRecord(e1, stream) == hipSuccess;
        ok = ok && hipEventSynchronize(e1) == hipSuccess;
        ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
        if (!ok) {
            (void)hipGetLastError();
            tperm_plan_destroy(h);
            result = TPERM_ERR_HIP;
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
    *plan = best;
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
