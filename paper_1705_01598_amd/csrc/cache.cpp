// Process-wide plan cache behind tperm_transpose / tperm_cache_*.
//
// Creating a plan costs a fraction of a millisecond with the heuristic selector and tens of
// milliseconds with measurement-based selection (Section 2.3), so callers that see the same
// (extents, permutation, element size) again and again want the plan kept.  The cache owns
// its plans; entries are handed out as shared references so that an entry evicted or cleared
// by one thread stays alive until the executes other threads have in flight on the host
// have returned.
#include <cstring>
#include <list>
#include <map>
#include <memory>
#include <mutex>
#include <vector>

#include "../../include/tperm.h"

namespace {

struct Key {
    int rank;
    int elem;
    int64_t dims[TPERM_MAX_RANK];
    int perm[TPERM_MAX_RANK];
    bool operator<(const Key& o) const {
        if (rank != o.rank) return rank < o.rank;
        if (elem != o.elem) return elem < o.elem;
        int c = std::memcmp(dims, o.dims, sizeof(int64_t) * (size_t)rank);
        if (c != 0) return c < 0;
        return std::memcmp(perm, o.perm, sizeof(int) * (size_t)rank) < 0;
    }
};

using PlanRef = std::shared_ptr<tperm_plan_s>;

struct Entry {
    PlanRef plan;
    bool measured = false;
    std::list<Key>::iterator lru;  // position in the recency list
};

constexpr size_t kCapacity = 4096;

std::mutex g_mutex;
std::map<Key, Entry> g_map;
std::list<Key> g_recent;  // front = most recently used
int64_t g_hits = 0, g_misses = 0;

PlanRef make_ref(tperm_plan_t p) {
    return PlanRef(p, [](tperm_plan_s* q) { tperm_plan_destroy(q); });
}

// Arguments must already be known to be a valid problem (rank in range, non-null arrays).
Key make_key(int rank, const int64_t* dims, const int* perm, size_t elem) {
    Key k;
    std::memset(&k, 0, sizeof(k));
    k.rank = rank;
    k.elem = (int)elem;
    for (int z = 0; z < rank; ++z) {
        k.dims[z] = dims[z];
        k.perm[z] = perm[z];
    }
    return k;
}

void touch(Entry& e, const Key& k) {
    g_recent.erase(e.lru);
    g_recent.push_front(k);
    e.lru = g_recent.begin();
}

// Caller holds g_mutex.
void install(const Key& k, PlanRef plan, bool measured) {
    auto it = g_map.find(k);
    if (it != g_map.end()) {
        it->second.plan = std::move(plan);
        it->second.measured = measured;
        touch(it->second, k);
        return;
    }
    while (g_map.size() >= kCapacity && !g_recent.empty()) {
        g_map.erase(g_recent.back());
        g_recent.pop_back();
    }
    g_recent.push_front(k);
    Entry e;
    e.plan = std::move(plan);
    e.measured = measured;
    e.lru = g_recent.begin();
    g_map.emplace(k, std::move(e));
}

tperm_status_t lookup_or_create(int rank, const int64_t* dims, const int* perm, size_t elem,
                                PlanRef* out) {
    if (dims == nullptr || perm == nullptr) return TPERM_ERR_NULL;
    if (rank < 1 || rank > TPERM_MAX_RANK) return TPERM_ERR_RANK;
    const Key k = make_key(rank, dims, perm, elem);
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        auto it = g_map.find(k);
        if (it != g_map.end()) {
            ++g_hits;
            touch(it->second, k);
            *out = it->second.plan;
            return TPERM_OK;
        }
        ++g_misses;
    }
    // plan creation runs outside the lock; two threads racing on one key both build a plan
    // and the second install wins, which is harmless
    tperm_plan_t p = nullptr;
    tperm_status_t st = tperm_plan_create(&p, rank, dims, perm, elem);
    if (st != TPERM_OK) return st;
    PlanRef ref = make_ref(p);
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        auto it = g_map.find(k);
        if (it != g_map.end() && it->second.measured) {
            ref = it->second.plan;  // a tuned plan arrived meanwhile: keep it
        } else {
            install(k, ref, false);
        }
    }
    *out = ref;
    return TPERM_OK;
}

}  // namespace

extern "C" {

tperm_status_t tperm_transpose(int rank, const int64_t* dims, const int* perm, size_t elem_size,
                               const void* in, void* out, void* hip_stream) {
    PlanRef ref;
    tperm_status_t st = lookup_or_create(rank, dims, perm, elem_size, &ref);
    if (st != TPERM_OK) return st;
    return tperm_execute(ref.get(), in, out, hip_stream);
}

tperm_status_t tperm_transpose_accumulate(int rank, const int64_t* dims, const int* perm,
                                          size_t elem_size, const void* in, void* out,
                                          void* hip_stream) {
    PlanRef ref;
    tperm_status_t st = lookup_or_create(rank, dims, perm, elem_size, &ref);
    if (st != TPERM_OK) return st;
    return tperm_execute_accumulate(ref.get(), in, out, hip_stream);
}

tperm_status_t tperm_cache_tune(int rank, const int64_t* dims, const int* perm, size_t elem_size,
                                const void* in, void* out, void* hip_stream) {
    if (dims == nullptr || perm == nullptr) return TPERM_ERR_NULL;
    if (rank < 1 || rank > TPERM_MAX_RANK) return TPERM_ERR_RANK;
    tperm_plan_t p = nullptr;
    tperm_status_t st =
        tperm_plan_create_measured(&p, rank, dims, perm, elem_size, in, out, hip_stream, 0);
    if (st != TPERM_OK) return st;
    const Key k = make_key(rank, dims, perm, elem_size);
    std::lock_guard<std::mutex> lock(g_mutex);
    install(k, make_ref(p), true);
    return TPERM_OK;
}

tperm_status_t tperm_cache_stats(int64_t* entries, int64_t* hits, int64_t* misses) {
    std::lock_guard<std::mutex> lock(g_mutex);
    if (entries) *entries = (int64_t)g_map.size();
    if (hits) *hits = g_hits;
    if (misses) *misses = g_misses;
    return TPERM_OK;
}

tperm_status_t tperm_cache_clear(void) {
    std::vector<PlanRef> doomed;  // destroyed after the lock is released
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        doomed.reserve(g_map.size());
        for (auto& kv : g_map) doomed.push_back(std::move(kv.second.plan));
        g_map.clear();
        g_recent.clear();
        g_hits = 0;
        g_misses = 0;
    }
    return TPERM_OK;
}

}  // extern "C"
