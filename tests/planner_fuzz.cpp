// Host-only fuzz driver for the planner, meant to be built with AddressSanitizer and
// UndefinedBehaviorSanitizer (see test_planner_host.py).  It links plan.cpp alone (the
// planner has no HIP dependency), creates plans for random problems and options, and checks
// every plan's index map for being a bijection of 0..vol-1.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <random>
#include <vector>

#include "../paper_1705_01598_amd/csrc/plan.hpp"

int main(int argc, char** argv) {
    const int iters = argc > 1 ? atoi(argv[1]) : 400;
    std::mt19937_64 rng(12345);
    int made = 0, rejected = 0, windows = 0, pair_windows = 0;
    for (int it = 0; it < iters; ++it) {
        const int rank = 1 + (int)(rng() % 16);
        int64_t dims[TPERM_MAX_RANK];
        int perm[TPERM_MAX_RANK];
        int64_t vol = 1;
        for (int z = 0; z < rank; ++z) {
            const int64_t cap = rank > 8 ? 3 : (rank > 4 ? 7 : 40);
            dims[z] = 1 + (int64_t)(rng() % cap);
            if (vol * dims[z] > 200000) dims[z] = 1;
            vol *= dims[z];
            perm[z] = z;
        }
        for (int z = rank - 1; z > 0; --z) std::swap(perm[z], perm[rng() % (z + 1)]);
        // every fourth problem of rank 2-4 gets a long leading output dim, so that the
        // line-aligned window form (chunks of whole lines along it) can apply
        const bool long_q0 = rank >= 2 && rank <= 4 && (it % 4) == 3 && perm[0] != 0;
        if (long_q0) {
            vol /= dims[perm[0]];
            dims[perm[0]] = 40 + (int64_t)(rng() % 300);
            for (int z = 0; z < rank && vol * dims[perm[0]] > 400000; ++z)
                if (z != perm[0] && dims[z] > 1) {
                    vol /= dims[z];
                    dims[z] = 1 + dims[z] / 4;
                    vol *= dims[z];
                }
            vol *= dims[perm[0]];
        }
        tperm_plan_opts_t o;
        std::memset(&o, 0, sizeof(o));
        o.lds_pad = -1;
        const size_t elem = ((it / 4) & 1) ? 4 : 8;
        const int mode = long_q0 ? 2 : (int)(rng() % 4);
        if (mode == 1) o.kernel_class = 1 + (int)(rng() % 5);
        if (mode == 0 && (rng() % 2)) o.selector = 1;  // tile chosen by the analytical model
        if (mode >= 2) {
            o.kernel_class = TPERM_KERNEL_PACKED;
            o.m = 1 + (int)(rng() % rank);
            o.k = 1 + (int)(rng() % rank);
            o.tile_in = (int64_t)(rng() % 50);
            o.tile_out = (int64_t)(rng() % 50);
            o.grid_mode = (int)(rng() % 9);
            o.window_in = (int)(rng() % 20);
            o.window_out = (int)(rng() % 20);
            o.threads = (rng() % 2) ? 64 : 256;
            o.lds_buffers = (int)(rng() % 3);
            o.align_out = (int)(rng() % 3);
            if (long_q0) {
                o.align_out = 2;
                // make the line-aligned window form likely: one leading output dim in the
                // tile, chunked in whole 128-byte lines
                o.k = 1;
                o.tile_out = (int64_t)(128 / (int)elem) * (1 + (int64_t)(rng() % 3));
                if (rng() % 2) o.tile_in &= ~(int64_t)1;  // pairs need an even tile extent
                o.threads = 256;
                o.vec2 = 0;
            }
            o.lds_pad = (int)(rng() % 8) - 1;
            o.vec2 = (int)(rng() % 3);
            if (long_q0 && elem == 4 && (rng() % 2)) {
                // pairs inside the windows: one input dim in the tile, even extent along it
                o.vec2 = 2;
                o.m = 1;
                o.tile_in = 2 + 2 * (int64_t)(rng() % 24);
            }
            o.loads_first = (int)(rng() % 3);
            o.tile_order = (int)(rng() % 3);
        }
        if ((rng() % 5) == 0) o.large = 1;  // planned the way tensors of 4 GiB and more are
        tperm::Plan* p = nullptr;
        const tperm_status_t st = tperm::create_plan(&p, rank, dims, perm, elem, &o);
        if (st != TPERM_OK) {
            if (st != TPERM_ERR_KERNEL) {
                std::printf("unexpected status %d at iteration %d\n", (int)st, it);
                return 1;
            }
            ++rejected;
            continue;
        }
        if (o.large == 1 && p->kclass != TPERM_KERNEL_COPY &&
            (!p->big || p->loads_first || (p->kclass != TPERM_KERNEL_NAIVE && (!p->use_lds || p->threads != 256)))) {
            std::printf("a large plan uses a form large tensors have no kernel for, iteration %d\n", it);
            return 1;
        }
        std::vector<int64_t> map((size_t)vol);
        const tperm_status_t ms = tperm::index_map(*p, map.data());
        if (ms != TPERM_OK) {
            std::printf("index map failed (%d) at iteration %d\n", (int)ms, it);
            return 1;
        }
        std::vector<char> seen((size_t)vol, 0);
        for (int64_t i = 0; i < vol; ++i) {
            if (map[(size_t)i] < 0 || map[(size_t)i] >= vol || seen[(size_t)map[(size_t)i]]) {
                std::printf("not a bijection at iteration %d\n", it);
                return 1;
            }
            seen[(size_t)map[(size_t)i]] = 1;
        }
        if (p->kclass == TPERM_KERNEL_ROWCOPY || p->kclass == TPERM_KERNEL_TILED || p->kclass == TPERM_KERNEL_PACKED) {
            // the analytical model walks sampled tiles with the kernel's arithmetic: its byte
            // count per tile can never exceed the tile, and the estimate must be finite
            tperm_model_t m;
            if (tperm::model_plan(*p, &m) != TPERM_OK || !(m.microseconds > 0.0) || !(m.microseconds < 1e12) ||
                m.useful_bytes_per_tile > (double)p->cand.tile_vol * (double)elem + 0.5) {
                std::printf("model failed at iteration %d\n", it);
                return 1;
            }
        }
        if (p->align_out) ++windows;
        if (p->align_out && p->vec2) ++pair_windows;
        delete p;
        ++made;
    }
    std::printf("ok: %d plans checked (%d with line-aligned windows, %d of them in pairs), %d option sets rejected\n", made, windows, pair_windows,
                rejected);
    return 0;
}
