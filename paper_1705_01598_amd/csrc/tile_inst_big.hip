// Instantiations of the tile kernel for tensors of 4 GiB and more (BIG): plain LDS-staged tiles,
// 256-thread workgroups, both element sizes, the four cache policies, and the accumulating
// form with cached accesses.
#include "tile_kernel.hpp"

namespace tperm {

template <typename T>
static const void* tile_kernel_big_select(int nreg, int nt, bool acc) {
    if (acc) return nt == 0 ? tile_kernel_ptr<T, 256, true, 0, false, true, false, false, true>(nreg) : nullptr;
    switch (nt) {
        case 0: return tile_kernel_ptr<T, 256, true, 0, false, false, false, false, true>(nreg);
        case 1: return tile_kernel_ptr<T, 256, true, 1, false, false, false, false, true>(nreg);
        case 2: return tile_kernel_ptr<T, 256, true, 2, false, false, false, false, true>(nreg);
        case 3: return tile_kernel_ptr<T, 256, true, 3, false, false, false, false, true>(nreg);
        default: return nullptr;
    }
}

const void* tile_kernel_big(int elem, int nreg, int nt, bool acc) {
    return elem == 8 ? tile_kernel_big_select<uint64_t>(nreg, nt, acc) : tile_kernel_big_select<uint32_t>(nreg, nt, acc);
}

}  // namespace tperm
