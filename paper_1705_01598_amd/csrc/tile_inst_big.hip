// Instantiations of the tile kernel for tensors of 4 GiB and more (BIG): LDS-staged tiles,
// 256-thread workgroups, both element sizes, the four cache policies, single elements or
// pairs, and the accumulating form (single elements, cached accesses).
#include "tile_kernel.hpp"

namespace tperm {

template <typename T>
static const void* tile_kernel_big_select(int nreg, int nt, bool acc, bool vec2) {
    if (acc) return (nt == 0 && !vec2) ? tile_kernel_ptr<T, 256, true, 0, false, true, false, false, true>(nreg) : nullptr;
    if (vec2) {
        switch (nt) {
            case 0: return tile_kernel_ptr<T, 256, true, 0, false, false, false, true, true>(nreg);
            case 1: return tile_kernel_ptr<T, 256, true, 1, false, false, false, true, true>(nreg);
            case 2: return tile_kernel_ptr<T, 256, true, 2, false, false, false, true, true>(nreg);
            case 3: return tile_kernel_ptr<T, 256, true, 3, false, false, false, true, true>(nreg);
            default: return nullptr;
        }
    }
    switch (nt) {
        case 0: return tile_kernel_ptr<T, 256, true, 0, false, false, false, false, true>(nreg);
        case 1: return tile_kernel_ptr<T, 256, true, 1, false, false, false, false, true>(nreg);
        case 2: return tile_kernel_ptr<T, 256, true, 2, false, false, false, false, true>(nreg);
        case 3: return tile_kernel_ptr<T, 256, true, 3, false, false, false, false, true>(nreg);
        default: return nullptr;
    }
}

const void* tile_kernel_big(int elem, int nreg, int nt, bool acc, bool vec2) {
    return elem == 8 ? tile_kernel_big_select<uint64_t>(nreg, nt, acc, vec2)
                     : tile_kernel_big_select<uint32_t>(nreg, nt, acc, vec2);
}

}  // namespace tperm
