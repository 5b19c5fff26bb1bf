// Instantiations of the tile kernel for tensors of 4 GiB and more (BIG), 4-byte elements:
// LDS-staged tiles of 256 threads, stores first, the four cache policies; single elements or
// pairs, plain or in line-aligned windows; the accumulating forms (single elements, cached).
#include "tile_kernel.hpp"

namespace tperm {

const void* tile_kernel_big_u32(int nreg, int nt, bool align, bool acc, bool vec2) {
    typedef uint32_t T;
    if (acc) {
        if (nt != 0 || vec2) return nullptr;
        return align ? tile_kernel_ptr<T, 256, true, 0, true, true, false, false, true>(nreg)
                     : tile_kernel_ptr<T, 256, true, 0, false, true, false, false, true>(nreg);
    }
    if (vec2 && align) {
        // pairs of 4-byte elements inside the windows
        switch (nt) {
            case 0: return tile_kernel_ptr<T, 256, true, 0, true, false, false, true, true>(nreg);
            case 1: return tile_kernel_ptr<T, 256, true, 1, true, false, false, true, true>(nreg);
            case 2: return tile_kernel_ptr<T, 256, true, 2, true, false, false, true, true>(nreg);
            case 3: return tile_kernel_ptr<T, 256, true, 3, true, false, false, true, true>(nreg);
            default: return nullptr;
        }
    }
#define TPERM_BIG_POLICIES(ALIGN_, VEC2_)                                                              \
    switch (nt) {                                                                                      \
        case 0: return tile_kernel_ptr<T, 256, true, 0, ALIGN_, false, false, VEC2_, true>(nreg);      \
        case 1: return tile_kernel_ptr<T, 256, true, 1, ALIGN_, false, false, VEC2_, true>(nreg);      \
        case 2: return tile_kernel_ptr<T, 256, true, 2, ALIGN_, false, false, VEC2_, true>(nreg);      \
        case 3: return tile_kernel_ptr<T, 256, true, 3, ALIGN_, false, false, VEC2_, true>(nreg);      \
        default: return nullptr;                                                                       \
    }
    if (vec2) { TPERM_BIG_POLICIES(false, true) }
    if (align) { TPERM_BIG_POLICIES(true, false) }
    TPERM_BIG_POLICIES(false, false)
#undef TPERM_BIG_POLICIES
}

}  // namespace tperm
