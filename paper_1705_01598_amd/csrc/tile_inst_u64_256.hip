// Instantiations of the tile kernel for uint64_t elements, 256-thread workgroups.
#include "tile_kernel.hpp"

namespace tperm {

const void* tile_kernel_u64_256(int nreg, bool use_lds, int nt, bool align, bool acc, bool loads_first, bool vec2) {
    return tile_kernel_select<uint64_t, 256>(nreg, use_lds, nt, align, acc, loads_first, vec2);
}

}  // namespace tperm
