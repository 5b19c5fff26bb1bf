// Launch interface between the C-ABI layer and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>

#include "plan.hpp"

namespace tperm {

// Workgroups of this plan's tile kernel that fit one compute unit (occupancy query).
hipError_t tile_blocks_per_cu(const Plan& plan, int* blocks);

// Cache policy of the kernel variant that launch_tile picks for the plan (see kernels.hip).
int tile_launch_policy(const Plan& plan, bool acc, bool sector_aligned_out);

// Whether a tile kernel is instantiated for the plan's combination of options.
bool tile_kernel_exists(const Plan& plan, bool acc);

// Enqueue the tile kernel (ROWCOPY / TILED / PACKED classes) with `grid` workgroups.
// accumulate: out = out + transposed in (elements are IEEE floats of the element size).
hipError_t launch_tile(const Plan& plan, const void* in, void* out, hipStream_t stream, int grid,
                       bool accumulate);

// Enqueue the naive one-thread-per-output-element gather.
hipError_t launch_naive(const Plan& plan, const void* in, void* out, hipStream_t stream,
                        bool accumulate);

// Enqueue out[i] = out[i] + in[i] over nbytes of `elem`-byte IEEE floats.
hipError_t launch_accumulate_copy(const void* in, void* out, size_t nbytes, int elem, int num_cu,
                                  hipStream_t stream);

// Enqueue a plain copy of nbytes; elem is the guaranteed pointer alignment (4 or 8).
hipError_t launch_copy(const void* in, void* out, size_t nbytes, int elem, int num_cu,
                       hipStream_t stream);

}  // namespace tperm
