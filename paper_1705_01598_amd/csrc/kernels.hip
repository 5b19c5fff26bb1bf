// Plain copy / accumulate and naive gather kernels, and the launch functions.  The tile
// kernel lives in tile_kernel.hpp and is instantiated in tile_inst_*.hip.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.hpp"
#include "tperm_desc.h"

namespace tperm {

const void* tile_kernel_u64_256(int nreg, bool use_lds, int nt, bool align, bool acc, bool loads_first, bool vec2);
const void* tile_kernel_u32_256(int nreg, bool use_lds, int nt, bool align, bool acc, bool loads_first, bool vec2);
const void* tile_kernel_u64_64(int nreg, bool use_lds, int nt, bool align, bool acc, bool loads_first, bool vec2);
const void* tile_kernel_u32_64(int nreg, bool use_lds, int nt, bool align, bool acc, bool loads_first, bool vec2);
const void* tile_kernel_big_u64(int nreg, int nt, bool align, bool acc, bool vec2);
const void* tile_kernel_big_u32(int nreg, int nt, bool align, bool acc, bool vec2);


// ---------------------------------------------------------------------------------------
// plain copy and naive gather
// ---------------------------------------------------------------------------------------

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Streaming copy, 16 bytes per lane, four independent nontemporal loads in flight per lane.
// Measured on MI355X, a copy is fastest with about 16 KiB in flight per compute unit: one
// workgroup of 256 threads per CU, each lane holding 4 x 16 bytes.
__global__ void __launch_bounds__(256)
copy16_kernel(const u32x4* __restrict__ in, u32x4* __restrict__ out, uint64_t n16) {
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 a = __builtin_nontemporal_load(in + i);
        const u32x4 b = __builtin_nontemporal_load(in + i + stride);
        const u32x4 c = __builtin_nontemporal_load(in + i + 2 * stride);
        const u32x4 e = __builtin_nontemporal_load(in + i + 3 * stride);
        __builtin_nontemporal_store(a, out + i);
        __builtin_nontemporal_store(b, out + i + stride);
        __builtin_nontemporal_store(c, out + i + 2 * stride);
        __builtin_nontemporal_store(e, out + i + 3 * stride);
    }
    for (; i < n16; i += stride) out[i] = in[i];
}

template <typename T>
__global__ void __launch_bounds__(256)
copy_elem_kernel(const T* __restrict__ in, T* __restrict__ out, uint64_t n) {
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    for (uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x; i < n; i += stride) out[i] = in[i];
}

// F is the arithmetic type when accumulating (float / double), else an unsigned integer.
template <typename F, bool ACC>
__global__ void __launch_bounds__(256)
naive_kernel(const NaiveDesc d, const F* __restrict__ in, F* __restrict__ out) {
    const uint64_t o = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (o < d.volume) {
        const F v = in[naive_input_offset(d, (uint32_t)o)];
        out[o] = ACC ? (F)(out[o] + v) : v;
    }
}

// out[i] = out[i] + in[i] (identity permutation in accumulate mode), four elements in
// flight per lane.
template <typename F>
__global__ void __launch_bounds__(256)
accumulate_kernel(const F* __restrict__ in, F* __restrict__ out, uint64_t n) {
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const F a0 = in[i], a1 = in[i + stride], a2 = in[i + 2 * stride], a3 = in[i + 3 * stride];
        const F b0 = out[i], b1 = out[i + stride], b2 = out[i + 2 * stride], b3 = out[i + 3 * stride];
        out[i] = b0 + a0;
        out[i + stride] = b1 + a1;
        out[i + 2 * stride] = b2 + a2;
        out[i + 3 * stride] = b3 + a3;
    }
    for (; i < n; i += stride) out[i] = out[i] + in[i];
}

// ---------------------------------------------------------------------------------------
// dispatch
// ---------------------------------------------------------------------------------------

// Cache policy (1 = cached, 2 = nontemporal loads and stores, 3 = nontemporal stores, 4 =
// nontemporal loads) of the kernel variant that runs the plan.  It is the plan's policy unless:
// the run accumulates (cached only); the output base pointer is not a multiple of 32 bytes
// (sector_aligned_out false: the planner's choice of nontemporal stores assumes whole sectors,
// from any other base the written pieces end inside sectors and cached stores are the right
// ones; line-aligned windows follow the pointer's phase by themselves); or the variant is not
// instantiated (nontemporal loads alone exist for stores-first 256-thread kernels; 64-thread
// kernels have cached and fully nontemporal forms).
int tile_launch_policy(const Plan& plan, bool acc, bool sector_aligned_out) {
    int pol = acc ? 1 : plan.cache_policy;
    if (!sector_aligned_out && !plan.align_out) pol = (pol == 2 || pol == 4) ? 4 : 1;
    if (pol == 4 && (plan.loads_first || plan.threads != 256)) pol = 1;
    if (pol == 3 && plan.threads != 256) pol = 2;
    return pol;
}

static const void* tile_kernel_for(const Plan& plan, bool acc, bool sector_aligned_out) {
    const int pol = tile_launch_policy(plan, acc, sector_aligned_out);
    const int nt = pol == 2 ? 2 : (pol == 3 ? 1 : (pol == 4 ? 3 : 0));  // template parameter NT
    const bool align = plan.align_out;
    if (plan.big) {
        if (!plan.use_lds || plan.loads_first || plan.threads != 256) return nullptr;
        return plan.elem == 8 ? tile_kernel_big_u64(plan.nreg, nt, align, acc, plan.vec2)
                              : tile_kernel_big_u32(plan.nreg, nt, align, acc, plan.vec2);
    }
    if (plan.elem == 8)
        return plan.threads == 64 ? tile_kernel_u64_64(plan.nreg, plan.use_lds, nt, align, acc, plan.loads_first, plan.vec2)
                                  : tile_kernel_u64_256(plan.nreg, plan.use_lds, nt, align, acc, plan.loads_first, plan.vec2);
    return plan.threads == 64 ? tile_kernel_u32_64(plan.nreg, plan.use_lds, nt, align, acc, plan.loads_first, plan.vec2)
                              : tile_kernel_u32_256(plan.nreg, plan.use_lds, nt, align, acc, plan.loads_first, plan.vec2);
}

bool tile_kernel_exists(const Plan& plan, bool acc) {
    return tile_kernel_for(plan, acc, true) != nullptr && tile_kernel_for(plan, acc, false) != nullptr;
}

hipError_t tile_blocks_per_cu(const Plan& plan, int* blocks) {
    const void* f = tile_kernel_for(plan, false, true);
    if (f == nullptr) return hipErrorInvalidValue;
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks, f, plan.threads,
                                                        (size_t)plan.lds_bytes * plan.tile.lds_buffers);
}

hipError_t launch_tile(const Plan& plan, const void* in, void* out, hipStream_t stream, int grid,
                       bool accumulate) {
    const void* f = tile_kernel_for(plan, accumulate, (reinterpret_cast<uintptr_t>(out) & 31u) == 0);
    if (f == nullptr || grid < 1) return hipErrorInvalidValue;
    TileDesc d = plan.tile;
    // large tensors: the range one buffer description covers from a tile's origin
    uint32_t nbytes = plan.big ? TPERM_BIG_RANGE : (uint32_t)((uint64_t)plan.c.volume * (uint64_t)plan.elem);
    void* args[] = {(void*)&d, (void*)&in, (void*)&out, (void*)&nbytes};
    return hipLaunchKernel(f, dim3((unsigned)grid), dim3((unsigned)plan.threads), args,
                           (size_t)plan.lds_bytes * plan.tile.lds_buffers, stream);
}

hipError_t launch_naive(const Plan& plan, const void* in, void* out, hipStream_t stream,
                        bool accumulate) {
    const uint64_t vol = (uint64_t)plan.c.volume;
    const unsigned grid = (unsigned)((vol + 255) / 256);
    if (accumulate) {
        if (plan.elem == 8)
            hipLaunchKernelGGL((naive_kernel<double, true>), dim3(grid), dim3(256), 0, stream,
                               plan.naive, (const double*)in, (double*)out);
        else
            hipLaunchKernelGGL((naive_kernel<float, true>), dim3(grid), dim3(256), 0, stream,
                               plan.naive, (const float*)in, (float*)out);
    } else if (plan.elem == 8) {
        hipLaunchKernelGGL((naive_kernel<uint64_t, false>), dim3(grid), dim3(256), 0, stream,
                           plan.naive, (const uint64_t*)in, (uint64_t*)out);
    } else {
        hipLaunchKernelGGL((naive_kernel<uint32_t, false>), dim3(grid), dim3(256), 0, stream,
                           plan.naive, (const uint32_t*)in, (uint32_t*)out);
    }
    return hipGetLastError();
}

hipError_t launch_accumulate_copy(const void* in, void* out, size_t nbytes, int elem, int num_cu,
                                  hipStream_t stream) {
    if (nbytes == 0) return hipSuccess;
    const uint64_t n = nbytes / (size_t)elem;
    const uint64_t cap = (uint64_t)(num_cu > 0 ? num_cu : 256) * 4u, g = (n + 255) / 256;
    const unsigned grid = (unsigned)(g < cap ? (g ? g : 1) : cap);
    if (elem == 8)
        hipLaunchKernelGGL(accumulate_kernel<double>, dim3(grid), dim3(256), 0, stream,
                           (const double*)in, (double*)out, n);
    else
        hipLaunchKernelGGL(accumulate_kernel<float>, dim3(grid), dim3(256), 0, stream,
                           (const float*)in, (float*)out, n);
    return hipGetLastError();
}

hipError_t launch_copy(const void* in, void* out, size_t nbytes, int elem, int num_cu,
                       hipStream_t stream) {
    if (nbytes == 0) return hipSuccess;
    const unsigned max_grid = (unsigned)(num_cu > 0 ? num_cu : 256);
    auto grid_for = [&](uint64_t n, unsigned per_cu = 1) {
        const uint64_t g = (n + 255) / 256, cap = (uint64_t)max_grid * per_cu;
        return (unsigned)(g < cap ? (g ? g : 1) : cap);
    };
    const bool aligned16 = (((uintptr_t)in | (uintptr_t)out) & 15u) == 0;
    if (aligned16 && nbytes >= 16) {
        const uint64_t n16 = nbytes / 16;
        hipLaunchKernelGGL(copy16_kernel, dim3(grid_for(n16)), dim3(256), 0, stream,
                           (const u32x4*)in, (u32x4*)out, n16);
        const size_t done = (size_t)n16 * 16, tail = nbytes - done;
        if (tail) {
            hipLaunchKernelGGL(copy_elem_kernel<uint32_t>, dim3(1), dim3(256), 0, stream,
                               (const uint32_t*)((const char*)in + done),
                               (uint32_t*)((char*)out + done), (uint64_t)(tail / 4));
        }
    } else if (elem == 8) {
        const uint64_t n = nbytes / 8;
        hipLaunchKernelGGL(copy_elem_kernel<uint64_t>, dim3(grid_for(n, 8)), dim3(256), 0, stream,
                           (const uint64_t*)in, (uint64_t*)out, n);
    } else {
        const uint64_t n = nbytes / 4;
        hipLaunchKernelGGL(copy_elem_kernel<uint32_t>, dim3(grid_for(n, 16)), dim3(256), 0, stream,
                           (const uint32_t*)in, (uint32_t*)out, n);
    }
    return hipGetLastError();
}

}  // namespace tperm
