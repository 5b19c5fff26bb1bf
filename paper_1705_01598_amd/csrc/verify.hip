// On-device multiset check behind tperm_execute_verified: after a transpose, the output must
// hold exactly the elements of the input, each as often (a transpose moves bits and creates or
// destroys none of them).  Three order-independent digests of the element words -- their sum
// and their exclusive-or, and the sum of a scrambled image of every word, all modulo 2^64 --
// are computed for both tensors and compared on the device.
//
// Work layout: the tensor is cut into chunks of kVerifyChunk elements; one workgroup digests
// one chunk and writes one partial result (32 bytes) into a scratch buffer, slot = chunk
// number; a last, single workgroup adds up the partials of both tensors, compares the two
// totals and writes the verdict.  Every slot that is read has been written by the same call,
// so the scratch needs no clearing.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "verify.hpp"

// Scratch of the entry point that allocates nothing: one copy of this array lives on every GPU
// the library runs on, from the moment its code is loaded there until the process ends.  Host
// code never passes the array's name to a kernel (on the host that name is only a handle for
// the symbol): verify_static_scratch() asks the runtime for the array's device address, once per
// device, and every kernel argument is built from that address.
static __device__ __align__(256) unsigned char scratch[tperm::kVerifyStaticBytes];

namespace tperm {

struct MultisetPartial {
    uint64_t sum, exor, mix, unused;
};
static_assert(sizeof(MultisetPartial) == kVerifyPartialBytes, "partial result size");

// 64-bit finaliser (multiply, fold, multiply): a word and its image share no linear relation,
// so two corrupted elements whose plain sums and exclusive-ors happen to cancel still show.
__device__ __forceinline__ uint64_t scramble(uint64_t e) {
    uint64_t h = e * 0x9E3779B97F4A7C15ull;
    h ^= h >> 29;
    return h * 0xBF58476D1CE4E5B9ull;
}

// Adds up three 64-bit values over the 256 threads of a workgroup; the totals end up in
// thread 0.  red has 3 * 256 entries.
__device__ __forceinline__ void block_reduce3(uint64_t* red, uint64_t* s, uint64_t* x, uint64_t* m) {
    const uint32_t tid = threadIdx.x;
    red[tid] = *s;
    red[256 + tid] = *x;
    red[512 + tid] = *m;
    __syncthreads();
    for (uint32_t half = 128; half > 0; half >>= 1) {
        if (tid < half) {
            red[tid] += red[tid + half];
            red[256 + tid] ^= red[256 + tid + half];
            red[512 + tid] += red[512 + tid + half];
        }
        __syncthreads();
    }
    *s = red[0];
    *x = red[256];
    *m = red[512];
}

// One workgroup per chunk of kVerifyChunk elements; T is the element word.
template <typename T>
__global__ void __launch_bounds__(256)
multiset_partial_kernel(const T* __restrict__ data, uint64_t n, MultisetPartial* __restrict__ partial) {
    __shared__ uint64_t red[3 * 256];
    const uint64_t begin = (uint64_t)blockIdx.x * kVerifyChunk;
    const uint64_t end = begin + kVerifyChunk < n ? begin + kVerifyChunk : n;
    uint64_t s = 0, x = 0, m = 0;
    for (uint64_t i = begin + threadIdx.x; i < end; i += 256u) {
        const uint64_t e = (uint64_t)data[i];
        s += e;
        x ^= e;
        m += scramble(e);
    }
    block_reduce3(red, &s, &x, &m);
    if (threadIdx.x == 0) {
        MultisetPartial p;
        p.sum = s;
        p.exor = x;
        p.mix = m;
        p.unused = 0;
        partial[blockIdx.x] = p;
    }
}

// Single workgroup: totals of both tensors' partials, compared.  *verdict = 0 when all three
// digests agree, else a bit mask of the ones that differ (1 sum, 2 exclusive-or, 4 scrambled sum).
__global__ void __launch_bounds__(256)
multiset_verdict_kernel(const MultisetPartial* __restrict__ pa, const MultisetPartial* __restrict__ pb,
                        uint32_t chunks, uint64_t* __restrict__ verdict) {
    __shared__ uint64_t red[3 * 256];
    uint64_t tot[2][3];
    for (int side = 0; side < 2; ++side) {
        const MultisetPartial* p = side == 0 ? pa : pb;
        uint64_t s = 0, x = 0, m = 0;
        for (uint32_t c = threadIdx.x; c < chunks; c += 256u) {
            s += p[c].sum;
            x ^= p[c].exor;
            m += p[c].mix;
        }
        block_reduce3(red, &s, &x, &m);
        tot[side][0] = s;
        tot[side][1] = x;
        tot[side][2] = m;
        __syncthreads();  // red is reused by the second side
    }
    if (threadIdx.x == 0)
        *verdict = (tot[0][0] != tot[1][0] ? 1u : 0u) | (tot[0][1] != tot[1][1] ? 2u : 0u) |
                   (tot[0][2] != tot[1][2] ? 4u : 0u);
}

hipError_t verify_static_scratch(void** ptr) {
    constexpr int kMaxDevices = 64;
    static std::mutex mutex;
    static void* address[kMaxDevices] = {};  // per device ordinal; nullptr = not asked yet
    *ptr = nullptr;
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mutex);
    if (address[dev] == nullptr) {
        void* p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // the current device's copy
        if (err != hipSuccess) return err;
        if (p == nullptr) return hipErrorInvalidSymbol;
        address[dev] = p;
    }
    *ptr = address[dev];
    return hipSuccess;
}

size_t verify_scratch_bytes(uint64_t n_elems) {
    const uint64_t chunks = (n_elems + kVerifyChunk - 1) / kVerifyChunk;
    return (size_t)(2 * chunks * kVerifyPartialBytes);
}

hipError_t launch_multiset_compare(const void* a, const void* b, uint64_t n_elems, int elem,
                                   void* scratch_dev, uint64_t* verdict_dev, hipStream_t stream) {
    const uint64_t chunks64 = (n_elems + kVerifyChunk - 1) / kVerifyChunk;
    if (chunks64 == 0 || chunks64 > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const uint32_t chunks = (uint32_t)chunks64;
    MultisetPartial* pa = static_cast<MultisetPartial*>(scratch_dev);
    MultisetPartial* pb = pa + chunks;
    if (elem == 8) {
        hipLaunchKernelGGL(multiset_partial_kernel<uint64_t>, dim3(chunks), dim3(256), 0, stream,
                           static_cast<const uint64_t*>(a), n_elems, pa);
        hipLaunchKernelGGL(multiset_partial_kernel<uint64_t>, dim3(chunks), dim3(256), 0, stream,
                           static_cast<const uint64_t*>(b), n_elems, pb);
    } else {
        hipLaunchKernelGGL(multiset_partial_kernel<uint32_t>, dim3(chunks), dim3(256), 0, stream,
                           static_cast<const uint32_t*>(a), n_elems, pa);
        hipLaunchKernelGGL(multiset_partial_kernel<uint32_t>, dim3(chunks), dim3(256), 0, stream,
                           static_cast<const uint32_t*>(b), n_elems, pb);
    }
    hipLaunchKernelGGL(multiset_verdict_kernel, dim3(1), dim3(256), 0, stream, pa, pb, chunks, verdict_dev);
    return hipGetLastError();
}

}  // namespace tperm
