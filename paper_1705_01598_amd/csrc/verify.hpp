// On-device multiset check (see verify.hip): interface towards the C-ABI layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace tperm {

constexpr uint64_t kVerifyChunk = 16384;       // elements digested by one workgroup
constexpr size_t kVerifyPartialBytes = 32;     // one partial result

// The entry point that allocates nothing keeps its partial results in a file-scope device
// array sized for tensors of up to kVerifyStaticMaxElems elements (512 KiB per GPU).
constexpr uint64_t kVerifyStaticMaxElems = (uint64_t)1 << 27;
constexpr size_t kVerifyStaticBytes = 2 * (size_t)(kVerifyStaticMaxElems / kVerifyChunk) * kVerifyPartialBytes;

// Device address of that array on the current device (resolved on the first call per device,
// then remembered).  The memory keeps whatever the last call left in it.
hipError_t verify_static_scratch(void** ptr);

// Scratch bytes the check of two tensors of n_elems elements needs: one partial result per
// chunk and tensor.
size_t verify_scratch_bytes(uint64_t n_elems);

// Enqueue the check of a against b (n_elems words of `elem` = 4 or 8 bytes each; device
// pointers aligned to the word size).  scratch_dev: device memory of at least
// verify_scratch_bytes(n_elems) bytes, 8-byte aligned; verdict_dev: device pointer to one
// 64-bit word, written last (0 = same multiset of words).
hipError_t launch_multiset_compare(const void* a, const void* b, uint64_t n_elems, int elem,
                                   void* scratch_dev, uint64_t* verdict_dev, hipStream_t stream);

}  // namespace tperm
