// On-device multiset check (see verify.hip): interface towards the C-ABI layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace tperm {

constexpr uint64_t kVerifyChunk = 16384;       // elements digested by one workgroup
constexpr size_t kVerifyPartialBytes = 32;     // one partial result

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
