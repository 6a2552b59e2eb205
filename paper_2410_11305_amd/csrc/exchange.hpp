// Exchange of partial sums between the workgroups of one launch (K-slices of
// one output block computed by different workgroups).
#pragma once
#include "common.hpp"

namespace qspec {

// Partial sums that several workgroups exchange inside one launch go past the
// per-XCD L2 caches (which are not coherent with each other): device-scope
// relaxed atomic accesses compile to write-through stores and cache-bypassing
// loads.  That is much cheaper than device-scope fences, each of which writes
// back and invalidates a whole L2.
__device__ __forceinline__ void store_shared_f2(float* p, float a, float b) {
  const uint64_t v = (uint64_t)__builtin_bit_cast(uint32_t, a) | ((uint64_t)__builtin_bit_cast(uint32_t, b) << 32);
  __hip_atomic_store(reinterpret_cast<uint64_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 load_shared_f2(const float* p) {
  const uint64_t v = __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return float2{__builtin_bit_cast(float, (uint32_t)v), __builtin_bit_cast(float, (uint32_t)(v >> 32))};
}
// Take a ticket of output block blk once every store of this workgroup has been
// performed; true for the workgroup that arrives last of S (it also puts the
// counter back to zero for the next launch).
__device__ __forceinline__ bool last_arrival(unsigned* tickets, int S, unsigned blk, unsigned* ticket_lds) {
  __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): this wave's write-through stores have been performed
  __syncthreads();                      // ... and those of the whole workgroup
  if (threadIdx.x == 0) {
    const unsigned old = atomicAdd(&tickets[blk], 1u);
    if (old == (unsigned)S - 1) atomicExch(&tickets[blk], 0u);
    *ticket_lds = old;
  }
  __syncthreads();
  return *ticket_lds == (unsigned)S - 1;
}

}  // namespace qspec
