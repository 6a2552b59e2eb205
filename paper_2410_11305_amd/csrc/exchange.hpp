// Exchange of partial sums between the workgroups of one launch (K-slices of
// one output block computed by different workgroups).
#pragma once
#include "common.hpp"

namespace qspec {

// Partial sums that several workgroups exchange inside one launch go past the
// per-XCD L2 caches (which are not coherent with each other): device-scope
// relaxed atomic accesses compile to write-through stores and cache-bypassing
// loads, so no dirty line of theirs is ever left in an L2 (see last_arrival).
// (A device-scope fence per WAVE was measured and doubled the kernel time.)
__device__ __forceinline__ void store_shared_f2(float* p, float a, float b) {
  const uint64_t v = (uint64_t)__builtin_bit_cast(uint32_t, a) | ((uint64_t)__builtin_bit_cast(uint32_t, b) << 32);
  __hip_atomic_store(reinterpret_cast<uint64_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 load_shared_f2(const float* p) {
  const uint64_t v = __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return float2{__builtin_bit_cast(float, (uint32_t)v), __builtin_bit_cast(float, (uint32_t)(v >> 32))};
}
// Take a ticket of output block blk once every partial sum of this workgroup has been
// performed at device scope; true for the workgroup that arrives last of S (it also puts
// the counter back to zero for the next launch).
//
// Ordering.  Reader side: the last arrival executes an ACQUIRE fence at agent scope after
// it has seen S-1 (one cache invalidate per output block), the workgroup barrier hands
// that to its other waves, and the slices are then read with relaxed agent-scope atomic
// loads.  Writer side: a release at agent scope is, in the compiler's code sequence for
// this target, "write back the dirty lines of this L2, wait until every earlier store has
// been acknowledged (vmcnt 0), then perform the atomic".  The partial sums are agent-scope
// atomic stores, i.e. write-through: they leave no dirty line, so the write-back has
// nothing of this exchange to do, and what remains of the sequence is issued by hand:
// every wave waits for vmcnt 0, the workgroup barrier collects the waves, thread 0
// increments the counter.  The write-back itself is not free even so (it still walks the
// L2 for the fp16 outputs other workgroups have stored): with the increment as a full
// RELEASE the K-sliced launches measured 5-24 % longer (28672 x 8192 at 128 draft tokens
// 66.6 -> 81.4 us, 13824 x 5120 at 384: 58.0 -> 69.6 us), with the acquire fence alone
// they are unchanged.  Define QSPEC_EXCHANGE_FULL_RELEASE to build the release form.
__device__ __forceinline__ bool last_arrival(unsigned* tickets, int S, unsigned blk, unsigned* ticket_lds) {
#ifdef QSPEC_EXCHANGE_FULL_RELEASE
  constexpr int kOrder = __ATOMIC_RELEASE;
#else
  constexpr int kOrder = __ATOMIC_RELAXED;
  __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): this wave's write-through stores have been acknowledged
#endif
  __syncthreads();                      // ... and those of the whole workgroup
  if (threadIdx.x == 0) {
    const unsigned old = __hip_atomic_fetch_add(&tickets[blk], 1u, kOrder, __HIP_MEMORY_SCOPE_AGENT);
    if (old == (unsigned)S - 1) {
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      __hip_atomic_store(&tickets[blk], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    *ticket_lds = old;
  }
  __syncthreads();
  return *ticket_lds == (unsigned)S - 1;
}

}  // namespace qspec
