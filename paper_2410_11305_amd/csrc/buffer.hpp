// Raw buffer loads for the gfx950 kernels.  A raw buffer load whose byte offset
// lies outside the buffer returns zero WITHOUT touching memory, so work that
// does not exist (a group past K, a token row past M, a weight tile past N) is
// expressed as an out-of-range offset instead of a branch around the load.
#pragma once
#include "common.hpp"

namespace qspec {

typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr uint32_t kOutOfRange = 0x80000000u;     // beyond any buffer this library accepts (< 2 GiB)

__device__ inline rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
__device__ inline uint4 buf_load16(rsrc_t r, uint32_t off) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
  return uint4{v.x, v.y, v.z, v.w};
}
// streaming variant (weights are read once: do not keep them in the caches)
__device__ inline uint4 buf_load16_stream(rsrc_t r, uint32_t off) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 2);
  return uint4{v.x, v.y, v.z, v.w};
}
__device__ inline uint2 buf_load8(rsrc_t r, uint32_t off) {
  typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
  const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0);
  return uint2{v.x, v.y};
}
__device__ inline uint16_t buf_load_u16(rsrc_t r, uint32_t off) {
  return (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, off, 0, 0);
}
// three consecutive floats (4-byte aligned; each component is range-checked on its own)
struct float3_t { float x, y, z; };
__device__ inline float3_t buf_load_f32x3(rsrc_t r, uint32_t off) {
  typedef unsigned int u32x3 __attribute__((ext_vector_type(3)));
  const u32x3 v = __builtin_amdgcn_raw_buffer_load_b96(r, off, 0, 0);
  const uint32_t a = v.x, b = v.y, c = v.z;      // (copies: bit_cast of a vector element lvalue reads element 0)
  return float3_t{__builtin_bit_cast(float, a), __builtin_bit_cast(float, b), __builtin_bit_cast(float, c)};
}
__device__ inline float buf_load_f32(rsrc_t r, uint32_t off) {
  return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0));
}

}  // namespace qspec
