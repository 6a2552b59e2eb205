// Activation quantiser of the draft mode (paper Sec. 1: W4A4 quantises the
// activations to 4 bit as well; Sec. 4.1: groups of 128).  Per token and
// group, all in binary32: a = max|x|, s = a / 7, q = clamp(rne(x / s), -8, 7),
// both divisions IEEE-exact (no reciprocal shortcut), ties to even.
#pragma once
#include "common.hpp"

namespace qspec {

// Data-parallel-primitive moves inside a row of 16 lanes: lane i reads its partner in
// the quad (0xB1: i^1, 0x4E: i^2), in its half row (0x141: 7 - i) or in the row
// (0x140: 15 - i).  Four of them in this order fold a row of 16; they run in the
// vector ALU, where a cross-lane shuffle takes a round trip through the LDS crossbar.
// Every lane of the row must be active.
template <int CTRL>
__device__ inline int dpp_i32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}

__device__ inline float row16_max(float a) {
  a = fmaxf(a, __builtin_bit_cast(float, dpp_i32<0xB1>(__builtin_bit_cast(int, a))));
  a = fmaxf(a, __builtin_bit_cast(float, dpp_i32<0x4E>(__builtin_bit_cast(int, a))));
  a = fmaxf(a, __builtin_bit_cast(float, dpp_i32<0x141>(__builtin_bit_cast(int, a))));
  a = fmaxf(a, __builtin_bit_cast(float, dpp_i32<0x140>(__builtin_bit_cast(int, a))));
  return a;
}

// One thread owns 8 consecutive activations (one 16-byte load, one 32-bit
// code word); 16 adjacent lanes (one row) own one group, so the absmax is a
// 4-step fold inside the row and no LDS is needed.
//
// quantise_word: the arithmetic alone.  v = this thread's 8 activations (fp16 values
// widened to binary32); returns its code word (8 nibbles in the device nibble order)
// and the group's scale.  Every lane of the wavefront must call it (the shuffles).
__device__ inline uint32_t quantise_word(const float (&v)[8], float* s_out) {
  float a = 0.0f;
#pragma unroll
  for (int e = 0; e < 8; ++e) a = fmaxf(a, fabsf(v[e]));
  a = row16_max(a);
  const float s = a / 7.0f;
  uint32_t w = 0;
  if (a > 0.0f) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float t = rintf(v[e] / s);                 // v_rndne: ties to even
      t = fminf(fmaxf(t, -8.0f), 7.0f);
      w |= ((uint32_t)(int)t & 0xFu) << (4 * nibble_pos(e));
    }
  }
  *s_out = s;
  return w;
}

// quantise_unit: quantise and store in the packed format.  idx = index of the thread's code
// word in the [M][K/8] word array; lanes that are not `live` pass zeros and store nothing.
// The number of words per row is a multiple of 16, so a 16-lane group is entirely live or not.
__device__ inline void quantise_unit(const float (&v)[8], bool live, size_t idx,
                                     uint32_t* __restrict__ qa_words, float* __restrict__ sa) {
  float s;
  const uint32_t w = quantise_word(v, &s);
  if (live) {
    // word position inside the group: k-word kw = 4i + kb is stored at 4kb + i, so
    // that the 16 bytes a GEMM lane (k-block kb) needs are contiguous
    const size_t kw = idx & 15;
    qa_words[(idx & ~(size_t)15) + ((kw & 3) << 2) + (kw >> 2)] = w;
    if ((threadIdx.x & 15) == 0) sa[idx >> 4] = s;
  }
}

// The same codes in the widened format the tiled draft kernel can take straight into LDS:
// per token row and group 128 bytes, byte b of the packed group's 64 giving two of them,
// 16 * (code in its low nibble) at b and 16 * (code in its high nibble) at 64 + b (a nibble
// moved to the high half of a byte is 16 * code as int8).  qa8_words: [M][K/4] words.
__device__ inline void quantise_unit_wide(const float (&v)[8], bool live, size_t idx,
                                          uint32_t* __restrict__ qa8_words, float* __restrict__ sa) {
  float s;
  const uint32_t w = quantise_word(v, &s);
  if (live) {
    const size_t kw = idx & 15;
    const size_t pos = ((kw & 3) << 2) + (kw >> 2);            // word position in the packed group
    const size_t gbase = (idx & ~(size_t)15) * 2;              // a widened group has 32 words
    qa8_words[gbase + pos] = (w << 4) & 0xF0F0F0F0u;
    qa8_words[gbase + 16 + pos] = w & 0xF0F0F0F0u;
    if ((threadIdx.x & 15) == 0) sa[idx >> 4] = s;
  }
}

__global__ __launch_bounds__(256) void quant_act_kernel(const uint4* __restrict__ x,
                                                        uint32_t* __restrict__ qa_words,
                                                        float* __restrict__ sa,
                                                        size_t n_words) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool live = idx < n_words;
  uint4 raw = {0u, 0u, 0u, 0u};
  if (live) raw = x[idx];
  float v[8];
  {
    const v8h h = __builtin_bit_cast(v8h, raw);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (float)h[e];
  }
  quantise_unit(v, live, idx, qa_words, sa);
}

__global__ __launch_bounds__(256) void quant_act_wide_kernel(const uint4* __restrict__ x,
                                                             uint32_t* __restrict__ qa8_words,
                                                             float* __restrict__ sa,
                                                             size_t n_words) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool live = idx < n_words;
  uint4 raw = {0u, 0u, 0u, 0u};
  if (live) raw = x[idx];
  float v[8];
  {
    const v8h h = __builtin_bit_cast(v8h, raw);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (float)h[e];
  }
  quantise_unit_wide(v, live, idx, qa8_words, sa);
}

}  // namespace qspec
