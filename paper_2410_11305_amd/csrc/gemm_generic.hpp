// Generic (any M) kernels for both modes of the shared-weight linear layer.
// One workgroup owns one 16-row weight tile column (16 outputs n) and up to
// TM*16 tokens; its wavefronts split the K groups between them (split-K inside
// the workgroup) and combine their fp32 sums through LDS.  Operands come
// straight from global memory in MFMA register layout:
//   A operand = weights (row i = n % 16, k-block = lane / 16),
//   B operand = activations (column j = m % 16, same k-block),
//   D[i][j]: lane holds rows i = 4*(lane/16) + r (r = 0..3), column lane % 16.
#pragma once
#include "common.hpp"

namespace qspec {

struct GemmArgs {
  const uint4* codes;        // blob, code tiles
  const uint16_t* scalesT;   // blob, fp16 scales [G][N]
  const void* act;           // W4A4: qa bytes [M][K/2];  W4A16: x fp16 [M][K]
  const float* sa;           // W4A4 only: [M][G]
  uint16_t* y;               // fp16 [M][N]
  int32_t* partials;         // debug entry only: [M][n_count][G]
  int M, N, K, G;
  int n0, n_count;           // debug entry: column window
};

template <int TM, int WAVES>
__device__ inline void reduce_and_store(float (&facc)[TM][4], const GemmArgs& p, int T, int m0) {
  __shared__ float red[WAVES][TM * 4][kWave];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r16 = lane & 15, kb = lane >> 4;
  if (WAVES > 1) {
#pragma unroll
    for (int t = 0; t < TM; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[wave][t * 4 + r][lane] = facc[t][r];
    __syncthreads();
  }
  for (int t = wave; t < TM; t += WAVES) {
    const int m = m0 + 16 * t + r16;
    float o[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (WAVES > 1) {
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) s += red[w][t * 4 + r][lane];
        o[r] = s;
      } else {
        o[r] = facc[t][r];
      }
    }
    if (m < p.M) {
      uint2 out;
      out.x = (uint32_t)float_to_half_bits(o[0]) | ((uint32_t)float_to_half_bits(o[1]) << 16);
      out.y = (uint32_t)float_to_half_bits(o[2]) | ((uint32_t)float_to_half_bits(o[3]) << 16);
      *reinterpret_cast<uint2*>(p.y + (size_t)m * p.N + T * 16 + 4 * kb) = out;
    }
  }
}

// ---------------------------------------------------------------- W4A4
// P[m,n,j] on int8 MFMA (exact int32), then y += float(P) * sa[m,j] * sw[n,j].
template <int TM, int WAVES, bool PARTIALS>
__global__ __launch_bounds__(WAVES * 64) void gemm_w4a4_generic(GemmArgs p) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r16 = lane & 15, kb = lane >> 4;
  const int T = blockIdx.x + (PARTIALS ? p.n0 / 16 : 0);
  const int m0 = blockIdx.y * (TM * 16);
  const int G = p.G;
  const int gchunk = (G + WAVES - 1) / WAVES;
  const int g_begin = wave * gchunk;
  const int g_end = min(G, g_begin + gchunk);
  const uint8_t* qa = static_cast<const uint8_t*>(p.act);

  float facc[TM][4];
#pragma unroll
  for (int t = 0; t < TM; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) facc[t][r] = 0.0f;

  for (int g = g_begin; g < g_end; ++g) {
    const uint4 wq = p.codes[((size_t)T * G + g) * 64 + lane];
    const I8Pair a = unpack_i8(wq);
    float sw[4];
    if (!PARTIALS) {
      const uint2 sraw = *reinterpret_cast<const uint2*>(p.scalesT + (size_t)g * p.N + T * 16 + 4 * kb);
      // both operands carry a factor 16: fold 2^-8 into the weight scale (exact)
      sw[0] = half_bits_to_float((uint16_t)(sraw.x & 0xFFFF)) * 0.00390625f;
      sw[1] = half_bits_to_float((uint16_t)(sraw.x >> 16)) * 0.00390625f;
      sw[2] = half_bits_to_float((uint16_t)(sraw.y & 0xFFFF)) * 0.00390625f;
      sw[3] = half_bits_to_float((uint16_t)(sraw.y >> 16)) * 0.00390625f;
    }
#pragma unroll
    for (int t = 0; t < TM; ++t) {
      const int m = m0 + 16 * t + r16;
      const bool valid = m < p.M;
      const int mc = valid ? m : p.M - 1;
      uint4 aq = *reinterpret_cast<const uint4*>(qa + (size_t)mc * (p.K / 2) + 64 * g + 16 * kb);
      if (!valid) aq = uint4{0u, 0u, 0u, 0u};
      const I8Pair b = unpack_i8(aq);
      v4i acc = {0, 0, 0, 0};
      acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a.lo, b.lo, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a.hi, b.hi, acc, 0, 0, 0);
      if (PARTIALS) {
        if (valid) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int nl = T * 16 + 4 * kb + r - p.n0;
            p.partials[((size_t)m * p.n_count + nl) * G + g] = acc[r] >> 8;   // exact: multiple of 256
          }
        }
      } else {
        const float s = valid ? p.sa[(size_t)mc * G + g] : 0.0f;
#pragma unroll
        for (int r = 0; r < 4; ++r) facc[t][r] += (float)acc[r] * (s * sw[r]);
      }
    }
  }
  if (!PARTIALS) reduce_and_store<TM, WAVES>(facc, p, T, m0);
}

// ---------------------------------------------------------------- W4A16
// Codes become exact fp16 integers in registers; x * code is accumulated on
// fp16 MFMA in fp32 over one group, then scaled by sw[n,j] in fp32.
template <int TM, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void gemm_w4a16_generic(GemmArgs p) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r16 = lane & 15, kb = lane >> 4;
  const int T = blockIdx.x;
  const int m0 = blockIdx.y * (TM * 16);
  const int G = p.G;
  const int gchunk = (G + WAVES - 1) / WAVES;
  const int g_begin = wave * gchunk;
  const int g_end = min(G, g_begin + gchunk);
  const uint16_t* x = static_cast<const uint16_t*>(p.act);

  float facc[TM][4];
#pragma unroll
  for (int t = 0; t < TM; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) facc[t][r] = 0.0f;

  for (int g = g_begin; g < g_end; ++g) {
    const uint4 wq = p.codes[((size_t)T * G + g) * 64 + lane];
    v8h wa[4];
    wa[0] = dequant_word(wq.x);
    wa[1] = dequant_word(wq.y);
    wa[2] = dequant_word(wq.z);
    wa[3] = dequant_word(wq.w);
    const uint2 sraw = *reinterpret_cast<const uint2*>(p.scalesT + (size_t)g * p.N + T * 16 + 4 * kb);
    float sw[4];
    sw[0] = half_bits_to_float((uint16_t)(sraw.x & 0xFFFF));
    sw[1] = half_bits_to_float((uint16_t)(sraw.x >> 16));
    sw[2] = half_bits_to_float((uint16_t)(sraw.y & 0xFFFF));
    sw[3] = half_bits_to_float((uint16_t)(sraw.y >> 16));
#pragma unroll
    for (int t = 0; t < TM; ++t) {
      const int m = m0 + 16 * t + r16;
      const bool valid = m < p.M;
      const int mc = valid ? m : p.M - 1;
      const uint16_t* xr = x + (size_t)mc * p.K + g * kGroup + kb * 8;
      v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint4 xq = *reinterpret_cast<const uint4*>(xr + 32 * i);
        if (!valid) xq = uint4{0u, 0u, 0u, 0u};
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa[i], __builtin_bit_cast(v8h, xq), acc, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) facc[t][r] += acc[r] * sw[r];
    }
  }
  reduce_and_store<TM, WAVES>(facc, p, T, m0);
}

}  // namespace qspec
