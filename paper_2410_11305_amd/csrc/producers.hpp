// The two producers of draft-mode activations in a Llama-shaped decoder block,
// each fused with the activation quantiser that follows it in the draft pass
// (paper Sec. 3.1, draft phase; Sec. 1: activations are quantised to 4 bit on
// the fly): RMSNorm (input of the q/k/v and gate/up projections) and
// SiLU(gate) * up (input of the down projection).  One launch instead of two
// and no fp16 round trip through memory; the codes and scales are exactly the
// quantiser's on the fp16 tensor the unfused producer would have written, and
// that tensor can be written as well (the verify pass reads it).
//
// Arithmetic (fixed so that the codes are reproducible): the statistic and the
// exponential in binary64, one binary32 rounding of everything that touches the
// result, one rounding to fp16:
//   RMSNorm:  r = fp32(1 / sqrt(sum(x^2) / K + eps)),  h = fp16(fp32((x * w) * r))
//   SiLU*up:  s = fp32(g / (1 + exp(-g))),             h = fp16(fp32(s * u))
// x * w is exact in binary32 (two 11-bit significands).  Both kernels are bound
// by launch latency at draft sizes; the binary64 work is a few thousand
// instructions per wavefront.
//
// Further down: the two outlier-aware forms of the quantiser itself, a Hadamard
// rotation of every group (also available behind both producers) and a reordering
// quantiser that carries outlier groups at 239 levels as two 4-bit groups.
#pragma once
#include "common.hpp"
#include "quant_act.hpp"

namespace qspec {

constexpr int kRowMaxThreads = 1024;

// A binary32 value that exists as such: without this the compiler may merge the
// multiplication with the conversion to fp16 that follows into one mixed-precision
// instruction with a single rounding, which differs from the two roundings stated
// above about once in 10^5 values.
__device__ inline float rounded_f32(float v) {
  asm volatile("" : "+v"(v));
  return v;
}

template <int CTRL>
__device__ inline double dpp_f64(double v) {
  const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
  const unsigned lo = (unsigned)dpp_i32<CTRL>((int)(unsigned)b);
  const unsigned hi = (unsigned)dpp_i32<CTRL>((int)(unsigned)(b >> 32));
  return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}

__device__ inline double lane_value_f64(double v, int lane) {
  const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
  const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, lane);
  const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(b >> 32), lane);
  return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}

// Sum over the wavefront (every lane active), the same value in every lane: four folds
// inside each row of 16, then the four row totals.
__device__ inline double wave_sum_f64(double v) {
  v += dpp_f64<0xB1>(v);
  v += dpp_f64<0x4E>(v);
  v += dpp_f64<0x141>(v);
  v += dpp_f64<0x140>(v);
  return (lane_value_f64(v, 0) + lane_value_f64(v, 16)) + (lane_value_f64(v, 32) + lane_value_f64(v, 48));
}

// ---- outlier-spreading rotation in front of the quantiser: every group of 128
// features times H_128 / 8 (Sylvester Hadamard matrix, natural order), the
// rotation-based quantisers' answer to single large channels (paper Sec. 4.1 names
// such a quantiser among those it builds on; the block-diagonal form, which keeps the
// transform inside one quantisation group and one row of 16 lanes, is this build's).
// The weights are stored in the rotated basis (w_g H_128 / 16, offline), so the
// product is unchanged.  Arithmetic: the fast transform in binary32, stage h = 1, 2,
// ..., 64 replacing (v[j], v[j+h]) by (v[j] + v[j+h], v[j] - v[j+h]); scaling by 2^-3
// (exact); one rounding to fp16.  A thread's 8 values cover stages 1, 2, 4; stages 8
// to 64 pair lane l with lane l ^ 1, 2, 4, 8 of its row (DPP moves).
template <int CTRL>
__device__ inline float dpp_f32(float v) {
  return __builtin_bit_cast(float, dpp_i32<CTRL>(__builtin_bit_cast(int, v)));
}

// One stage across lanes: `other` is the partner lane's value, `upper` says whether
// this lane holds the v[j+h] side of its pairs.
__device__ inline float butterfly(float mine, float other, bool upper) {
  return upper ? other - mine : mine + other;
}

// The transform of one group held by a row of 16 lanes, 8 consecutive values per lane
// (l = lane within the row); every lane of the row must be active.
__device__ inline void hadamard_row16(float (&v)[8], int l) {
  // stages 1, 2, 4 inside the thread
#pragma unroll
  for (int h = 1; h < 8; h <<= 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if ((e & h) == 0) {
        const float a = v[e], b = v[e + h];
        v[e] = a + b;
        v[e + h] = a - b;
      }
    }
  }
  // stages 8, 16, 32, 64 across the 16 lanes of the row
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float t = v[e];
    t = butterfly(t, dpp_f32<0xB1>(t), (l & 1) != 0);                  // lane ^ 1
    t = butterfly(t, dpp_f32<0x4E>(t), (l & 2) != 0);                  // lane ^ 2
    // lane ^ 4: four lanes up for the lower side (a rotation by 12), four down for the upper
    const float up4 = dpp_f32<0x12C>(t), down4 = dpp_f32<0x124>(t);
    t = butterfly(t, (l & 4) ? down4 : up4, (l & 4) != 0);
    t = butterfly(t, dpp_f32<0x128>(t), (l & 8) != 0);                 // lane ^ 8: a rotation by 8
    v[e] = t;
  }
}

// v: 8 fp16 values widened to binary32.  Rotates (if asked), rounds to fp16, stores the
// fp16 tensor (if asked) and quantises, into the packed or (wide) the widened code format.
// Every lane of the wavefront calls it.
__device__ inline void finish_unit(float (&v)[8], bool rotate, bool live, size_t idx,
                                   uint32_t* __restrict__ qa_words, float* __restrict__ sa,
                                   uint4* __restrict__ h_out, bool wide = false) {
  v8h hh;
  if (rotate) {
    hadamard_row16(v, threadIdx.x & 15);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      hh[e] = (_Float16)(v[e] * 0.125f);                               // exact scaling: one rounding either way
      v[e] = (float)hh[e];
    }
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) hh[e] = (_Float16)v[e];                // v holds fp16 values: exact
  }
  if (h_out != nullptr && live) h_out[idx] = __builtin_bit_cast(uint4, hh);
  if (wide) quantise_unit_wide(v, live, idx, qa_words, sa);
  else quantise_unit(v, live, idx, qa_words, sa);
}

// 1/sqrt(v) in binary64 to within a few units in the last place, v > 0 and normal: the
// hardware estimate and three Newton steps (each squares the relative error), instead of
// the correctly rounded square root and division, whose long dependent chains would sit
// on this kernel's critical path.  The result is rounded to binary32 straight away.
__device__ inline double rsqrt_f64(double v) {
  double y = __builtin_amdgcn_rsq(v);
#pragma unroll
  for (int it = 0; it < 3; ++it) {
    const double e = fma(-v * y, y, 1.0);                  // 1 - v y^2
    y = fma(y * 0.5, e, y);                                // y (1 + e/2)
  }
  return y;
}

// grid M (one workgroup per token row), T = blockDim.x threads (a multiple of 64, at most
// 1024), 8 features per thread and pass.  NCH > 0: K <= NCH * 8 T and the row (and the norm
// weight) stay in registers between the two passes; NCH == 0: any K, the row is read again
// (from cache).  inv_K = 1 / K.  h_out may be null.
template <int NCH>
__global__ __launch_bounds__(kRowMaxThreads) void rmsnorm_quant_kernel(const uint4* __restrict__ x,
                                                                       const uint4* __restrict__ w, float eps,
                                                                       int K, double inv_K,
                                                                       uint32_t* __restrict__ qa_words,
                                                                       float* __restrict__ sa,
                                                                       uint4* __restrict__ h_out, int rotate) {
  const int tid = threadIdx.x, T = blockDim.x;
  const int kw = K / 8;                                    // 16-byte pieces per row
  const size_t row0 = (size_t)blockIdx.x * kw;
  const int chunks = NCH > 0 ? NCH : (kw + T - 1) / T;
  const uint4 zero = {0u, 0u, 0u, 0u};
  uint4 keep[NCH > 0 ? NCH : 1], wkeep[NCH > 0 ? NCH : 1];

  double ss = 0.0;
#pragma unroll
  for (int c = 0; c < chunks; ++c) {
    const int piece = c * T + tid;
    const uint4 raw = piece < kw ? x[row0 + piece] : zero;
    if (NCH > 0) {
      keep[c] = raw;
      wkeep[c] = piece < kw ? w[piece] : zero;             // in flight during the reduction
    }
    const v8h h = __builtin_bit_cast(v8h, raw);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const double d = (double)(float)h[e];
      ss += d * d;                                         // the square is exact
    }
  }
  ss = wave_sum_f64(ss);
  __shared__ double part[kRowMaxThreads / 64];
  if ((tid & 63) == 0) part[tid >> 6] = ss;
  __syncthreads();
  double total = part[0];
  for (int i = 1; i < (T >> 6); ++i) total += part[i];
  const double v = total * inv_K + (double)eps;
  // v == 0 only for a zero row with eps == 0: the outputs are 0 * r, and r = inf would make them NaN
  const float r = v > 0.0 ? (float)rsqrt_f64(v) : 0.0f;

#pragma unroll
  for (int c = 0; c < chunks; ++c) {
    const int piece = c * T + tid;
    const bool live = piece < kw;
    const uint4 raw = NCH > 0 ? keep[c] : (live ? x[row0 + piece] : zero);
    const uint4 wraw = NCH > 0 ? wkeep[c] : (live ? w[piece] : zero);
    const v8h xh = __builtin_bit_cast(v8h, raw);
    const v8h wh = __builtin_bit_cast(v8h, wraw);
    float v8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float t = (float)xh[e] * (float)wh[e];         // exact
      v8[e] = (float)(_Float16)rounded_f32(t * r);
    }
    finish_unit(v8, (rotate & 1) != 0, live, row0 + piece, qa_words, sa, h_out, (rotate & 2) != 0);
  }
}

// gate_up: fp16 [M][2I], the gate in the first I columns.  One thread per 8 outputs,
// n_words = M * I / 8.  h_out may be null.
__global__ __launch_bounds__(256) void silu_mul_quant_kernel(const uint4* __restrict__ gate_up, int I8,
                                                             uint32_t* __restrict__ qa_words,
                                                             float* __restrict__ sa, uint4* __restrict__ h_out,
                                                             size_t n_words, int rotate) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool live = idx < n_words;
  uint4 graw = {0u, 0u, 0u, 0u}, uraw = {0u, 0u, 0u, 0u};
  if (live) {
    const size_t m = idx / (size_t)I8, p = idx - m * (size_t)I8;
    graw = gate_up[m * 2 * (size_t)I8 + p];
    uraw = gate_up[m * 2 * (size_t)I8 + (size_t)I8 + p];
  }
  const v8h gh = __builtin_bit_cast(v8h, graw);
  const v8h uh = __builtin_bit_cast(v8h, uraw);
  float v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const double g = (double)(float)gh[e];
    const float s = (float)(g / (1.0 + exp(-g)));
    v[e] = (float)(_Float16)rounded_f32(s * (float)uh[e]);
  }
  finish_unit(v, (rotate & 1) != 0, live, idx, qa_words, sa, h_out, (rotate & 2) != 0);
}

__global__ __launch_bounds__(256) void hadamard_quant_kernel(const uint4* __restrict__ x,
                                                             uint32_t* __restrict__ qa_words,
                                                             float* __restrict__ sa, uint4* __restrict__ h_out,
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
  finish_unit(v, true, live, idx, qa_words, sa, h_out);
}

// ---- reordering quantiser: outlier channels last, their groups at 239 levels.
// The reorder-and-keep-outliers-in-higher-precision quantisers that the paper
// builds on (Sec. 4.1; no detail given) need a mixed-precision GEMM; this form does
// not: an outlier group is quantised with s = a / 119, q8 in [-119, 119], and
// written as two ordinary 4-bit groups, q8 = 16 hi + lo with lo in [-8, 7] and hi in
// [-7, 7], scales 16 s and s, which multiply the same weight group (held twice in
// the packed weights).  The draft-mode GEMM sees K' = K + 128 G_o input features.
//   perm[p]: input channel at position p of the reordered row (entries are clamped
//   to [0, K)); the last G_o groups of the reordered row are the outlier groups.
// Output groups: the ordinary ones in order, then hi, lo of each outlier group.
// One thread per 8 reordered positions, 16 lanes per group.  h_out (may be null):
// fp16 [M][K'], the gathered row with a zero group after each outlier group, i.e.
// the verify-mode input for the same expanded weights.
__global__ __launch_bounds__(256) void reorder_quant_kernel(const uint16_t* __restrict__ x,
                                                            const int* __restrict__ perm, int K, int Go,
                                                            uint32_t* __restrict__ qa_words,
                                                            float* __restrict__ sa, uint4* __restrict__ h_out,
                                                            size_t n_words) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool live = idx < n_words;
  const int K8 = K / 8, G = K / kGroup;
  const size_t m = idx / (size_t)K8;
  const int p8 = (int)(idx - m * (size_t)K8);
  const int g = p8 >> 4, kw = p8 & 15;
  float v[8];
  v8h raw;
#pragma unroll
  for (int e = 0; e < 8; ++e) raw[e] = (_Float16)0.0f;
  if (live) {
    const int4 c0 = *reinterpret_cast<const int4*>(perm + 8 * p8);
    const int4 c1 = *reinterpret_cast<const int4*>(perm + 8 * p8 + 4);
    const int ch[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
    const uint16_t* row = x + m * (size_t)K;
#pragma unroll
    for (int e = 0; e < 8; ++e) raw[e] = __builtin_bit_cast(_Float16, row[min(max(ch[e], 0), K - 1)]);
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (float)raw[e];
  float a = 0.0f;
#pragma unroll
  for (int e = 0; e < 8; ++e) a = fmaxf(a, fabsf(v[e]));
  a = row16_max(a);
  if (!live) return;

  const int Gx = G + Go;                                  // groups of the output
  const bool outlier = g >= G - Go;
  const int og = outlier ? (G - Go) + 2 * (g - (G - Go)) : g;    // output group (the hi group of an outlier group)
  // word position inside a group: k-word kw = 4i + kb is stored at 4kb + i
  const int wpos = ((kw & 3) << 2) + (kw >> 2);
  const size_t wbase = (m * (size_t)Gx + og) * 16 + wpos;
  const size_t hbase = (m * (size_t)Gx + og) * 16 + kw;   // 16-byte pieces of the fp16 row
  if (!outlier) {
    const float s = a / 7.0f;
    uint32_t w = 0;
    if (a > 0.0f) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float t = rintf(v[e] / s);
        t = fminf(fmaxf(t, -8.0f), 7.0f);
        w |= ((uint32_t)(int)t & 0xFu) << (4 * nibble_pos(e));
      }
    }
    qa_words[wbase] = w;
    if (kw == 0) sa[m * (size_t)Gx + og] = s;
    if (h_out != nullptr) h_out[hbase] = __builtin_bit_cast(uint4, raw);
  } else {
    const float s = a / 119.0f;
    uint32_t whi = 0, wlo = 0;
    if (a > 0.0f) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float t = rintf(v[e] / s);
        t = fminf(fmaxf(t, -119.0f), 119.0f);
        const int q8 = (int)t;
        const int lo = ((q8 + 8) & 15) - 8;
        const int hi = (q8 - lo) >> 4;                    // exact: q8 - lo is a multiple of 16
        whi |= ((uint32_t)hi & 0xFu) << (4 * nibble_pos(e));
        wlo |= ((uint32_t)lo & 0xFu) << (4 * nibble_pos(e));
      }
    }
    qa_words[wbase] = whi;
    qa_words[wbase + 16] = wlo;
    if (kw == 0) {
      sa[m * (size_t)Gx + og] = s * 16.0f;
      sa[m * (size_t)Gx + og + 1] = s;
    }
    if (h_out != nullptr) {
      const uint4 zero = {0u, 0u, 0u, 0u};
      h_out[hbase] = __builtin_bit_cast(uint4, raw);
      h_out[hbase + 16] = zero;
    }
  }
}

}  // namespace qspec
