// Small-M (memory-bound) kernels for both modes: the weights are streamed once
// from HBM with a register prefetch ring, everything that is re-used (the
// activation chunk, its scales, the weight scales) is staged in LDS.
//
// A workgroup has WN x WK wavefronts and owns WN weight tiles (16 outputs
// each) over one K-chunk (chunk c of S along K).  Waves with the same wn
// share an output tile and split the chunk's groups between them (WK-way
// split-K inside the workgroup, combined through LDS).  With S > 1 the
// workgroup writes fp32 partial sums to the workspace and a second tiny
// kernel adds the S slices and rounds to fp16; with S == 1 it stores fp16.
//
// MFMA operand roles are those of gemm_generic.hpp (A = weights, B = acts).
#pragma once
#include "common.hpp"

namespace qspec {

struct SmallArgs {
  const uint4* codes;        // blob code tiles
  const uint16_t* scalesT;   // blob fp16 scales [G][N]
  const void* act;           // W4A4: qa bytes [M][K/2]; W4A16: x fp16 [M][K]
  const float* sa;           // W4A4: [M][G]
  uint16_t* y;               // fp16 [M][N]
  float* ws;                 // fp32 [S][M][N] when S > 1
  int M, N, K, G;
  int S;                     // K-chunks (grid.y)
  int gc_max;                // largest number of groups in a chunk
};

// 16-byte streaming load: weights are read exactly once, keep them from
// displacing the re-used operands in the caches.
constexpr int kStageU = 8;   // 16-byte activation pieces a thread stages in its single pass

__device__ inline uint4 load_stream(const uint4* p) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return uint4{v.x, v.y, v.z, v.w};
}

template <bool W4A4, int TM>
struct SmallLds {
  // byte offsets inside the dynamic LDS block, all multiples of 16
  int act_pitch;   // bytes per activation row (padded so that 16 rows hit 16 different 16-byte slots)
  int act_bytes, sw_off, sw_bytes, sa_off, sa_bytes, total;
  __host__ __device__ SmallLds(int gc_max, int WN) {
    const int row = W4A4 ? gc_max * 64 : gc_max * 256;
    act_pitch = row + 16;
    act_bytes = TM * 16 * act_pitch;
    sw_off = act_bytes;
    sw_bytes = gc_max * WN * 32;
    sa_off = sw_off + sw_bytes;
    sa_bytes = W4A4 ? gc_max * TM * 16 * 4 : 0;
    total = sa_off + sa_bytes;
  }
};

template <bool W4A4, int TM, int WN, int WK, int D>
__global__ __launch_bounds__(WN * WK * 64) void gemm_small_kernel(SmallArgs p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  constexpr int NTHREADS = WN * WK * 64;
  constexpr int ROWS = TM * 16;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps control flow scalar
  const int wn = wave % WN, wk = wave / WN;
  const int r16 = lane & 15, kb = lane >> 4;
  const int G = p.G;
  const int T = blockIdx.x * WN + wn;
  const bool active = T < p.N / 16;
  const int c = blockIdx.y;
  const int g0 = (int)(((long long)c * G) / p.S);
  const int g1 = (int)(((long long)(c + 1) * G) / p.S);
  const int gcl = g1 - g0;
  const SmallLds<W4A4, TM> L(p.gc_max, WN);

  // ---- start streaming this wave's weight tiles before anything else
  const int h0 = g0 + (wk * gcl) / WK;
  const int h1 = g0 + ((wk + 1) * gcl) / WK;
  const int n_it = active ? h1 - h0 : 0;
  // All loads below are unconditional with clamped indices: a load inside a
  // branch makes the compiler drain the whole memory pipeline (vmcnt(0)) at
  // every use, which serialises the stream.
  const int last_it = max(h1 - h0, 1) - 1;
  const uint4* wp = p.codes + ((size_t)(active ? T : 0) * G + h0) * 64 + lane;
  uint4 buf[D];
#pragma unroll
  for (int d = 0; d < D; ++d) buf[d] = load_stream(wp + (size_t)min(d, last_it) * 64);

  // ---- stage the re-used operands of this chunk.  Straight-line code (the
  // host guarantees that one pass of kStageU pieces per thread covers a row):
  // all global loads are issued back to back, then stored to LDS.
  {
    constexpr int TPR = NTHREADS / ROWS;                    // threads per activation row
    constexpr int U = kStageU;
    const int row_pieces = gcl * (W4A4 ? 4 : 16);           // 16-byte pieces per activation row
    const int row_bytes = W4A4 ? p.K / 2 : p.K * 2;
    const int col0 = g0 * (W4A4 ? 64 : 256);
    const int m = tid / TPR, j = tid % TPR;
    const uint8_t* src = static_cast<const uint8_t*>(p.act) + (size_t)min(m, p.M - 1) * row_bytes + col0;
    uint8_t* dst = lds + m * L.act_pitch;
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int pc = min(j + u * TPR, row_pieces - 1);
      v[u] = *reinterpret_cast<const uint4*>(src + pc * 16);
    }
    // weight scales: [gl][WN*16] fp16, 8-byte pieces (4 scales); at most one piece per thread
    const int n_base = blockIdx.x * WN * 16;
    const int sw_pieces = gcl * WN * 4;
    const int qs = min(tid, sw_pieces - 1);
    const int sgl = qs / (WN * 4), sj = qs - sgl * (WN * 4);
    const int sn = min(n_base + sj * 4, p.N - 4);
    const uint2 swv = *reinterpret_cast<const uint2*>(p.scalesT + (size_t)(g0 + sgl) * p.N + sn);
    // activation scales (W4A4): [gl][ROWS] floats, at most two per thread
    float sav[2] = {0.0f, 0.0f};
    if (W4A4) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int q = min(tid + u * NTHREADS, gcl * ROWS - 1);
        const int mm = q / gcl, gl = q - mm * gcl;
        sav[u] = p.sa[(size_t)min(mm, p.M - 1) * G + g0 + gl];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int pc = j + u * TPR;
      if (m >= p.M) v[u] = uint4{0u, 0u, 0u, 0u};
      if (pc < row_pieces) *reinterpret_cast<uint4*>(dst + pc * 16) = v[u];
    }
    if (tid < sw_pieces) *reinterpret_cast<uint2*>(lds + L.sw_off + tid * 8) = swv;
    if (W4A4) {
      float* sa_l = reinterpret_cast<float*>(lds + L.sa_off);
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int q = tid + u * NTHREADS;
        const int mm = q / gcl, gl = q - mm * gcl;
        if (q < gcl * ROWS) sa_l[gl * ROWS + mm] = mm < p.M ? sav[u] : 0.0f;
      }
    }
  }
  __syncthreads();

  float facc[TM][4];
#pragma unroll
  for (int t = 0; t < TM; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) facc[t][r] = 0.0f;

  {
    for (int it = 0; it < n_it; it += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        if (it + d < n_it) {
          const uint4 wq = buf[d];
          const int gl = h0 + it + d - g0;
          const uint2 sraw = *reinterpret_cast<const uint2*>(lds + L.sw_off + ((gl * WN + wn) * 4 + kb) * 8);
          float sw[4];
          const float fold = W4A4 ? 0.00390625f : 1.0f;   // both int8 operands carry a factor 16
          sw[0] = half_bits_to_float((uint16_t)(sraw.x & 0xFFFF)) * fold;
          sw[1] = half_bits_to_float((uint16_t)(sraw.x >> 16)) * fold;
          sw[2] = half_bits_to_float((uint16_t)(sraw.y & 0xFFFF)) * fold;
          sw[3] = half_bits_to_float((uint16_t)(sraw.y >> 16)) * fold;
          if (W4A4) {
            const I8Pair a = unpack_i8(wq);
            const float* sa_l = reinterpret_cast<const float*>(lds + L.sa_off) + gl * ROWS;
#pragma unroll
            for (int t = 0; t < TM; ++t) {
              const uint4 aq = *reinterpret_cast<const uint4*>(lds + (16 * t + r16) * L.act_pitch + gl * 64 + kb * 16);
              const I8Pair b = unpack_i8(aq);
              v4i acc = {0, 0, 0, 0};
              acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a.lo, b.lo, acc, 0, 0, 0);
              acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a.hi, b.hi, acc, 0, 0, 0);
              const float s = sa_l[16 * t + r16];
#pragma unroll
              for (int r = 0; r < 4; ++r) facc[t][r] += (float)acc[r] * (s * sw[r]);
            }
          } else {
            v8h wa[4];
            wa[0] = dequant_word(wq.x);
            wa[1] = dequant_word(wq.y);
            wa[2] = dequant_word(wq.z);
            wa[3] = dequant_word(wq.w);
#pragma unroll
            for (int t = 0; t < TM; ++t) {
              const uint8_t* xr = lds + (16 * t + r16) * L.act_pitch + gl * 256 + kb * 16;
              v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                const uint4 xq = *reinterpret_cast<const uint4*>(xr + 64 * i);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa[i], __builtin_bit_cast(v8h, xq), acc, 0, 0, 0);
              }
#pragma unroll
              for (int r = 0; r < 4; ++r) facc[t][r] += acc[r] * sw[r];
            }
          }
        }
      }
      if (it + D < n_it) {                 // refill the ring for the next batch
#pragma unroll
        for (int d = 0; d < D; ++d) buf[d] = load_stream(wp + (size_t)min(it + D + d, last_it) * 64);
      }
    }
  }

  // ---- combine the WK split-K waves of each tile through LDS (re-uses the act region)
  if (WK > 1) {
    __syncthreads();                                  // everyone is done reading the staged operands
    float* red = reinterpret_cast<float*>(lds);       // [wk][wn][TM*4][64]
#pragma unroll
    for (int t = 0; t < TM; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[((wk * WN + wn) * TM * 4 + t * 4 + r) * 64 + lane] = facc[t][r];
    __syncthreads();
    if (wk == 0) {
#pragma unroll
      for (int t = 0; t < TM; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float s = facc[t][r];
#pragma unroll
          for (int w = 1; w < WK; ++w) s += red[((w * WN + wn) * TM * 4 + t * 4 + r) * 64 + lane];
          facc[t][r] = s;
        }
    }
  }
  if (wk != 0 || !active) return;

#pragma unroll
  for (int t = 0; t < TM; ++t) {
    const int m = 16 * t + r16;
    if (m >= p.M) continue;
    const size_t o = (size_t)m * p.N + T * 16 + 4 * kb;
    if (p.S > 1) {
      *reinterpret_cast<float4*>(p.ws + (size_t)c * p.M * p.N + o) =
          float4{facc[t][0], facc[t][1], facc[t][2], facc[t][3]};
    } else {
      uint2 out;
      out.x = (uint32_t)float_to_half_bits(facc[t][0]) | ((uint32_t)float_to_half_bits(facc[t][1]) << 16);
      out.y = (uint32_t)float_to_half_bits(facc[t][2]) | ((uint32_t)float_to_half_bits(facc[t][3]) << 16);
      *reinterpret_cast<uint2*>(p.y + o) = out;
    }
  }
}

// y = fp16( sum over the S K-chunk slices ), 4 outputs per thread
__global__ __launch_bounds__(256) void splitk_finish_kernel(const float4* __restrict__ ws, uint2* __restrict__ y,
                                                            size_t n_quads, int S) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_quads) return;
  float4 s = ws[i];
  for (int c = 1; c < S; ++c) {
    const float4 v = ws[(size_t)c * n_quads + i];
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  uint2 out;
  out.x = (uint32_t)float_to_half_bits(s.x) | ((uint32_t)float_to_half_bits(s.y) << 16);
  out.y = (uint32_t)float_to_half_bits(s.z) | ((uint32_t)float_to_half_bits(s.w) << 16);
  y[i] = out;
}

}  // namespace qspec
