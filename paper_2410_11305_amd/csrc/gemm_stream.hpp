// Memory-bound (small M) kernels for both modes, wave-autonomous form.
//
// A workgroup of 8 wavefronts owns NT adjacent weight tiles (16 outputs each)
// over the whole of K.  Wave w takes the K groups g = w, w+8, w+16, ...; for
// each of them it loads the activation operand of that group ONCE into
// registers (straight from global memory: the activations are small and stay
// in L2) and re-uses it against the NT weight tiles, which stream from HBM
// exactly once.  Nothing is staged in LDS, so there is no barrier in the
// streaming loop and no split-K pass over a workspace: the eight per-wave
// fp32 sums of a tile are combined through LDS at the very end and stored as
// fp16.
//
// All global loads are unconditional buffer loads (work that does not exist
// gets an out-of-range offset, which reads as zero without memory traffic;
// a load inside a branch would make the compiler drain the whole memory
// pipeline at every use) and two register sets alternate, so that the loads
// of the next group are in flight while the current one is computed.
//
// MFMA operand roles: A = weights (row = n % 16), B = activations (column =
// m % 16), k-block = lane / 16; D[i][j]: lane holds rows 4*(lane/16)+r.
#pragma once
#include "buffer.hpp"
#include "exchange.hpp"
#include "common.hpp"

namespace qspec {

struct StreamArgs {
  const uint4* codes;        // blob code tiles
  const uint16_t* scalesT;   // blob fp16 scales [G][N]
  const void* act;           // W4A4: qa bytes [M][K/2]; W4A16: x fp16 [M][K]
  const float* sa;           // W4A4: [M][G]
  uint16_t* y;               // fp16 [M][N]
  float* ws;                 // S > 1: fp32 partial sums [S][tile block][output fragment]
  unsigned* tickets;         // S > 1: one arrival counter per tile block, zero on entry and on exit
  int M, N, K, G;
  int S;                     // K-slices: workgroup b owns tile block b / S, slice b % S
};

constexpr int kStreamWaves = 8;

struct StreamRsrc {
  rsrc_t codes, scales, act, sa;
};

// From this many tiles per workgroup on, the scales of two groups come in one load
// (below that the two ds_bpermute per tile cost more than the load they replace).
#ifndef QSPEC_PAIR_SCALES_MIN_NT
#define QSPEC_PAIR_SCALES_MIN_NT 2
#endif
__device__ __host__ inline constexpr bool pair_scales(int nt) { return nt >= QSPEC_PAIR_SCALES_MIN_NT; }

template <bool W4A4, int TM, int NT>
struct GroupRegs {
  uint4 w[NT];                      // one weight tile slice per n-tile
  uint2 sw[NT];                     // 4 fp16 weight scales (rows 4*kb .. 4*kb+3 of the tile); unused with pair scales
  uint4 a[W4A4 ? TM : TM * 4];      // activation operand(s) of this group
  float sa[W4A4 ? TM : 1];          // activation scales (W4A4)
};

// Issue every load of group g (valid == false: all offsets out of range, no traffic).
// wlds != nullptr: the weight tiles of this workgroup were copied to LDS beforehand, tile j
// of group g at wlds + (j * G + g) * 1024, and are read from there.
template <bool W4A4, int TM, int NT>
__device__ inline void load_group(GroupRegs<W4A4, TM, NT>& R, const StreamRsrc& rs, const StreamArgs& p, int g,
                                  bool valid, int T0, int nt_valid, int lane, const uint8_t* wlds = nullptr) {
  const int r16 = lane & 15, kb = lane >> 4;
  // activations first: loads return in order, and the (L2-resident) activations
  // must not queue behind the HBM weight tiles
#pragma unroll
  for (int t = 0; t < TM; ++t) {
    const uint32_t m = 16 * t + r16;               // rows past M lie past the end of the buffer: they read as 0
    if (W4A4) {
      R.a[t] = buf_load16(rs.act, valid ? m * (uint32_t)(p.K / 2) + 64u * g + 16u * kb : kOutOfRange);
      R.sa[t] = buf_load_f32(rs.sa, valid ? (m * p.G + g) * 4u : kOutOfRange);
    } else {
      // Coalesced form: load u = 4t + i covers token rows 4u .. 4u+3, 256 contiguous
      // bytes (one group) per row, 16 lanes per row.  compute_group turns this into
      // the MFMA operand layout through a wave-private LDS buffer.  (Loading the
      // operand layout directly touches 16 rows x 64 bytes at a 2K-byte stride per
      // instruction, which the caches serve at a fraction of their bandwidth.)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t row = 4u * (4 * t + i) + kb;
        R.a[t * 4 + i] = buf_load16(rs.act, valid ? (row * (uint32_t)p.K + (uint32_t)g * kGroup) * 2u + r16 * 16u
                                                  : kOutOfRange);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const bool ok = valid && j < nt_valid;
    const uint32_t T = (uint32_t)(T0 + j);
    if (wlds != nullptr) {
      R.w[j] = ok ? *reinterpret_cast<const uint4*>(wlds + ((size_t)(j * p.G + g) * 1024u + lane * 16u)) : uint4{0u, 0u, 0u, 0u};
    } else {
      R.w[j] = buf_load16_stream(rs.codes, ok ? (T * p.G + g) * 1024u + lane * 16u : kOutOfRange);
    }
    if (!pair_scales(NT)) R.sw[j] = buf_load8(rs.scales, ok ? ((uint32_t)g * p.N + T * 16u + 4u * kb) * 2u : kOutOfRange);
  }
}

// Weight scales of a PAIR of groups (ga: the even step, gb: the odd one) and all NT
// tiles in one load instruction: lane (c = lane % 16, kb = lane / 16) fetches the four
// fp16 scales of rows 4*kb .. 4*kb+3 of tile c % NT of group ga (c < NT) or gb
// (NT <= c < 2*NT).  compute_group fetches them from that lane with ds_bpermute (no
// LDS memory involved).  Measured: every further load instruction per group costs
// streaming time even when it hits in cache (the vector memory queue, not DRAM, is
// what it occupies), so 2*NT small loads per pair became one.
template <int NT>
__device__ inline uint2 load_pair_scales(const StreamRsrc& rs, const StreamArgs& p, int ga, int gb, bool va, bool vb,
                                         int T0, int nt_valid, int lane) {
  static_assert(2 * NT <= 16, "one lane row holds both groups of all tiles");
  const int c = lane & 15, kb = lane >> 4;
  const int q = c / NT, j = c - q * NT;
  const bool ok = (q == 0 ? va : (q == 1 && vb)) && j < nt_valid;
  const uint32_t g = (uint32_t)(q == 0 ? ga : gb);
  return buf_load8(rs.scales, ok ? (g * (uint32_t)p.N + (uint32_t)(T0 + j) * 16u + 4u * kb) * 2u : kOutOfRange);
}

// The scales of tile j in step Q (0: even, 1: odd) of the pair, from the lane that loaded them.
template <int NT, int Q>
__device__ inline uint2 pair_scales_of(uint2 swp, int j, int lane) {
  const int idx = ((lane & 48) + Q * NT + j) << 2;
  uint2 r;
  r.x = (uint32_t)__builtin_amdgcn_ds_bpermute(idx, (int)swp.x);
  r.y = (uint32_t)__builtin_amdgcn_ds_bpermute(idx, (int)swp.y);
  return r;
}

constexpr int kXPitch = 256 + 16;     // bytes per token row of the transpose buffer (odd number of 16-byte slots)

template <bool W4A4, int TM, int NT, int Q>
__device__ inline void compute_group(const GroupRegs<W4A4, TM, NT>& R, uint2 swp, float (&facc)[NT][TM][4],
                                     uint8_t* xbuf, int lane) {
  if (W4A4) {
    // weight operands and scales of all NT tiles first, then token tile by token tile
    // (one unpacked activation operand live at a time: TM goes up to 8)
    I8Pair a[NT];
    float sw[NT][4];
    // With two or more token tiles the int32 -> fp32 conversion is folded away: the MFMA
    // chain starts from the bit pattern of 1.5 * 2^23, so the finished int32 register READ
    // AS A FLOAT is 12582912 + 256 P exactly (|256 P| <= 2^21: inside the binade, one unit
    // in the last place = 1), and fma(that, sw, -12582912 * sw) is the correctly rounded
    // 256 P * sw (the constant is exact: sw has 11 significant bits, 1.5 * 2^23 two).  Two
    // vector instructions per output and group instead of three, plus one per weight row
    // and group that the TM token tiles share.
    constexpr bool kMagic = TM >= 2;
    constexpr int kMagicBits = 0x4B400000;              // 12582912.0f
    float swc[NT][4];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      a[j] = unpack_i8(R.w[j]);
      const uint2 sq = pair_scales(NT) ? pair_scales_of<NT, Q>(swp, j, lane) : R.sw[j];
      // both int8 operands carry a factor 16: fold 2^-8 into the weight scale (exact)
      sw[j][0] = half_bits_to_float((uint16_t)(sq.x & 0xFFFF)) * 0.00390625f;
      sw[j][1] = half_bits_to_float((uint16_t)(sq.x >> 16)) * 0.00390625f;
      sw[j][2] = half_bits_to_float((uint16_t)(sq.y & 0xFFFF)) * 0.00390625f;
      sw[j][3] = half_bits_to_float((uint16_t)(sq.y >> 16)) * 0.00390625f;
      if (kMagic) {
#pragma unroll
        for (int r = 0; r < 4; ++r) swc[j][r] = sw[j][r] * -12582912.0f;
      }
    }
#pragma unroll
    for (int t = 0; t < TM; ++t) {
      const I8Pair b = unpack_i8(R.a[t]);
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        v4i acc = kMagic ? v4i{kMagicBits, kMagicBits, kMagicBits, kMagicBits} : v4i{0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[j].lo, b.lo, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[j].hi, b.hi, acc, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (kMagic) {
            const int bits = acc[r];                    // (a copy: bit_cast of a vector element lvalue reads element 0)
            facc[j][t][r] = __builtin_fmaf(__builtin_fmaf(__builtin_bit_cast(float, bits), sw[j][r], swc[j][r]),
                                           R.sa[t], facc[j][t][r]);
          } else {
            facc[j][t][r] += (float)acc[r] * (R.sa[t] * sw[j][r]);
          }
        }
      }
    }
  } else {
    // rows x 256 B (as loaded) -> operand layout: lane (r16, kb), step i reads the
    // 16 bytes of row 16t + r16 that hold k = 32i + 8kb .. +8.  Only this wave
    // touches xbuf and LDS executes a wave's accesses in order: no barrier.
    const int r16 = lane & 15, kb = lane >> 4;
#pragma unroll
    for (int u = 0; u < TM * 4; ++u)
      *reinterpret_cast<uint4*>(xbuf + (4 * u + kb) * kXPitch + r16 * 16) = R.a[u];
    uint4 xb[TM * 4];
#pragma unroll
    for (int t = 0; t < TM; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        xb[t * 4 + i] = *reinterpret_cast<const uint4*>(xbuf + (16 * t + r16) * kXPitch + (4 * i + kb) * 16);
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      v8h wa[4];
      wa[0] = dequant_word(R.w[j].x);
      wa[1] = dequant_word(R.w[j].y);
      wa[2] = dequant_word(R.w[j].z);
      wa[3] = dequant_word(R.w[j].w);
      const uint2 sq = pair_scales(NT) ? pair_scales_of<NT, Q>(swp, j, lane) : R.sw[j];
      float sw[4];
      sw[0] = half_bits_to_float((uint16_t)(sq.x & 0xFFFF));
      sw[1] = half_bits_to_float((uint16_t)(sq.x >> 16));
      sw[2] = half_bits_to_float((uint16_t)(sq.y & 0xFFFF));
      sw[3] = half_bits_to_float((uint16_t)(sq.y >> 16));
#pragma unroll
      for (int t = 0; t < TM; ++t) {
        v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int i = 0; i < 4; ++i)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa[i], __builtin_bit_cast(v8h, xb[t * 4 + i]), acc, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) facc[j][t][r] += acc[r] * sw[r];
      }
    }
  }
}

template <bool W4A4, int TM, int NT>
__global__ __launch_bounds__(kStreamWaves * 64) void gemm_stream_kernel(StreamArgs p) {
  constexpr int W = kStreamWaves;
  // LDS: per-wave transpose buffers while streaming (verify mode), re-used as the
  // split-K reduction buffer at the end
  constexpr int kChunk = NT * TM < W ? NT * TM : W;      // output tiles combined per pass, one per wave
  constexpr int kRedBytes = W * kChunk * 4 * kWave * 4;
  constexpr int kXBytes = W4A4 ? 0 : W * TM * 16 * kXPitch;
  __shared__ __attribute__((aligned(16))) uint8_t lds[kRedBytes > kXBytes ? kRedBytes : kXBytes];
  float (*red)[kChunk * 4][kWave] = reinterpret_cast<float (*)[kChunk * 4][kWave]>(lds);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r16 = lane & 15, kb = lane >> 4;
  const int tb = blockIdx.x / p.S, slice = blockIdx.x - tb * p.S;
  const int T0 = tb * NT;
  const int nt_valid = min(NT, p.N / 16 - T0);        // >= 1 by construction of the grid
  const int G = p.G;
  // token-row blocks along gridDim.y (only without K-slices): this workgroup owns rows m_base .. m_base + 16*TM - 1
  const int m_base = (int)blockIdx.y * (16 * TM);
  const int Mloc = p.M - m_base;
  if (Mloc <= 0) return;                           // (the whole workgroup: uniform)
  uint16_t* const yloc = p.y + (size_t)m_base * p.N;
  const int g0 = (int)(((long long)slice * G) / p.S), g1 = (int)(((long long)(slice + 1) * G) / p.S);
  // groups of this wave: g0 + wave, g0 + wave + W, ...  (n_g of them, possibly none)
  const int n_g = max(0, (g1 - g0 - wave + W - 1) / W);

  float facc[NT][TM][4];
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int t = 0; t < TM; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) facc[j][t][r] = 0.0f;

  uint8_t* xbuf = lds + (W4A4 ? 0 : wave * TM * 16 * kXPitch);
  if (n_g > 0) {
    StreamRsrc rs;
    rs.codes = make_rsrc(p.codes, (uint32_t)((size_t)p.N * p.K / 2));
    rs.scales = make_rsrc(p.scalesT, (uint32_t)((size_t)p.N * G * 2));
    const uint8_t* act0 = static_cast<const uint8_t*>(p.act) + (size_t)m_base * (W4A4 ? p.K / 2 : p.K * 2);
    rs.act = make_rsrc(act0, (uint32_t)(W4A4 ? (size_t)Mloc * p.K / 2 : (size_t)Mloc * p.K * 2));
    rs.sa = make_rsrc(W4A4 ? (const void*)(p.sa + (size_t)m_base * G) : (const void*)act0, (uint32_t)((size_t)Mloc * G * 4));
    // Workgroups start at different points of their K sequence so that the 256
    // CUs do not all ask L2 for the same activation lines at the same moment.
    const int rot = (int)(blockIdx.x % (unsigned)n_g);
    auto grp = [&](int it) { int q = it + rot; q = q >= n_g ? q - n_g : q; return g0 + wave + q * W; };
    // Two register sets alternate: the loads of the next group are in flight
    // while one group is computed.  (A third set was measured and is slower: the
    // memory system is throughput-bound here, more requests in flight only
    // queue up.)  The scheduling barriers pin the order "issue loads, then
    // compute": without them the compiler sinks the loads below the arithmetic.
    GroupRegs<W4A4, TM, NT> A, B;
    uint2 sw_cur = {0u, 0u}, sw_nxt = {0u, 0u};
    if (pair_scales(NT)) sw_cur = load_pair_scales<NT>(rs, p, grp(0), grp(1), true, 1 < n_g, T0, nt_valid, lane);
    load_group<W4A4, TM, NT>(A, rs, p, grp(0), true, T0, nt_valid, lane);
    for (int it = 0; it < n_g; it += 2) {
      // the scales of the next pair go out ahead of this pair's second group: they are
      // back (loads return in order) long before the register move at the bottom
      if (pair_scales(NT)) sw_nxt = load_pair_scales<NT>(rs, p, grp(it + 2), grp(it + 3), it + 2 < n_g, it + 3 < n_g, T0, nt_valid, lane);
      load_group<W4A4, TM, NT>(B, rs, p, grp(it + 1), it + 1 < n_g, T0, nt_valid, lane);
      __builtin_amdgcn_sched_barrier(0);
      compute_group<W4A4, TM, NT, 0>(A, sw_cur, facc, xbuf, lane);
      __builtin_amdgcn_sched_barrier(0);
      load_group<W4A4, TM, NT>(A, rs, p, grp(it + 2), it + 2 < n_g, T0, nt_valid, lane);
      __builtin_amdgcn_sched_barrier(0);
      if (it + 1 < n_g) compute_group<W4A4, TM, NT, 1>(B, sw_cur, facc, xbuf, lane);
      __builtin_amdgcn_sched_barrier(0);
      sw_cur = sw_nxt;
    }
  }

  // ---- combine the eight per-wave sums of every output tile, kChunk tiles per pass
  // through LDS (the transpose buffers are dead from here on).  With K-slices the
  // sums go to the workspace first (one 16-byte piece per lane and output tile,
  // contiguous per wavefront); the workgroup that arrives last at the tile block's
  // counter adds the slices in slice order and stores fp16.
  __shared__ unsigned ticket;
  const int nblocks = gridDim.x / p.S;
  auto frag = [&](int c, int o) -> float* {
    return p.ws + ((((size_t)c * nblocks + tb) * (NT * TM) + o) * kWave + lane) * 4;
  };
#pragma unroll
  for (int base = 0; base < NT * TM; base += kChunk) {
    // the buffer must be free: the last pass has been read, and (verify mode) every
    // wave is done with its transpose buffer, which the sums overwrite
    if (!W4A4 || base > 0) __syncthreads();
#pragma unroll
    for (int c = 0; c < kChunk; ++c) {
      const int o = base + c;                      // compile-time: facc stays in registers
      if (o < NT * TM) {
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][c * 4 + r][lane] = facc[o / TM][o % TM][r];
      }
    }
    __syncthreads();
    const int o = base + wave;
    if (wave < kChunk && o < NT * TM) {
      const int j = o / TM, t = o - j * TM;
      float s[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < W; ++w) v += red[w][wave * 4 + r][lane];
        s[r] = v;
      }
      if (p.S > 1) {
        float* f = frag(slice, o);
        store_shared_f2(f, s[0], s[1]);
        store_shared_f2(f + 2, s[2], s[3]);
      } else {
        const int m = 16 * t + r16;
        if (j < nt_valid && m < Mloc) {
          uint2 out;
          out.x = (uint32_t)float_to_half_bits(s[0]) | ((uint32_t)float_to_half_bits(s[1]) << 16);
          out.y = (uint32_t)float_to_half_bits(s[2]) | ((uint32_t)float_to_half_bits(s[3]) << 16);
          *reinterpret_cast<uint2*>(yloc + (size_t)m * p.N + (T0 + j) * 16 + 4 * kb) = out;
        }
      }
    }
  }
  if (p.S == 1) return;
  if (!last_arrival(p.tickets, p.S, (unsigned)tb, &ticket)) return;
  for (int o = wave; o < NT * TM; o += W) {
    const int j = o / TM, t = o - j * TM;
    float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int c = 0; c < p.S; ++c) {            // fixed order: the result does not depend on who came last
      const float* f = frag(c, o);
      const float2 a = load_shared_f2(f), b = load_shared_f2(f + 2);
      s[0] += a.x; s[1] += a.y; s[2] += b.x; s[3] += b.y;
    }
    const int m = 16 * t + r16;
    if (j < nt_valid && m < Mloc) {
      uint2 out;
      out.x = (uint32_t)float_to_half_bits(s[0]) | ((uint32_t)float_to_half_bits(s[1]) << 16);
      out.y = (uint32_t)float_to_half_bits(s[2]) | ((uint32_t)float_to_half_bits(s[3]) << 16);
      *reinterpret_cast<uint2*>(yloc + (size_t)m * p.N + (T0 + j) * 16 + 4 * kb) = out;
    }
  }
}

}  // namespace qspec
