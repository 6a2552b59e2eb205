// Shared pieces of the tiled (M > 32) kernels of both modes: launch arguments,
// the workgroup -> output block mapping, the int4 -> fp16 pair dequantiser, and
// the exchange of K-slice partial sums between workgroups.
//
// With S > 1 K-slices the S workgroups of one output block write their fp32
// accumulators to the workspace; the one that arrives last (an atomic ticket per
// output block) adds the S slices in slice order and stores fp16.  Nobody waits
// for anybody, so no workgroup needs another one to be resident.
#pragma once
#include "buffer.hpp"
#include "common.hpp"
#include "exchange.hpp"

#include <type_traits>

namespace qspec {

struct TileArgs {
  const uint4* codes;        // blob code tiles
  const uint16_t* scalesT;   // blob fp16 scales [G][N]
  const void* act;           // W4A4: qa bytes [M][K/2]; W4A16: x fp16 [M][K]
  const float* sa;           // W4A4: [M][G]
  uint16_t* y;               // fp16 [M][N]
  float* ws;                 // S > 1: fp32 partial sums, [S][output block][accumulator fragment]
  unsigned* tickets;         // S > 1: one counter per output block, zero on entry, zero on exit
  int M, N, K, G;
  int S;                     // K-slices
  int nb, mb;                // output blocks along N and along M
};

// Which output block and K-slice a workgroup owns.  Workgroup ids are dealt
// round-robin to the 8 XCDs (each with its own L2): ids with the same id % 8 are
// renumbered to be neighbours, so that the blocks sharing a weight stripe (same
// n-block, all m-blocks and K-slices) run on one XCD and fetch it from HBM once.
struct TileCoord { int nblk, mblk, slice, g0, g1; };

__device__ __forceinline__ TileCoord tile_coord(const TileArgs& p) {
  const int total = p.nb * p.mb * p.S;
  int logical = blockIdx.x;
  const int per = total >> 3;                   // ids per XCD in the part that divides evenly
  if ((int)blockIdx.x < per * 8) logical = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
  TileCoord c;
  c.nblk = logical / (p.mb * p.S);
  const int rem = logical - c.nblk * (p.mb * p.S);
  c.mblk = rem / p.S;
  c.slice = rem - c.mblk * p.S;
  c.g0 = (int)(((long long)c.slice * p.G) / p.S);
  c.g1 = (int)(((long long)(c.slice + 1) * p.G) / p.S);
  return c;
}

// Pair h (0..3) of a word: codes (c_2h, c_2h+1) -> fp16 weights code*scale.
__device__ inline v2h dequant_pair_scaled(uint32_t w, int h, v2h s2) {
  const uint32_t v = h < 2 ? w : w >> 8;
  if ((h & 1) == 0) {
    const uint32_t b = (v & 0x000F000Fu) ^ 0x64086408u;           // 1024 + (code + 8)
    const v2h k1032 = {(_Float16)1032.0f, (_Float16)1032.0f};
    return (__builtin_bit_cast(v2h, b) - k1032) * s2;
  }
  const uint32_t b = (v & 0x00F000F0u) ^ 0x64806480u;             // 1024 + 16 * (code + 8)
  const v2h k72 = {(_Float16)72.0f, (_Float16)72.0f};
  const v2h k16th = {(_Float16)0.0625f, (_Float16)0.0625f};
  return (__builtin_bit_cast(v2h, b) * k16th - k72) * s2;
}

__device__ inline uint32_t word_of(const uint4& q, int i) {
  return i == 0 ? q.x : i == 1 ? q.y : i == 2 ? q.z : q.w;
}

// The partial sums of K-slice c of output block blk: the workgroup's accumulator
// registers in register-pair-major, thread-minor order (pair q of thread t at float
// 2*(q*threads + t)), so that every wave-wide store or load is one contiguous run
// of 512 bytes whatever the MFMA register layout is.
__device__ __forceinline__ float* slice_frag(const TileArgs& p, int c, unsigned blk, int floats_per_block) {
  return p.ws + ((size_t)c * (p.nb * p.mb) + blk) * (size_t)floats_per_block;
}
// fp16 store of a wave's PN x PM accumulator tiles of 32 x 32 (first output feature n0,
// first token row mrow0).  Two MFMA D layouts (h = lane / 32; a, r = 0..3; register 4a + r):
//   LANE_IS_TOKEN   lane holds token m = lane % 32 and features 8a + 4h + r: four runs of
//                   four consecutive output features of one token (8-byte stores);
//   !LANE_IS_TOKEN  lane holds feature n = lane % 32 and tokens 8a + 4h + r: per register
//                   the 32 lanes of a half write 64 contiguous bytes of one token row.
template <int PN, int PM, bool LANE_IS_TOKEN>
__device__ __forceinline__ void tile_write_fp16(const TileArgs& p, const float (&acc)[PN][PM][16], int n0, int mrow0) {
  const int lane = threadIdx.x & 63;
  const int l32 = lane & 31, h = lane >> 5;
#pragma unroll
  for (int j = 0; j < PN; ++j)
#pragma unroll
    for (int t = 0; t < PM; ++t) {
      if (LANE_IS_TOKEN) {
        const int m = mrow0 + 32 * t + l32;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          const int n = n0 + 32 * j + 8 * a + 4 * h;
          if (m < p.M && n < p.N) {
            uint2 out;
            out.x = (uint32_t)float_to_half_bits(acc[j][t][4 * a + 0]) | ((uint32_t)float_to_half_bits(acc[j][t][4 * a + 1]) << 16);
            out.y = (uint32_t)float_to_half_bits(acc[j][t][4 * a + 2]) | ((uint32_t)float_to_half_bits(acc[j][t][4 * a + 3]) << 16);
            *reinterpret_cast<uint2*>(p.y + (size_t)m * p.N + n) = out;
          }
        }
      } else {
        const int n = n0 + 32 * j + l32;
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int m = mrow0 + 32 * t + 8 * a + 4 * h + r;
            if (m < p.M && n < p.N) p.y[(size_t)m * p.N + n] = float_to_half_bits(acc[j][t][4 * a + r]);
          }
      }
    }
}

// Output of a wave's PN x PM tiles of 32 x 32.  S == 1: fp16 stores.  S > 1: see the
// head of this file.
template <int PN, int PM, bool LANE_IS_TOKEN = true>
__device__ __forceinline__ void tile_store32(const TileArgs& p, const TileCoord& tc, float (&acc)[PN][PM][16],
                                             int n0, int mrow0) {
  const int tid = threadIdx.x;
  if (p.S == 1) {
    tile_write_fp16<PN, PM, LANE_IS_TOKEN>(p, acc, n0, mrow0);
    return;
  }
  const unsigned blk = (unsigned)(tc.nblk * p.mb + tc.mblk);
  const int nthr = blockDim.x;
  constexpr int kAcc = PN * PM * 16;
  float* mine = slice_frag(p, tc.slice, blk, nthr * kAcc);
#pragma unroll
  for (int j = 0; j < PN; ++j)
#pragma unroll
    for (int t = 0; t < PM; ++t)
#pragma unroll
      for (int e = 0; e < 8; ++e)
        store_shared_f2(mine + 2 * (((j * PM + t) * 8 + e) * nthr + tid), acc[j][t][2 * e], acc[j][t][2 * e + 1]);
  __shared__ unsigned ticket32;
  if (!last_arrival(p.tickets, p.S, blk, &ticket32)) return;
  // Add the slices in the fixed order 0 .. S-1 whoever arrives last (its own slice is
  // read back like the others), so the result does not depend on timing.  The loads
  // bypass the caches and each costs a trip to memory: sixteen are kept in flight.
#pragma unroll
  for (int j = 0; j < PN; ++j)
#pragma unroll
    for (int t = 0; t < PM; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][t][r] = 0.0f;
  for (int c = 0; c < p.S; ++c) {
    const float* f = slice_frag(p, c, blk, nthr * kAcc);
#pragma unroll
    for (int j = 0; j < PN; ++j)
#pragma unroll
      for (int tp = 0; tp < PM; tp += 2) {          // two tiles = 16 loads in flight at a time
        float2 v[2][8];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int e = 0; e < 8; ++e) v[t][e] = load_shared_f2(f + 2 * (((j * PM + tp + t) * 8 + e) * nthr + tid));
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int e = 0; e < 8; ++e) { acc[j][tp + t][2 * e] += v[t][e].x; acc[j][tp + t][2 * e + 1] += v[t][e].y; }
      }
  }
  tile_write_fp16<PN, PM, LANE_IS_TOKEN>(p, acc, n0, mrow0);
}

}  // namespace qspec
