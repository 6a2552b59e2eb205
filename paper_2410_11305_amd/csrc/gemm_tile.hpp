// Tiled (large-M) kernels for both modes of the shared-weight linear layer.
//
// A workgroup of WGN x WGM wavefronts owns a BN x BM block of the output
// (BN = 16*TN*WGN output features, BM = 16*TMW*WGM tokens) over a range of K
// groups; a wavefront owns TN x TMW MFMA tiles of 16 x 16.  Per K group
//   - the activation block (BM tokens x 128 k) is copied global -> registers
//     -> LDS once per workgroup, double buffered, one barrier per group;
//   - every wavefront fetches the weight tiles of its own TN n-tiles straight
//     from global memory into registers in MFMA operand layout (one 16-byte
//     load per lane and tile), through a ring of kTileRing groups.
// MFMA operand roles: A = weights (row = n % 16), B = activations (column =
// m % 16), k-block = lane / 16; D: lane holds rows 4*(lane/16)+r, column
// lane % 16, i.e. four consecutive output features of one token.
//
// Verify mode (W4A16): the codes are turned into fp16 weights code*scale in
// registers (the run-time dequantisation to fp16 the paper describes, Sec. 1
// item (1)) and accumulated on v_mfma_f32_16x16x32_f16 in fp32 over all of K.
// Draft mode (W4A4): both operands are int8 = 16*code; one K group is two
// v_mfma_i32_16x16x64_i8 into a fresh int32 tile, which is converted and
// scaled by sa[m,g]*sw[n,g]*2^-8 into the fp32 accumulator.
//
// With S > 1 K-slices the workgroups of one output block write fp32 partial
// blocks to the workspace; the one that arrives last (an atomic ticket per
// output block) adds the S slices and stores fp16.  Nobody waits for anybody.
#pragma once
#include "buffer.hpp"
#include "common.hpp"

#include <type_traits>

namespace qspec {

constexpr int kTileRing = 3;      // K groups of weight tiles in flight per wavefront (at most 4)

struct TileArgs {
  const uint4* codes;        // blob code tiles
  const uint16_t* scalesT;   // blob fp16 scales [G][N]
  const void* act;           // W4A4: qa bytes [M][K/2]; W4A16: x fp16 [M][K]
  const float* sa;           // W4A4: [M][G]
  uint16_t* y;               // fp16 [M][N]
  float* ws;                 // S > 1: fp32 [S][M][N] partial sums
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

template <bool W4A4, int TN, int TMW, int WGN, int WGM>
struct TileCfg {
  static constexpr int kThreads = 64 * WGN * WGM;
  static constexpr int BN = 16 * TN * WGN;
  static constexpr int BM = 16 * TMW * WGM;
  // LDS bytes per token row and group: fp16 x (256) or int8 operands, low-nibble and high-nibble halves (64 + 64)
  static constexpr int kRowBytes = W4A4 ? 128 : 256;
  static constexpr int kActBytes = BM * kRowBytes;
  static constexpr int kStageBytes = kActBytes + (W4A4 ? BM * 4 : 0);   // + sa[m] of the group
  static constexpr int kChunksPerRow = W4A4 ? 4 : 16;                   // 16-byte global pieces per row and group
  static constexpr int kChunks = BM * kChunksPerRow;
  static constexpr int U = (kChunks + kThreads - 1) / kThreads;         // pieces a thread stages per group
  static constexpr int kLdsBytes = 2 * kStageBytes;
};

// One word (8 codes) -> 8 fp16 weights code*scale (s2 = the row's scale, twice).
__device__ inline v8h dequant_word_scaled(uint32_t w, v2h s2) {
  const uint32_t w8 = w >> 8;
  const uint32_t b0 = (w & 0x000F000Fu) ^ 0x64086408u;
  const uint32_t b1 = (w & 0x00F000F0u) ^ 0x64806480u;
  const uint32_t b2 = (w8 & 0x000F000Fu) ^ 0x64086408u;
  const uint32_t b3 = (w8 & 0x00F000F0u) ^ 0x64806480u;
  const v2h k1032 = {(_Float16)1032.0f, (_Float16)1032.0f};
  const v2h k72 = {(_Float16)72.0f, (_Float16)72.0f};
  const v2h k16th = {(_Float16)0.0625f, (_Float16)0.0625f};
  // the integer code is recovered exactly first; the product with the scale is the only rounding
  const v2h h0 = (__builtin_bit_cast(v2h, b0) - k1032) * s2;
  const v2h h1 = (__builtin_bit_cast(v2h, b1) * k16th - k72) * s2;
  const v2h h2 = (__builtin_bit_cast(v2h, b2) - k1032) * s2;
  const v2h h3 = (__builtin_bit_cast(v2h, b3) * k16th - k72) * s2;
  return v8h{h0.x, h0.y, h1.x, h1.y, h2.x, h2.y, h3.x, h3.y};
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

// Output of a wave's TN x TMW tiles (first n-tile T0, first token row mrow0).
// S == 1: fp16 stores.  S > 1: publish this K-slice, take a ticket, the workgroup
// that arrives last adds the slices up in slice order.
template <int TN, int TMW>
__device__ __forceinline__ void tile_store(const TileArgs& p, const TileCoord& tc, float (&acc)[TN][TMW][4], int T0, int mrow0) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int r16 = lane & 15, kb = lane >> 4;
  const int tilesN = p.N >> 4;
  // ---- output
  if (p.S == 1) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if (T0 + j >= tilesN) continue;
#pragma unroll
      for (int t = 0; t < TMW; ++t) {
        const int m = mrow0 + 16 * t + r16;
        if (m >= p.M) continue;
        uint2 out;
        out.x = (uint32_t)float_to_half_bits(acc[j][t][0]) | ((uint32_t)float_to_half_bits(acc[j][t][1]) << 16);
        out.y = (uint32_t)float_to_half_bits(acc[j][t][2]) | ((uint32_t)float_to_half_bits(acc[j][t][3]) << 16);
        *reinterpret_cast<uint2*>(p.y + (size_t)m * p.N + (T0 + j) * 16 + 4 * kb) = out;
      }
    }
    return;
  }

  // ---- S > 1: publish this tc.slice, take a ticket, the last arrival adds up
  const size_t slice_elems = (size_t)p.M * p.N;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    if (T0 + j >= tilesN) continue;
#pragma unroll
    for (int t = 0; t < TMW; ++t) {
      const int m = mrow0 + 16 * t + r16;
      if (m >= p.M) continue;
      *reinterpret_cast<float4*>(p.ws + tc.slice * slice_elems + (size_t)m * p.N + (T0 + j) * 16 + 4 * kb) =
          float4{acc[j][t][0], acc[j][t][1], acc[j][t][2], acc[j][t][3]};
    }
  }
  __threadfence();                      // this thread's partial sums are visible device-wide ...
  __syncthreads();                      // ... for every thread of the workgroup, before the ticket is taken
  __shared__ unsigned ticket;
  if (tid == 0) {
    const unsigned blk = (unsigned)(tc.nblk * p.mb + tc.mblk);
    const unsigned old = atomicAdd(&p.tickets[blk], 1u);
    if (old == (unsigned)p.S - 1) atomicExch(&p.tickets[blk], 0u);   // nobody else touches it any more in this launch
    ticket = old;
  }
  __syncthreads();
  if (ticket != (unsigned)p.S - 1) return;
  __threadfence();                      // the other tc.slices' stores are visible to the loads below
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    if (T0 + j >= tilesN) continue;
#pragma unroll
    for (int t = 0; t < TMW; ++t) {
      const int m = mrow0 + 16 * t + r16;
      if (m >= p.M) continue;
      const size_t o = (size_t)m * p.N + (T0 + j) * 16 + 4 * kb;
      // fixed order 0 .. S-1 whoever arrives last (its own slice is read back like the
      // others): the result does not depend on timing
      float4 s = {0.0f, 0.0f, 0.0f, 0.0f};
      for (int c = 0; c < p.S; ++c) {
        const float4 v = *reinterpret_cast<const float4*>(p.ws + c * slice_elems + o);
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
      }
      uint2 out;
      out.x = (uint32_t)float_to_half_bits(s.x) | ((uint32_t)float_to_half_bits(s.y) << 16);
      out.y = (uint32_t)float_to_half_bits(s.z) | ((uint32_t)float_to_half_bits(s.w) << 16);
      *reinterpret_cast<uint2*>(p.y + o) = out;
    }
  }
}

template <bool W4A4, int TN, int TMW, int WGN, int WGM, int OCC>
__global__ __launch_bounds__(64 * WGN * WGM, OCC) void gemm_tile_kernel(TileArgs p) {
  using C = TileCfg<W4A4, TN, TMW, WGN, WGM>;
  constexpr int NW = kTileRing;
  static_assert(!W4A4 || C::BM <= C::kThreads, "one thread per token row stages the activation scales");
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wn = wave % WGN, wm = wave / WGN;
  const int r16 = lane & 15, kb = lane >> 4;
  const int G = p.G;

  const TileCoord tc = tile_coord(p);
  const int nblk = tc.nblk, mblk = tc.mblk, g0 = tc.g0, g1 = tc.g1;
  const int tilesN = p.N >> 4;
  const int T0 = nblk * (TN * WGN) + wn * TN;      // first n-tile of this wave
  const int m0 = mblk * C::BM;                     // first token row of the workgroup
  const int mw0 = wm * (TMW * 16);                 // first row of this wave inside the block

  const rsrc_t r_codes = make_rsrc(p.codes, (uint32_t)((size_t)p.N * p.K / 2));
  const rsrc_t r_scales = make_rsrc(p.scalesT, (uint32_t)((size_t)p.N * G * 2));
  const rsrc_t r_act = make_rsrc(p.act, (uint32_t)(W4A4 ? (size_t)p.M * p.K / 2 : (size_t)p.M * p.K * 2));
  const rsrc_t r_sa = make_rsrc(W4A4 ? (const void*)p.sa : p.act, (uint32_t)((size_t)p.M * G * 4));

  // ---- staging of the activation block (global -> registers -> LDS)
  uint4 xs[C::U];
  float sas = 0.0f;
  // Work that does not exist is expressed in the load offset (bit 31 set = out of
  // range = zeros, no traffic), computed with plain arithmetic: a select between two
  // offsets tempts the compiler into a branch around two different load instructions.
  auto past_end = [&](int g) -> uint32_t { return (uint32_t)((g1 - 1 - g) >> 31) << 31; };   // g >= g1 ? bit 31 : 0
  static_assert(C::kChunks % C::kThreads == 0, "every thread stages the same number of pieces");
  auto load_x = [&](int g) {
    const uint32_t gone = past_end(g);
#pragma unroll
    for (int u = 0; u < C::U; ++u) {
      const int idx = tid + u * C::kThreads;
      const int row = idx / C::kChunksPerRow, c = idx % C::kChunksPerRow;
      const uint32_t m = (uint32_t)(m0 + row);      // rows past M lie past the end of the buffer: zeros
      const uint32_t off = W4A4 ? m * (uint32_t)(p.K / 2) + (uint32_t)g * 64u + c * 16u
                                : (m * (uint32_t)p.K + (uint32_t)g * kGroup) * 2u + c * 16u;
      xs[u] = buf_load16(r_act, off | gone);
    }
    if (W4A4) {
      const uint32_t idle = (uint32_t)((C::BM - 1 - tid) >> 31) << 31;                      // tid >= BM
      sas = buf_load_f32(r_sa, (((uint32_t)(m0 + tid) * G + g) * 4u) | gone | idle);
    }
  };
  auto store_x = [&](int stage) {
    uint8_t* base = lds + stage * C::kStageBytes;
#pragma unroll
    for (int u = 0; u < C::U; ++u) {
      const int idx = tid + u * C::kThreads;
      const int row = idx / C::kChunksPerRow, c = idx % C::kChunksPerRow;
      {
        if (W4A4) {
          // widen to int8 = 16*code once per workgroup; 8 slots of 16 bytes per row
          // (slot kb: low nibbles, slot 4+kb: high nibbles), slot index xor-ed with
          // (row/2)%8 so that 16 rows at one slot hit 16 different bank groups
          const I8Pair q = unpack_i8(xs[u]);
          const int sw = (row >> 1) & 7;
          *reinterpret_cast<v4i*>(base + row * 128 + ((c ^ sw) << 4)) = q.lo;
          *reinterpret_cast<v4i*>(base + row * 128 + (((c + 4) ^ sw) << 4)) = q.hi;
        } else {
          // 16 slots of 16 bytes per row, slot index xor-ed with row%16
          *reinterpret_cast<uint4*>(base + row * 256 + ((c ^ (row & 15)) << 4)) = xs[u];
        }
      }
    }
    if (W4A4 && tid < C::BM) *reinterpret_cast<float*>(base + C::kActBytes + tid * 4) = sas;
  };

  // ---- weight tiles of this wave: a ring of NW groups in registers.  Slot d holds
  // group g with (g - g0) % NW == d; it is refilled for group g + NW as soon as its
  // last word has been consumed, so a fetch has NW - 1 group times to arrive.  (The
  // slots are named statically - the group loop below is unrolled NW times - because
  // moving a register whose load is still in flight would wait for that load.)
  uint4 wq[NW][TN];
  uint32_t sq[NW][TN][2];       // raw scales: W4A16 one fp16 (row r16), W4A4 four fp16 (rows 4kb..4kb+3)
  uint32_t no_tile[TN];          // bit 31 set for an n-tile past N
#pragma unroll
  for (int j = 0; j < TN; ++j) no_tile[j] = (uint32_t)((tilesN - 1 - (T0 + j)) >> 31) << 31;
  auto load_w = [&](uint4 (&w)[TN], uint32_t (&s)[TN][2], int g) {
    const uint32_t gone = past_end(g);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const uint32_t T = (uint32_t)(T0 + j);
      const uint32_t skip = gone | no_tile[j];
      w[j] = buf_load16(r_codes, ((T * G + g) * 1024u + lane * 16u) | skip);
      if (W4A4) {
        const uint2 v = buf_load8(r_scales, (((uint32_t)g * p.N + T * 16u + 4u * kb) * 2u) | skip);
        s[j][0] = v.x; s[j][1] = v.y;
      } else {
        s[j][0] = buf_load_u16(r_scales, (((uint32_t)g * p.N + T * 16u + r16) * 2u) | skip);
        s[j][1] = 0;
      }
    }
  };

  float acc[TN][TMW][4];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int t = 0; t < TMW; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[j][t][r] = 0.0f;

  load_x(g0);
#pragma unroll
  for (int d = 0; d < NW; ++d) load_w(wq[d], sq[d], g0 + d);
  store_x(0);
  __syncthreads();

  // verify mode: fp16 scales of the current group's tiles, and its first k-step
  // already dequantised
  v2h s2[TN], s2n[TN], wa0[TN][4];
  if (!W4A4) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const _Float16 sc = __builtin_bit_cast(_Float16, (uint16_t)sq[0][j][0]);
      s2[j] = v2h{sc, sc};
      s2n[j] = s2[j];
#pragma unroll
      for (int h = 0; h < 4; ++h) wa0[j][h] = dequant_pair_scaled(word_of(wq[0][j], 0), h, s2[j]);
    }
  }

  // One K group.  SLOT is the ring slot of group g (a compile-time constant).
  auto group_body = [&](auto slot_c, int g) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_c)::value;
    const int stage = (g - g0) & 1;
    const uint8_t* xl = lds + stage * C::kStageBytes;
    load_x(g + 1);                             // lands in LDS at the end of this group
    __builtin_amdgcn_sched_barrier(0);         // keep these loads ahead of the ring refill below

    if (W4A4) {
      I8Pair a[TN];
      float swf[TN][4];
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        a[j] = unpack_i8(wq[SLOT][j]);
        // both int8 operands carry a factor 16: fold 2^-8 into the weight scale (exact)
        swf[j][0] = half_bits_to_float((uint16_t)(sq[SLOT][j][0] & 0xFFFF)) * 0.00390625f;
        swf[j][1] = half_bits_to_float((uint16_t)(sq[SLOT][j][0] >> 16)) * 0.00390625f;
        swf[j][2] = half_bits_to_float((uint16_t)(sq[SLOT][j][1] & 0xFFFF)) * 0.00390625f;
        swf[j][3] = half_bits_to_float((uint16_t)(sq[SLOT][j][1] >> 16)) * 0.00390625f;
      }
      load_w(wq[SLOT], sq[SLOT], g + NW);      // the slot's words are in a[] and swf[] now
      // operands of token tile t, fetched one tile ahead of the MFMAs that use them
      v4i blo[2], bhi[2];
      float sam[2];
      auto read_tile = [&](int t, int b) {
        const int row = mw0 + 16 * t + r16;
        const int sw = (row >> 1) & 7;
        blo[b] = *reinterpret_cast<const v4i*>(xl + row * 128 + ((kb ^ sw) << 4));
        bhi[b] = *reinterpret_cast<const v4i*>(xl + row * 128 + (((kb + 4) ^ sw) << 4));
        sam[b] = *reinterpret_cast<const float*>(xl + C::kActBytes + row * 4);
      };
      read_tile(0, 0);
#pragma unroll
      for (int t = 0; t < TMW; ++t) {
        if (t + 1 < TMW) read_tile(t + 1, (t + 1) & 1);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          v4i pa = {0, 0, 0, 0};
          pa = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[j].lo, blo[t & 1], pa, 0, 0, 0);
          pa = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[j].hi, bhi[t & 1], pa, 0, 0, 0);
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[j][t][r] += (float)pa[r] * (sam[t & 1] * swf[j][r]);
        }
      }
    } else {
      // Order of issue, pinned with scheduling fences because the compiler's own
      // order leaves every LDS read next to its first use:
      //   unit u (one k-step of BT token tiles) = the BT LDS reads of unit u+1, then
      //   the TN*BT MFMAs of unit u with the dequantisation of the NEXT k-step cut
      //   into pieces (one fp16 pair = 3 VALU ops) and spread between them.
      // The first k-step of a group is dequantised during the last k-step of the
      // group before (wa0 is carried from body to body).
      constexpr int BT = TMW >= 4 ? 4 : TMW;
      constexpr int NB = TMW / BT;                 // units per k-step
      constexpr int Q = TN * TMW;                  // MFMAs per k-step
      constexpr int P = 4 * TN;                    // dequantisation pieces per k-step
      constexpr int EVERY = Q / P > 0 ? Q / P : 1; // MFMAs between two pieces
      constexpr int PER = P / (Q / EVERY) > 0 ? P / (Q / EVERY) : 1;   // pieces per slot
      static_assert(TMW % BT == 0, "token tiles per wave must be a multiple of the unit");
      static_assert((Q / EVERY) * PER >= P, "all pieces of a k-step fit between its MFMAs");
      constexpr int NEXT = (SLOT + 1) % NW;
      uint4 xb[2][BT];
      auto read_unit = [&](int u, uint4 (&dst)[BT]) {
        const int i = u / NB, tb = u % NB;
#pragma unroll
        for (int t = 0; t < BT; ++t) {
          const int row = mw0 + 16 * (tb * BT + t) + r16;
          dst[t] = *reinterpret_cast<const uint4*>(xl + row * 256 + (((4 * i + kb) ^ r16) << 4));
        }
      };
      read_unit(0, xb[0]);
      __builtin_amdgcn_sched_barrier(0);
      v2h wa[2][TN][4];                            // k-step i lives in wa[i & 1]
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int h = 0; h < 4; ++h) wa[0][j][h] = wa0[j][h];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int q = 0; q < Q; ++q) {
          const int t = q / TN, j = q % TN;        // token tile, n-tile
          const int u = i * NB + t / BT;
          if (q % (BT * TN) == 0) {                // first MFMA of a unit: fetch the next unit's operands
            if (u + 1 < 4 * NB) read_unit(u + 1, xb[(u + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
          }
          {
            const v8h av = v8h{wa[i & 1][j][0].x, wa[i & 1][j][0].y, wa[i & 1][j][1].x, wa[i & 1][j][1].y,
                               wa[i & 1][j][2].x, wa[i & 1][j][2].y, wa[i & 1][j][3].x, wa[i & 1][j][3].y};
            const v8h xv = __builtin_bit_cast(v8h, xb[u & 1][t % BT]);
            v4f d = {acc[j][t][0], acc[j][t][1], acc[j][t][2], acc[j][t][3]};
            d = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, xv, d, 0, 0, 0);
            acc[j][t][0] = d[0]; acc[j][t][1] = d[1]; acc[j][t][2] = d[2]; acc[j][t][3] = d[3];
          }
          if ((q + 1) % EVERY == 0) {
#pragma unroll
            for (int e = 0; e < PER; ++e) {
              const int pp = ((q + 1) / EVERY - 1) * PER + e;     // piece of the next k-step
              if (pp < P) {
                const int jj = pp / 4, h = pp % 4;
                if (i < 3) {
                  wa[(i + 1) & 1][jj][h] = dequant_pair_scaled(word_of(wq[SLOT][jj], i + 1), h, s2[jj]);
                } else {
                  wa0[jj][h] = dequant_pair_scaled(word_of(wq[NEXT][jj], 0), h, s2n[jj]);
                }
              }
            }
            if (i == 2 && q + 1 == Q) {
              // every word of this slot is in registers as fp16 now: refill it, and
              // turn the next slot's scales (fetched NW-1 groups ago) into fp16 pairs
              load_w(wq[SLOT], sq[SLOT], g + NW);
#pragma unroll
              for (int jn = 0; jn < TN; ++jn) {
                const _Float16 sn = __builtin_bit_cast(_Float16, (uint16_t)sq[NEXT][jn][0]);
                s2n[jn] = v2h{sn, sn};
              }
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) s2[j] = s2n[j];
    }

    store_x(stage ^ 1);                        // zeros after the last group
    __syncthreads();
  };

  // Straight-line body of NW groups (no branch around a group: the compiler's
  // wait-count bookkeeping stays exact only without control flow).  Groups past
  // the end of the slice run on zeros: their loads are out of range.
  for (int g = g0; g < g1; g += NW) {
    group_body(std::integral_constant<int, 0>{}, g);
    if constexpr (NW > 1) group_body(std::integral_constant<int, 1 % NW>{}, g + 1);
    if constexpr (NW > 2) group_body(std::integral_constant<int, 2 % NW>{}, g + 2);
    if constexpr (NW > 3) group_body(std::integral_constant<int, 3 % NW>{}, g + 3);
  }

  tile_store<TN, TMW>(p, tc, acc, T0, m0 + mw0);
}

}  // namespace qspec
