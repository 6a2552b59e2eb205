// Tiled verify-mode (W4A16) kernel for M > 32: in-register int4 -> fp16
// dequantisation feeding v_mfma_f32_16x16x32_f16 (paper Sec. 1 item (1): the
// 4-bit weights are dequantised to fp16 at run time; Sec. 4.1: groups of 128).
//
// A workgroup of WGN x WGM wavefronts owns BN x BM outputs (BN = 16*TN*WGN
// features, BM = 16*TMW*WGM tokens) over a range of K groups.
//   - Activations: the BM x 128 fp16 block of a group travels global -> LDS
//     with buffer loads that write LDS directly (no registers, no ds_write),
//     one group ahead, into two stages that are separate arrays (the compiler
//     then knows that a transfer into one never aliases a read of the other
//     and inserts no wait between them).  A wave-wide transfer fills 1 KB of
//     LDS linearly (lane l -> bytes 16l..16l+15) = four token rows; the
//     16-byte slot s of row r holds k-chunk s ^ (r % 16), chosen on the
//     global-address side, so that the 16 rows an MFMA operand read touches
//     fall into 16 different bank groups.
//   - Weights: every wavefront fetches the 16 x 128 code tiles of its own TN
//     n-tiles straight into registers in MFMA operand layout (one 16-byte
//     load per lane and tile) through a ring of NW groups, and dequantises
//     them itself.
//   - Order of issue inside a group is pinned with scheduling fences: the LDS
//     reads of unit u+1 (one k-step of BT token tiles), then the TN*BT MFMAs
//     of unit u with the dequantisation of the NEXT k-step cut into pieces
//     (one fp16 pair = 3 VALU ops) between them.  Left to itself the compiler
//     puts every LDS read next to its first use.
// MFMA operand roles: A = weights (row = n % 16), B = activations (column =
// m % 16), k-block = lane / 16; D: lane holds rows 4*(lane/16)+r, column
// lane % 16.
#pragma once
#include "gemm_tile.hpp"

namespace qspec {

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// s_waitcnt immediate for "at most n vector-memory operations outstanding",
// leaving the other counters alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4, lgkmcnt 11:8).
constexpr int waitcnt_vm(int n) { return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4) | (0xF << 8); }

template <int TN, int TMW, int WGN, int WGM, int NW, int OCC>
__global__ __launch_bounds__(64 * WGN * WGM, OCC) void gemm_tile16_kernel(TileArgs p) {
  constexpr int kWaves = WGN * WGM;
  constexpr int BM = 16 * TMW * WGM;
  constexpr int kStageBytes = BM * 256;
  constexpr int U = kStageBytes / 1024 / kWaves;       // wave-wide transfers per wave and group
  static_assert(kStageBytes % (1024 * kWaves) == 0, "the stage divides evenly among the waves");
  static_assert(NW == 2 || NW == 4, "the stage of a group must follow from its ring slot");
  static_assert(kWaves == 4 || kWaves == 8 || kWaves == 2 || kWaves == 1, "row % 16 of a transfer must not depend on u");
  __shared__ __attribute__((aligned(1024))) uint8_t xs0[kStageBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t xs1[kStageBytes];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wn = wave % WGN, wm = wave / WGN;
  const int r16 = lane & 15, kb = lane >> 4;
  const int G = p.G;
  const TileCoord tc = tile_coord(p);
  const int g0 = tc.g0, g1 = tc.g1;
  const int tilesN = p.N >> 4;
  const int T0 = tc.nblk * (TN * WGN) + wn * TN;
  const int m0 = tc.mblk * BM;
  const int mw0 = wm * (TMW * 16);

  const rsrc_t r_codes = make_rsrc(p.codes, (uint32_t)((size_t)p.N * p.K / 2));
  const rsrc_t r_scales = make_rsrc(p.scalesT, (uint32_t)((size_t)p.N * G * 2));
  const rsrc_t r_act = make_rsrc(p.act, (uint32_t)((size_t)p.M * p.K * 2));

  // Work that does not exist gets bit 31 in its load offset (out of range: zeros,
  // no traffic), by arithmetic rather than by a select the compiler could turn
  // into a branch around two load instructions.
  auto past_end = [&](int g) -> uint32_t { return (uint32_t)((g1 - 1 - g) >> 31) << 31; };

  // ---- activations: global -> LDS.  Transfer u of this wave fills block q = wave +
  // u*kWaves (1 KB = rows 4q..4q+3).  Lane l writes slot l%16 of row 4q + l/16 and so
  // must fetch k-chunk (l%16) ^ (row%16); row%16 = (4*wave + l/16) % 16 for every u
  // when kWaves is 4 or 8 (then 4*kWaves*u is a multiple of 16).
  const int row_in_blk = 4 * wave + (lane >> 4);
  const uint32_t x_voff = (uint32_t)(m0 + row_in_blk) * (uint32_t)p.K * 2u +
                          (uint32_t)(((lane & 15) ^ (row_in_blk & 15)) << 4);   // rows past M: out of range
  const uint32_t x_ustep = (uint32_t)(4 * kWaves) * (uint32_t)p.K * 2u;         // bytes between transfers u, u+1
  auto dma_x = [&](int g, uint8_t* stage) {
    const uint32_t gbase = (uint32_t)g * 256u + past_end(g);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t off = x_voff + (gbase + (uint32_t)u * x_ustep);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r_act, (lds_ptr_t)(stage + (wave + u * kWaves) * 1024), 16, off, 0, 0, 0);
    }
  };

  // ---- weights: ring of NW groups, slot d holds group g with (g - g0) % NW == d
  uint4 wq[NW][TN];
  uint32_t sq[NW][TN];           // fp16 scale of row r16 of each tile
  uint32_t no_tile[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) no_tile[j] = (uint32_t)((tilesN - 1 - (T0 + j)) >> 31) << 31;
  auto load_w = [&](uint4 (&w)[TN], uint32_t (&s)[TN], int g) {
    const uint32_t gone = past_end(g);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const uint32_t T = (uint32_t)(T0 + j);
      const uint32_t skip = gone | no_tile[j];
      w[j] = buf_load16(r_codes, ((T * G + g) * 1024u + lane * 16u) | skip);
      s[j] = buf_load_u16(r_scales, (((uint32_t)g * p.N + T * 16u + r16) * 2u) | skip);
    }
  };

  float acc[TN][TMW][4];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int t = 0; t < TMW; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[j][t][r] = 0.0f;

  // Both stages start as zeros: a stage that no transfer ever fills (a slice of one
  // group) or rows past M must not hold whatever an earlier kernel left in LDS,
  // because 0 * NaN would poison the accumulators.
#pragma unroll
  for (int o = tid * 16; o < kStageBytes; o += 64 * kWaves * 16) {
    *reinterpret_cast<uint4*>(xs0 + o) = uint4{0u, 0u, 0u, 0u};
    *reinterpret_cast<uint4*>(xs1 + o) = uint4{0u, 0u, 0u, 0u};
  }
  __syncthreads();
  dma_x(g0, xs0);
#pragma unroll
  for (int d = 0; d < NW; ++d) load_w(wq[d], sq[d], g0 + d);

  // fp16 scale pairs of the current group, and its first k-step already dequantised
  v2h s2[TN], s2n[TN], wa0[TN][4];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const _Float16 sc = __builtin_bit_cast(_Float16, (uint16_t)sq[0][j]);
    s2[j] = v2h{sc, sc};
    s2n[j] = s2[j];
#pragma unroll
    for (int h = 0; h < 4; ++h) wa0[j][h] = dequant_pair_scaled(word_of(wq[0][j], 0), h, s2[j]);
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
  __builtin_amdgcn_s_barrier();

  constexpr int BT = TN >= 4 ? 2 : (TMW >= 4 ? 4 : TMW);   // token tiles per unit
  constexpr int NB = TMW / BT;                 // units per k-step
  constexpr int Q = TN * TMW;                  // MFMAs per k-step
  constexpr int P = 4 * TN;                    // dequantisation pieces per k-step
  constexpr int EVERY = Q / P > 0 ? Q / P : 1; // MFMAs between two pieces
  constexpr int PER = (P * EVERY + Q - 1) / Q; // pieces per slot
  static_assert(TMW % BT == 0, "token tiles per wave must be a multiple of the unit");
  static_assert((Q / EVERY) * PER >= P, "all pieces of a k-step fit between its MFMAs");

  auto group_body = [&](auto slot_c, int g) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_c)::value;
    constexpr int NEXT = (SLOT + 1) % NW;
    const uint8_t* xl = (SLOT & 1) ? xs1 : xs0;
    uint8_t* xnext = (SLOT & 1) ? xs0 : xs1;
    // the other stage was last read in the group before this one, and every wave
    // has passed the barrier that ended it
    dma_x(g + 1, xnext);
    __builtin_amdgcn_sched_barrier(0);

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
            // every word of this slot is in registers as fp16 now: refill it, and turn
            // the next slot's scales (fetched NW-1 groups ago) into fp16 pairs
            load_w(wq[SLOT], sq[SLOT], g + NW);
#pragma unroll
            for (int jn = 0; jn < TN; ++jn) {
              const _Float16 sn = __builtin_bit_cast(_Float16, (uint16_t)sq[NEXT][jn]);
              s2n[jn] = v2h{sn, sn};
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) s2[j] = s2n[j];
    // The transfers of the next group's activations were issued before this
    // group's 2*TN ring loads, and memory operations complete in order: at most
    // 2*TN outstanding means they have landed.  Every LDS read of this group has
    // returned (its MFMAs are behind us), so after the barrier the stage just read
    // may be overwritten.
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(2 * TN));
    __builtin_amdgcn_s_barrier();
  };

  // Straight-line body of NW groups (no branch around a group: the compiler's
  // wait-count bookkeeping stays exact only without control flow).  Groups past
  // the end of the slice run on zero weights: their loads are out of range.
  for (int g = g0; g < g1; g += NW) {
    group_body(std::integral_constant<int, 0>{}, g);
    group_body(std::integral_constant<int, 1>{}, g + 1);
    if constexpr (NW > 2) group_body(std::integral_constant<int, 2 % NW>{}, g + 2);
    if constexpr (NW > 2) group_body(std::integral_constant<int, 3 % NW>{}, g + 3);
  }

  tile_store<TN, TMW>(p, tc, acc, T0, m0 + mw0);
}

// ---------------------------------------------------------------------------
// The same kernel on v_mfma_f32_32x32x16_f16: half as many matrix instructions
// for the same arithmetic (a wavefront issues them at a better rate) and half
// the dequantised-operand registers.  A wavefront owns PN x PM tiles of 32 x 32.
//
// A operand (32 rows x 16 k): lane l supplies 8 consecutive k of row l % 32,
// lanes 0..31 the first 8 k of the step, lanes 32..63 the second 8.  In the blob
// the 16 bytes of tile lane (r, kb) are words i = 0..3 holding k-chunks (8 k each)
// 4i + kb.  So lane l = (h = l / 32, row = l % 32) fetches, from the 16-row tile
// that holds its row, the 16 bytes of tile lane (row % 16, h) ["lo"] and of tile
// lane (row % 16, h + 2) ["hi"]: word i of lo is chunk 4i + h, word i of hi is
// chunk 4i + 2 + h, and step s = 2i + e (e = 0: lo, 1: hi) covers the 16
// consecutive k = 32i + 16e .. +15.  The B operand of that step is, for lane
// (h, m = l % 32), chunk 4i + 2e + h of token row m.
// D: lane holds column m = l % 32 and rows 8a + 4h + r (a, r = 0..3) in
// register 4a + r: four runs of four consecutive output features.
template <int PN, int PM>
__device__ __forceinline__ void tile_store32(const TileArgs& p, const TileCoord& tc, float (&acc)[PN][PM][16],
                                             int n0, int mrow0) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int m32 = lane & 31, h = lane >> 5;
  if (p.S == 1) {
#pragma unroll
    for (int j = 0; j < PN; ++j)
#pragma unroll
      for (int t = 0; t < PM; ++t) {
        const int m = mrow0 + 32 * t + m32;
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
      }
    return;
  }
  const size_t slice_elems = (size_t)p.M * p.N;
#pragma unroll
  for (int j = 0; j < PN; ++j)
#pragma unroll
    for (int t = 0; t < PM; ++t) {
      const int m = mrow0 + 32 * t + m32;
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const int n = n0 + 32 * j + 8 * a + 4 * h;
        if (m < p.M && n < p.N)
          *reinterpret_cast<float4*>(p.ws + tc.slice * slice_elems + (size_t)m * p.N + n) =
              float4{acc[j][t][4 * a + 0], acc[j][t][4 * a + 1], acc[j][t][4 * a + 2], acc[j][t][4 * a + 3]};
      }
    }
  __threadfence();                      // this thread's partial sums are visible device-wide ...
  __syncthreads();                      // ... for every thread of the workgroup, before the ticket is taken
  __shared__ unsigned ticket32;
  if (tid == 0) {
    const unsigned blk = (unsigned)(tc.nblk * p.mb + tc.mblk);
    const unsigned old = atomicAdd(&p.tickets[blk], 1u);
    if (old == (unsigned)p.S - 1) atomicExch(&p.tickets[blk], 0u);   // nobody else touches it any more in this launch
    ticket32 = old;
  }
  __syncthreads();
  if (ticket32 != (unsigned)p.S - 1) return;
  __threadfence();                      // the other slices' stores are visible to the loads below
#pragma unroll
  for (int j = 0; j < PN; ++j)
#pragma unroll
    for (int t = 0; t < PM; ++t) {
      const int m = mrow0 + 32 * t + m32;
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const int n = n0 + 32 * j + 8 * a + 4 * h;
        if (m < p.M && n < p.N) {
          const size_t o = (size_t)m * p.N + n;
          float4 s = {0.0f, 0.0f, 0.0f, 0.0f};
          for (int c = 0; c < p.S; ++c) {       // fixed order: the result does not depend on who came last
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
}

template <int PN, int PM, int WGN, int WGM, int NW, int OCC>
__global__ __launch_bounds__(64 * WGN * WGM, OCC) void gemm_tile16w_kernel(TileArgs p) {
  constexpr int kWaves = WGN * WGM;
  constexpr int BM = 32 * PM * WGM;
  constexpr int kStageBytes = BM * 256;
  constexpr int U = kStageBytes / 1024 / kWaves;       // wave-wide transfers per wave and group
  static_assert(kStageBytes % (1024 * kWaves) == 0, "the stage divides evenly among the waves");
  static_assert(NW == 2 || NW == 4, "the stage of a group must follow from its ring slot");
  static_assert(kWaves == 4 || kWaves == 8, "row % 16 of a transfer must not depend on u");
  __shared__ __attribute__((aligned(1024))) uint8_t xs0[kStageBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t xs1[kStageBytes];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wn = wave % WGN, wm = wave / WGN;
  const int m32 = lane & 31, h = lane >> 5;
  const int G = p.G;
  const TileCoord tc = tile_coord(p);
  const int g0 = tc.g0, g1 = tc.g1;
  const int tilesN = p.N >> 4;
  const int n0 = (tc.nblk * (PN * WGN) + wn * PN) * 32;      // first output feature of this wave
  const int m0 = tc.mblk * BM;
  const int mw0 = wm * (PM * 32);

  const rsrc_t r_codes = make_rsrc(p.codes, (uint32_t)((size_t)p.N * p.K / 2));
  const rsrc_t r_scales = make_rsrc(p.scalesT, (uint32_t)((size_t)p.N * G * 2));
  const rsrc_t r_act = make_rsrc(p.act, (uint32_t)((size_t)p.M * p.K * 2));
  auto past_end = [&](int g) -> uint32_t { return (uint32_t)((g1 - 1 - g) >> 31) << 31; };

  // ---- activations: global -> LDS, as in gemm_tile16_kernel
  const int row_in_blk = 4 * wave + (lane >> 4);
  const uint32_t x_voff = (uint32_t)(m0 + row_in_blk) * (uint32_t)p.K * 2u +
                          (uint32_t)(((lane & 15) ^ (row_in_blk & 15)) << 4);
  const uint32_t x_ustep = (uint32_t)(4 * kWaves) * (uint32_t)p.K * 2u;
  auto dma_x = [&](int g, uint8_t* stage) {
    const uint32_t gbase = (uint32_t)g * 256u + past_end(g);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t off = x_voff + (gbase + (uint32_t)u * x_ustep);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r_act, (lds_ptr_t)(stage + (wave + u * kWaves) * 1024), 16, off, 0, 0, 0);
    }
  };

  // ---- weights: per 32-row pair two 16-byte pieces (lo, hi) and the row's scale
  uint4 wlo[NW][PN], whi[NW][PN];
  uint32_t sq[NW][PN];
  // per-lane offsets of pair 0 inside a group (bit 31: the lane's tile lies past N;
  // then so do the tiles of the pairs after it, and pair j adds a wave-uniform step)
  const int n_lane = n0 + m32;          // this lane's weight row in pair 0
  const uint32_t w_voff = (uint32_t)(n_lane >> 4) * G * 1024u + (uint32_t)((n_lane & 15) + 16 * h) * 16u;
  auto load_w = [&](int d, int g) {
    const uint32_t gone = past_end(g);
#pragma unroll
    for (int j = 0; j < PN; ++j) {
      const uint32_t none = (uint32_t)((p.N - 1 - (n_lane + 32 * j)) >> 31) << 31;
      const uint32_t skip = gone | none;
      const uint32_t wo = w_voff + (uint32_t)(2 * j) * G * 1024u + (uint32_t)g * 1024u;
      wlo[d][j] = buf_load16(r_codes, wo | skip);
      whi[d][j] = buf_load16(r_codes, (wo + 512u) | skip);
      sq[d][j] = buf_load_u16(r_scales, (((uint32_t)g * (uint32_t)p.N + (uint32_t)(n_lane + 32 * j)) * 2u) | skip);
    }
  };

  float acc[PN][PM][16];
#pragma unroll
  for (int j = 0; j < PN; ++j)
#pragma unroll
    for (int t = 0; t < PM; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][t][r] = 0.0f;

  // both stages start as zeros (see gemm_tile16_kernel)
#pragma unroll
  for (int o = tid * 16; o < kStageBytes; o += 64 * kWaves * 16) {
    *reinterpret_cast<uint4*>(xs0 + o) = uint4{0u, 0u, 0u, 0u};
    *reinterpret_cast<uint4*>(xs1 + o) = uint4{0u, 0u, 0u, 0u};
  }
  __syncthreads();
  dma_x(g0, xs0);
#pragma unroll
  for (int d = 0; d < NW; ++d) load_w(d, g0 + d);

  v2h s2[PN], s2n[PN], wa0[PN][4];
#pragma unroll
  for (int j = 0; j < PN; ++j) {
    const _Float16 sc = __builtin_bit_cast(_Float16, (uint16_t)sq[0][j]);
    s2[j] = v2h{sc, sc};
    s2n[j] = s2[j];
#pragma unroll
    for (int hh = 0; hh < 4; ++hh) wa0[j][hh] = dequant_pair_scaled(wlo[0][j].x, hh, s2[j]);
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
  __builtin_amdgcn_s_barrier();

  constexpr int Q = PN * PM;                   // MFMAs per k-step (16 k), one LDS read feeds PN of them
  constexpr int P = 4 * PN;                    // dequantisation pieces per k-step
  static_assert(Q >= P / 2, "at most two pieces between MFMAs");
  constexpr int PER = (P + Q - 1) / Q;         // pieces after each MFMA

  auto group_body = [&](auto slot_c, int g) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_c)::value;
    constexpr int NEXT = (SLOT + 1) % NW;
    const uint8_t* xl = (SLOT & 1) ? xs1 : xs0;
    uint8_t* xnext = (SLOT & 1) ? xs0 : xs1;
    uint4 xb[2][PM];
    auto read_step = [&](int s, uint4 (&dst)[PM]) {
      const int c = 4 * (s >> 1) + 2 * (s & 1) + h;      // this lane's k-chunk of step s
#pragma unroll
      for (int t = 0; t < PM; ++t) {
        const int row = mw0 + 32 * t + m32;
        dst[t] = *reinterpret_cast<const uint4*>(xl + row * 256 + ((c ^ (row & 15)) << 4));
      }
    };
    auto word_of_step = [&](int d, int j, int s) -> uint32_t {
      const uint4& q = (s & 1) ? whi[d][j] : wlo[d][j];
      return word_of(q, s >> 1);
    };
    read_step(0, xb[0]);
    __builtin_amdgcn_sched_barrier(0);
    v2h wa[2][PN][4];                            // k-step s lives in wa[s & 1]
#pragma unroll
    for (int j = 0; j < PN; ++j)
#pragma unroll
      for (int hh = 0; hh < 4; ++hh) wa[0][j][hh] = wa0[j][hh];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      if (s + 1 < 8) read_step(s + 1, xb[(s + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);
      if (s == 1) {
        // the other stage was last read in the group before this one and every wave has
        // passed the barrier that ended it; issued here rather than at the top so that
        // the first MFMAs of the group do not queue behind eight address computations
        dma_x(g + 1, xnext);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int q = 0; q < Q; ++q) {
        const int t = q / PN, j = q % PN;
        {
          const v8h av = v8h{wa[s & 1][j][0].x, wa[s & 1][j][0].y, wa[s & 1][j][1].x, wa[s & 1][j][1].y,
                             wa[s & 1][j][2].x, wa[s & 1][j][2].y, wa[s & 1][j][3].x, wa[s & 1][j][3].y};
          const v8h xv = __builtin_bit_cast(v8h, xb[s & 1][t]);
          v16f d;
#pragma unroll
          for (int r = 0; r < 16; ++r) d[r] = acc[j][t][r];
          d = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, xv, d, 0, 0, 0);
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[j][t][r] = d[r];
        }
#pragma unroll
        for (int e = 0; e < PER; ++e) {
          const int pp = q * PER + e;            // piece of the next k-step
          if (pp < P) {
            const int jj = pp / 4, hh = pp % 4;
            if (s < 7) wa[(s + 1) & 1][jj][hh] = dequant_pair_scaled(word_of_step(SLOT, jj, s + 1), hh, s2[jj]);
            else wa0[jj][hh] = dequant_pair_scaled(wlo[NEXT][jj].x, hh, s2n[jj]);
          }
        }
        if (s == 6 && q + 1 == Q) {
          // every word of this slot is in registers as fp16 now: refill it, and turn the
          // next slot's scales (fetched NW-1 groups ago) into fp16 pairs
          load_w(SLOT, g + NW);
#pragma unroll
          for (int jn = 0; jn < PN; ++jn) {
            const _Float16 sn = __builtin_bit_cast(_Float16, (uint16_t)sq[NEXT][jn]);
            s2n[jn] = v2h{sn, sn};
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int j = 0; j < PN; ++j) s2[j] = s2n[j];
    // Activation transfers were issued before this group's 3*PN ring loads, and loads
    // complete in order: at most 3*PN outstanding means they have landed.  (No store
    // may sit between them: stores complete out of order with loads, so this kernel
    // must compile without register spills.)
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(3 * PN));
    __builtin_amdgcn_s_barrier();
  };

  for (int g = g0; g < g1; g += NW) {
    group_body(std::integral_constant<int, 0>{}, g);
    group_body(std::integral_constant<int, 1>{}, g + 1);
    if constexpr (NW > 2) group_body(std::integral_constant<int, 2 % NW>{}, g + 2);
    if constexpr (NW > 2) group_body(std::integral_constant<int, 3 % NW>{}, g + 3);
  }

  tile_store32<PN, PM>(p, tc, acc, n0, m0 + mw0);
}

}  // namespace qspec
