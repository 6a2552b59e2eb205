// Tiled verify-mode (W4A16) kernel for M > 32: in-register int4 -> fp16
// dequantisation feeding v_mfma_f32_32x32x16_f16 (paper Sec. 1 item (1): the
// 4-bit weights are dequantised to fp16 at run time; Sec. 4.1: groups of 128).
//
// A workgroup of WGN x WGM wavefronts owns BN x BM outputs (BN = 32*PN*WGN
// features, BM = 32*PM*WGM tokens) over a range of K groups; a wavefront owns
// PN x PM MFMA tiles of 32 x 32.
//   - Activations: the BM x 128 fp16 block of a group travels global -> LDS
//     with buffer loads that write LDS directly (no registers, no ds_write),
//     NS-1 groups ahead, into NS stages that are separate arrays (the compiler
//     then knows that a transfer into one never aliases a read of another
//     and inserts no wait between them).  A wave-wide transfer fills 1 KB of
//     LDS linearly (lane l -> bytes 16l..16l+15) = four token rows; the
//     16-byte slot s of row r holds k-chunk s ^ (r % 16), chosen on the
//     global-address side, so that the 16 rows a quarter-wave reads fall into
//     16 different bank groups.
//   - Weights: every wavefront fetches the code tiles of its own rows straight
//     into registers in MFMA operand layout through a ring of NW groups and
//     dequantises them itself.
//   - Order of issue inside a group is pinned with scheduling fences: the LDS
//     reads of a later k-step first, then the MFMAs of this k-step with the
//     dequantisation of the NEXT k-step cut into pieces (one fp16 pair = 3
//     VALU ops) between them.  Left to itself the compiler puts every LDS
//     read next to its first use.
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
#pragma once
#include "tile_common.hpp"

namespace qspec {

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// s_waitcnt immediate for "at most n vector-memory operations outstanding",
// leaving the other counters alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4, lgkmcnt 11:8).
constexpr int waitcnt_vm(int n) { return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4) | (0xF << 8); }
// the same with lgkmcnt(0): every LDS (and scalar-memory) operation of the wave has completed too
constexpr int waitcnt_vm_lgkm0(int n) { return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4); }
#ifndef QSPEC_TILE16_EARLY
#define QSPEC_TILE16_EARLY 1
#endif

template <int PN, int PM, int WGN, int WGM, int NW, int NS, int OCC>
__global__ __launch_bounds__(64 * WGN * WGM, OCC) void gemm_tile16w_kernel(TileArgs p) {
  constexpr int kWaves = WGN * WGM;
  constexpr int BM = 32 * PM * WGM;
  constexpr int kStageBytes = BM * 256;
  constexpr int U = kStageBytes / 1024 / kWaves;       // wave-wide transfers per wave and group
  static_assert(kStageBytes % (1024 * kWaves) == 0, "the stage divides evenly among the waves");
  static_assert(NW == 2 || NW == 4, "the stage of a group must follow from its ring slot");
  static_assert(NS == 2 || (NS == 4 && NW == 4), "stage = ring slot % NS");
  constexpr int D = NS - 1;                            // activations are fetched D groups ahead
  static_assert(kWaves == 4 || kWaves == 8, "row % 16 of a transfer must not depend on u");
  // NS stages, each an array of its own (see the head of this file)
  __shared__ __attribute__((aligned(1024))) uint8_t xs0[kStageBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t xs1[kStageBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t xs2[NS > 2 ? kStageBytes : 16];
  __shared__ __attribute__((aligned(1024))) uint8_t xs3[NS > 2 ? kStageBytes : 16];
  auto stage_ptr = [&](int i) -> uint8_t* { return i == 0 ? xs0 : i == 1 ? xs1 : i == 2 ? xs2 : xs3; };

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wn = wave % WGN, wm = wave / WGN;
  const int m32 = lane & 31, h = lane >> 5;
  const int G = p.G;
  const TileCoord tc = tile_coord(p);
  const int g0 = tc.g0, g1 = tc.g1;
  const int n0 = (tc.nblk * (PN * WGN) + wn * PN) * 32;      // first output feature of this wave
  const int m0 = tc.mblk * BM;
  const int mw0 = wm * (PM * 32);

  const rsrc_t r_codes = make_rsrc(p.codes, (uint32_t)((size_t)p.N * p.K / 2));
  const rsrc_t r_scales = make_rsrc(p.scalesT, (uint32_t)((size_t)p.N * G * 2));
  const rsrc_t r_act = make_rsrc(p.act, (uint32_t)((size_t)p.M * p.K * 2));
  // Every workgroup walks its K groups in the same order, q = 0 .. ng-1 -> group g0 + q:
  // the workgroups of an XCD then need the same narrow window of activation columns at
  // about the same time and find it in their L2.  (Starting each weight stripe at a
  // different group was measured: no faster, and 9x the algorithmic bytes fetched,
  // because the whole activation matrix then has to live in a 4 MB L2.)
  const int ng = g1 - g0;
  auto group_of = [&](int q) -> int { return g0 + q; };
  auto past_end = [&](int q) -> uint32_t { return (uint32_t)((ng - 1 - q) >> 31) << 31; };   // q >= ng ? bit 31 : 0

  // ---- activations: global -> LDS.  Transfer u of this wave fills block q = wave +
  // u*kWaves (1 KB = rows 4q..4q+3).  Lane l writes slot l%16 of row 4q + l/16 and so
  // must fetch k-chunk (l%16) ^ (row%16); row%16 = (4*wave + l/16) % 16 for every u
  // because 4*kWaves*u is a multiple of 16.  Rows past M lie past the end of the
  // buffer.
  const int row_in_blk = 4 * wave + (lane >> 4);
  const uint32_t x_voff = (uint32_t)(m0 + row_in_blk) * (uint32_t)p.K * 2u +
                          (uint32_t)(((lane & 15) ^ (row_in_blk & 15)) << 4);
  const uint32_t x_ustep = (uint32_t)(4 * kWaves) * (uint32_t)p.K * 2u;
  auto dma_x = [&](int q, uint8_t* stage) {
    const uint32_t gbase = (uint32_t)group_of(q) * 256u;
    const uint32_t gone = past_end(q);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // (the marker is OR-ed in last: a sum could carry out of bit 31 for rows near 2 GiB)
      const uint32_t off = (x_voff + (gbase + (uint32_t)u * x_ustep)) | gone;
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
  auto load_w = [&](int d, int q) {
    const uint32_t gone = past_end(q);
    const int g = group_of(q);
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

  // All stages start as zeros: a stage that no transfer ever fills (a slice shorter
  // than the pipeline) or rows past M must not hold whatever an earlier kernel left
  // in LDS, because 0 * NaN would poison the accumulators.
#pragma unroll
  for (int o = tid * 16; o < kStageBytes; o += 64 * kWaves * 16) {
    *reinterpret_cast<uint4*>(xs0 + o) = uint4{0u, 0u, 0u, 0u};
    *reinterpret_cast<uint4*>(xs1 + o) = uint4{0u, 0u, 0u, 0u};
    if (NS > 2) {
      *reinterpret_cast<uint4*>(xs2 + o) = uint4{0u, 0u, 0u, 0u};
      *reinterpret_cast<uint4*>(xs3 + o) = uint4{0u, 0u, 0u, 0u};
    }
  }
  __syncthreads();
#pragma unroll
  for (int d = 0; d < D; ++d) dma_x(d, stage_ptr(d));
#pragma unroll
  for (int d = 0; d < NW; ++d) load_w(d, d);

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

  // LDS reads run XB-1 k-steps ahead of the MFMAs that consume them: a k-step of a
  // small wave tile is too short (PN*PM*32 cycles) to cover the LDS latency alone.
  // EARLY (wave tiles of four or more MFMAs per k-step, reads one step ahead): the barrier
  // that ends a group stands in front of its LAST k-step instead of behind it.  By then a
  // wave has issued every LDS read of the group, so the barrier certifies what the one at
  // the end did (everyone is done with this stage, everyone's transfers of the next stage
  // have landed), and the first operands of the next group are read under the last
  // k-step's MFMAs: no wave starts a group by waiting for LDS with nothing to issue.
  constexpr bool EARLY = QSPEC_TILE16_EARLY && PN * PM >= 4;
  constexpr int XB = EARLY ? 2 : (PN * PM >= 8 ? 2 : (PN * PM >= 4 ? 3 : 4));
  uint4 xb[XB][PM];
  auto read_step_from = [&](const uint8_t* xl, int s, uint4 (&dst)[PM]) {
    const int c = 4 * (s >> 1) + 2 * (s & 1) + h;      // this lane's k-chunk of step s
#pragma unroll
    for (int t = 0; t < PM; ++t) {
      const int row = mw0 + 32 * t + m32;
      dst[t] = *reinterpret_cast<const uint4*>(xl + row * 256 + ((c ^ (row & 15)) << 4));
    }
  };
  if constexpr (EARLY) read_step_from(xs0, 0, xb[0]);      // group 0, k-step 0

  auto group_body = [&](auto slot_c, int g) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_c)::value;
    constexpr int NEXT = (SLOT + 1) % NW;
    const uint8_t* xl = stage_ptr(SLOT % NS);
    const uint8_t* xl_next = stage_ptr((SLOT + 1) % NS);
    uint8_t* xnext = stage_ptr((SLOT + D) % NS);   // last read in the group before this one
    auto read_step = [&](int s, uint4 (&dst)[PM]) { read_step_from(xl, s, dst); };
    auto word_of_step = [&](int d, int j, int s) -> uint32_t {
      const uint4& q = (s & 1) ? whi[d][j] : wlo[d][j];
      return word_of(q, s >> 1);
    };
    if constexpr (!EARLY) {
#pragma unroll
      for (int s = 0; s < XB - 1; ++s) read_step(s, xb[s]);
    }
    __builtin_amdgcn_sched_barrier(0);
    v2h wa[2][PN][4];                            // k-step s lives in wa[s & 1]
#pragma unroll
    for (int j = 0; j < PN; ++j)
#pragma unroll
      for (int hh = 0; hh < 4; ++hh) wa[0][j][hh] = wa0[j][hh];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      if (s + XB - 1 < 8) read_step(s + XB - 1, xb[(s + XB - 1) % XB]);
      if constexpr (EARLY) {
        if (s == 7) {
          // (the count as at the end of the group: the ring refill of k-step 6 is the youngest
          // load; lgkmcnt(0): this wave's reads of the stage have completed, not only issued)
          __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((D - 1) * (U + 3 * PN) + 3 * PN));
          __builtin_amdgcn_s_barrier();
          read_step_from(xl_next, 0, xb[0]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (s == 1) {
        // every wave has passed the barrier that ended the last group reading that
        // stage; issued here rather than at the top so that the first MFMAs of the
        // group do not queue behind the address computations
        dma_x(g + D, xnext);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int q = 0; q < Q; ++q) {
        const int t = q / PN, j = q % PN;
        {
          const v8h av = v8h{wa[s & 1][j][0].x, wa[s & 1][j][0].y, wa[s & 1][j][1].x, wa[s & 1][j][1].y,
                             wa[s & 1][j][2].x, wa[s & 1][j][2].y, wa[s & 1][j][3].x, wa[s & 1][j][3].y};
          const v8h xv = __builtin_bit_cast(v8h, xb[s % XB][t]);
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
    // The next group's activations were requested D-1 groups ago, before D-1 further
    // batches of U transfers and D batches of 3*PN ring loads.  Loads complete in
    // order: at most that many outstanding means those activations have landed.  (No
    // store may sit between them - stores complete out of order with loads - so this
    // kernel must compile without register spills in the loop.)
    if constexpr (!EARLY) {
      __builtin_amdgcn_s_waitcnt(waitcnt_vm((D - 1) * (U + 3 * PN) + 3 * PN));
      __builtin_amdgcn_s_barrier();
    }
  };

  for (int q = 0; q < ng; q += NW) {
    group_body(std::integral_constant<int, 0>{}, q);
    group_body(std::integral_constant<int, 1>{}, q + 1);
    if constexpr (NW > 2) group_body(std::integral_constant<int, 2 % NW>{}, q + 2);
    if constexpr (NW > 2) group_body(std::integral_constant<int, 3 % NW>{}, q + 3);
  }

  tile_store32<PN, PM>(p, tc, acc, n0, m0 + mw0);
}

}  // namespace qspec
