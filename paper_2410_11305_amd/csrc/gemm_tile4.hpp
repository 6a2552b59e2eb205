// Tiled draft-mode (W4A4) kernel for M > 64 on v_mfma_i32_32x32x32_i8 (paper
// Sec. 1 item (2): both operands stay 4-bit integers on the low-precision matrix
// units; Sec. 4.1: groups of 128).
//
// Per K group and 32 x 32 output tile: four MFMAs (32 k each) into a fresh int32
// tile P (exact), then  acc += float(P) * (sa[m,g] * 2^-8) * sw[n,g]  in fp32.
// Both int8 operands are 16*code (a nibble moved to the high half of a byte), so
// P is 256 times the true partial sum and 2^-8 rides on the activation scale.
// With g = 128 that rescaling, not the matrix unit, bounds the kernel (one fp32
// operation per output and group costs as many cycles as the MFMAs of that
// group), so the kernel is built around doing it in TWO vector instructions per
// output and group and nothing else per output:
//   - MFMA roles: A = activations, B = weights.  A lane's 16 accumulator registers
//     are then 16 tokens of ONE output feature, so the weight scale is one value
//     per lane and group (one conversion, one multiply) instead of sixteen.
//   - The int32 -> fp32 conversion is folded away: the MFMA chain of a tile starts
//     from a register set holding the bit pattern of 1.5 * 2^23, so the finished
//     register READ AS A FLOAT is 12582912 + 256 P exactly (|256 P| <= 2^21), and
//     t = fma(that, sw, -12582912 * sw) is the correctly rounded 256 P * sw (the
//     constant is exact: sw has 11 significant bits, 1.5 * 2^23 two).
//   - acc = fma(t, sa[token], acc): the sixteen token scales of a tile sit in ONE
//     register (lane i of each row of 16 lanes holds the scale of the token that
//     accumulator register i belongs to) and reach the multiply through the DPP
//     row-broadcast operand of v_fmac_f32: no register per token, no move.
//   - The rescaling of a tile runs under the MFMAs of the next tile, the one of a
//     group's last tile under the first MFMAs of the next group.
//
// A workgroup of WGN x WGM wavefronts owns BN x BM outputs (BN = 32*PN*WGN,
// BM = 32*PM*WGM) over a range of K groups.
//   - Activations: the BM x 64 B code block of a group and its BM scales go global
//     -> registers three groups ahead, are widened to int8 once per workgroup and
//     written to one of three LDS stages two groups ahead, at the TOP of a group (the
//     writes land under that group's arithmetic); one barrier per group.  Row layout: 8 slots of 16 bytes (slot kb: low nibbles of k-block kb,
//     slot 4+kb: high nibbles), slot index xor-ed with act_swizzle(row) so that the
//     operand reads and the staging writes are free of bank conflicts.
//     With the quantiser's widened format (WIDE: one int8 = 16 * code per code, 128 bytes
//     per row and group in exactly this row layout) the rows go global -> LDS by loads
//     that write LDS directly, two groups ahead: no widening, no staging registers.
//   - Weights and their scales: straight into registers in MFMA operand layout
//     through a ring of three groups (slots named statically: the group loop is
//     unrolled three times, which also fixes the LDS stage of a group).
//
// B operand (32 k x 32 features): lane l = (h = l / 32, col = l % 32) supplies 16 k
// of its weight row.  It fetches the 16 bytes of blob tile lane (col % 16, kb = h)
// ["lo"] and (col % 16, kb = h + 2) ["hi"] of the 16-row tile holding its row; each
// gives two operands (low nibbles, high nibbles), four MFMA steps in all.  The A
// operand of a step is, for lane (h, m = l % 32), the matching slot of token row m:
// kb = h or h + 2, low or high nibbles.  Any assignment of k to steps and lanes is
// valid as long as both operands use the same one: a group's dot product is
// order-free.  D: lane holds output feature n = l % 32 and tokens 8a + 4h + r
// (a, r = 0..3) in register 4a + r.
#pragma once
#include "gemm_tile16.hpp"

namespace qspec {

typedef int v16i __attribute__((ext_vector_type(16)));

// acc += S[lane R of this lane's row of 16] * t  in one instruction: v_fmac_f32 whose
// first operand comes through the DPP row broadcast.  (The compiler does not fold a DPP
// move into the multiply-add by itself; written out, it is one VALU operation.)  S must
// not have been written by a vector ALU instruction in the two instructions before.
template <int R>
__device__ __forceinline__ void fmac_row_bcast(float& acc, float S, float t) {
  asm volatile("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(S), "v"(t), "n"(R));
}
__device__ __forceinline__ void fmac_row_bcast_r(float& acc, float S, float t, int r) {   // r is a constant after unrolling
  switch (r) {
    case 0: fmac_row_bcast<0>(acc, S, t); break;
    case 1: fmac_row_bcast<1>(acc, S, t); break;
    case 2: fmac_row_bcast<2>(acc, S, t); break;
    case 3: fmac_row_bcast<3>(acc, S, t); break;
    case 4: fmac_row_bcast<4>(acc, S, t); break;
    case 5: fmac_row_bcast<5>(acc, S, t); break;
    case 6: fmac_row_bcast<6>(acc, S, t); break;
    case 7: fmac_row_bcast<7>(acc, S, t); break;
    case 8: fmac_row_bcast<8>(acc, S, t); break;
    case 9: fmac_row_bcast<9>(acc, S, t); break;
    case 10: fmac_row_bcast<10>(acc, S, t); break;
    case 11: fmac_row_bcast<11>(acc, S, t); break;
    case 12: fmac_row_bcast<12>(acc, S, t); break;
    case 13: fmac_row_bcast<13>(acc, S, t); break;
    case 14: fmac_row_bcast<14>(acc, S, t); break;
    default: fmac_row_bcast<15>(acc, S, t); break;
  }
}

// LDS slot swizzle of an activation row (8 slots of 16 bytes in a 128-byte row): slot s of
// row r is stored at slot s ^ act_swizzle(r).  Chosen so that a 16-byte access per lane is
// free of bank conflicts whether the LDS serves 8 lanes (128 B) or 16 lanes (256 B) per
// clock: 8 consecutive rows at one slot land in 8 different slots, and among 16
// consecutive rows the 8 of equal parity (which share the same half of a 256-byte window)
// do as well.
__device__ __forceinline__ int act_swizzle(int row) { return (row & 7) ^ ((row >> 3) & 1); }

template <int PN, int PM, int WGN, int WGM, int OCC, bool WIDE = false>
__global__ __launch_bounds__(64 * WGN * WGM, OCC) void gemm_tile4w_kernel(TileArgs p) {
  constexpr int kWaves = WGN * WGM;
  constexpr int kThreads = 64 * kWaves;
  constexpr int BM = 32 * PM * WGM;
  constexpr int NW = 3;                              // weight ring = LDS stages
  constexpr int kActBytes = BM * 128;
  constexpr int kChunks = BM * 4;                    // 16-byte pieces of codes per group
  constexpr int U = (kChunks + kThreads - 1) / kThreads;
  constexpr int kTiles = PN * PM;
  static_assert(kChunks % kThreads == 0 || kChunks < kThreads, "whole passes, or one partial pass");
  static_assert(BM <= kThreads, "one thread per token row stages the activation scale");
  static_assert(PM % 2 == 0 && kTiles % 2 == 0, "the last tile of a group and the first of the next use different int32 tiles");
  // three stages, each an array of its own: with the widened activation format the codes come
  // in by loads that write LDS directly, and the compiler then knows that a transfer into one
  // stage never feeds a read of another (no wait between them)
  // (and the token scales sa[m] * 2^-8 of a stage, written by ordinary LDS stores, sit in
  // arrays apart from the codes: a store into an array that a transfer is filling would wait
  // for that transfer)
  __shared__ __attribute__((aligned(1024))) uint8_t stage0[kActBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t stage1[kActBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t stage2[kActBytes];
  __shared__ float scale0[BM], scale1[BM], scale2[BM];
  auto stage_ptr = [&](int i) -> uint8_t* { return i == 0 ? stage0 : i == 1 ? stage1 : stage2; };
  auto scale_ptr = [&](int i) -> float* { return i == 0 ? scale0 : i == 1 ? scale1 : scale2; };

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wn = wave % WGN, wm = wave / WGN;
  const int l32 = lane & 31, h = lane >> 5;
  const int G = p.G;
  const TileCoord tc = tile_coord(p);
  const int g0 = tc.g0, g1 = tc.g1;
  const int ng = g1 - g0;
  const int n0 = (tc.nblk * (PN * WGN) + wn * PN) * 32;      // first output feature of this wave
  const int m0 = tc.mblk * BM;
  const int mw0 = wm * (PM * 32);

  const rsrc_t r_codes = make_rsrc(p.codes, (uint32_t)((size_t)p.N * p.K / 2));
  const rsrc_t r_scales = make_rsrc(p.scalesT, (uint32_t)((size_t)p.N * G * 2));
  const rsrc_t r_act = make_rsrc(p.act, (uint32_t)((size_t)p.M * p.K / (WIDE ? 1 : 2)));
  const rsrc_t r_sa = make_rsrc(p.sa, (uint32_t)((size_t)p.M * G * 4));
  // Work that does not exist gets bit 31 in its load offset (out of range: zeros, no
  // traffic), by arithmetic: a select between offsets tempts the compiler into a
  // branch around two load instructions, which ruins its wait-count bookkeeping.
  auto past_end = [&](int q) -> uint32_t { return (uint32_t)((ng - 1 - q) >> 31) << 31; };   // q >= ng ? bit 31 : 0

  // ---- activations: global -> registers (rows past M lie past the end of the buffer)
  uint4 xs[U];
  // The activation scales of a token row are consecutive in memory along the groups, and a
  // load of one scale per row touches one cache line per lane: three groups are fetched at
  // a time (groups 3k .. 3k+2 at the top of group 3k-3), a third of the line visits.
  float sas[NW] = {0.0f, 0.0f, 0.0f};
  const uint32_t idle_sa = (uint32_t)((BM - 1 - tid) >> 31) << 31;                 // tid >= BM
  auto load_sa3 = [&](int q) {                                                     // groups q, q+1, q+2 of this slice
    const float3_t v = buf_load_f32x3(r_sa, (((uint32_t)(m0 + tid) * G + (uint32_t)(g0 + q)) * 4u) | past_end(q) | idle_sa);
    sas[0] = v.x; sas[1] = v.y; sas[2] = v.z;
  };
  auto load_x = [&](int q) {
    const uint32_t gone = past_end(q);
    const int g = g0 + q;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = tid + u * kThreads;
      const int row = idx >> 2, c = idx & 3;
      const uint32_t idle = (uint32_t)((kChunks - 1 - idx) >> 31) << 31;           // idx >= kChunks
      xs[u] = buf_load16(r_act, ((uint32_t)(m0 + row) * (uint32_t)(p.K / 2) + (uint32_t)g * 64u + c * 16u) | gone | idle);
    }
  };
  auto store_x = [&](int stage) {                                                  // stage = (group index in the slice) % 3
    uint8_t* base = stage_ptr(stage);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = tid + u * kThreads;
      const int row = idx >> 2, c = idx & 3;
      if (kChunks % kThreads == 0 || idx < kChunks) {
        const I8Pair q = unpack_i8(xs[u]);
        const int sw = act_swizzle(row);
        // Four lanes write one row.  Rows whose bits 0 and 1 differ write their high-nibble
        // half first: the lanes that share a clock (two or four rows) then never meet in a bank.
        const bool hi_first = ((row ^ (row >> 1)) & 1) != 0;
        const int s0 = hi_first ? c + 4 : c, s1 = hi_first ? c : c + 4;
        *reinterpret_cast<v4i*>(base + row * 128 + ((s0 ^ sw) << 4)) = hi_first ? q.hi : q.lo;
        *reinterpret_cast<v4i*>(base + row * 128 + ((s1 ^ sw) << 4)) = hi_first ? q.lo : q.hi;
      }
    }
    if (tid < BM) scale_ptr(stage)[tid] = sas[stage] * 0.00390625f;   // 2^-8, exact
  };
  // ---- activations in the widened format (WIDE): a token row's group is 128 bytes of int8
  // in exactly the order of an LDS row, and goes global -> LDS without passing registers.
  // A wave-wide transfer fills 1 KB = rows 8t .. 8t+7 linearly; wave w issues transfers
  // t = w + u * kWaves.  Lane l writes slot l % 8 of row 8t + l / 8 and so must fetch slot
  // (l % 8) ^ act_swizzle(row); act_swizzle(8t + r) = r ^ (t & 1) and t & 1 = w & 1 for every u
  // because kWaves is even.  Rows past M lie past the end of the buffer (zeros or nothing:
  // their outputs are never stored).
  constexpr int kXfers = BM / 8;
  constexpr int UD = kXfers / kWaves;
  static_assert(!WIDE || (kXfers % kWaves == 0 && kWaves % 2 == 0), "whole transfers per wave; the swizzle of a transfer must not depend on u");
  const int drow = lane >> 3;
  const uint32_t xw_voff = (uint32_t)(m0 + 8 * wave + drow) * (uint32_t)p.K + (uint32_t)((((lane & 7) ^ drow ^ (wave & 1))) << 4);
  auto dma_x = [&](int q, uint8_t* stage) {
    const uint32_t gone = past_end(q);
    const uint32_t gbase = (uint32_t)(g0 + q) * 128u;
#pragma unroll
    for (int u = 0; u < UD; ++u) {
      const uint32_t off = (xw_voff + gbase + (uint32_t)(u * 8 * kWaves) * (uint32_t)p.K) | gone;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r_act, (lds_ptr_t)(stage + (wave + u * kWaves) * 1024), 16, off, 0, 0, 0);
    }
  };
  auto store_sa = [&](int stage) {
    if (tid < BM) scale_ptr(stage)[tid] = sas[stage] * 0.00390625f;
  };

  // ---- weights: ring of NW groups; per 32-row pair two 16-byte pieces and the scale
  // of this lane's row
  uint4 wlo[NW][PN], whi[NW][PN];
  uint32_t sq[NW][PN];
  const int n_lane = n0 + l32;          // this lane's weight row in pair 0
  const uint32_t w_voff = (uint32_t)(n_lane >> 4) * G * 1024u + (uint32_t)((n_lane & 15) + 16 * h) * 16u;
  auto load_w = [&](int d, int q) {
    const uint32_t gone = past_end(q);
    const int g = g0 + q;
#pragma unroll
    for (int j = 0; j < PN; ++j) {
      const uint32_t skip = gone | ((uint32_t)((p.N - 1 - (n_lane + 32 * j)) >> 31) << 31);
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

  // the start value of every int32 tile (see the head of this file), in a register set of
  // its own that the loop never rebuilds
  constexpr int kSeedBits = 0x4B400000;                // 12582912.0f = 1.5 * 2^23
  v16i seed;
#pragma unroll
  for (int r = 0; r < 16; ++r) seed[r] = kSeedBits;
  asm volatile("" : "+v"(seed));
  v16i P[2];                                           // int32 tiles, alternating
  P[0] = seed;
  P[1] = seed;
  // the rescaling still owed to the last tile of the group before (none yet: zeros)
  float pend_sw = 0.0f, pend_swc = 0.0f, pend_S = 0.0f;

  // t = 256 P sw (correctly rounded), acc += (sa 2^-8) t, for registers 4*part .. 4*part+3
  auto rescale_quarter = [&](const v16i& Pt, float sw, float swc, float S, float (&a)[16], int part) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 4 * part; r < 4 * part + 4; ++r) {
      const int bits = Pt[r];                          // (a copy: bit_cast of a vector element lvalue reads element 0)
      const float t = __builtin_fmaf(__builtin_bit_cast(float, bits), sw, swc);
      fmac_row_bcast_r(a[r], S, t, r);
    }
  };

  // this lane's entry of a token tile's scale register: lane i of a row of 16 holds the
  // scale of the token that accumulator register i belongs to (8 (i/4) + 4 h + i % 4)
  const int s_row = 8 * ((lane & 15) >> 2) + 4 * h + (lane & 3);

  // A operands: one register quad per MFMA step; the quad of step st is refilled with the
  // NEXT token tile's step st right after the MFMA that consumed it has been issued (a whole
  // tile ahead of its use, at half the registers of two complete operand sets)
  v4i a[4];
  float S[2];                                    // the sixteen token scales of tile t live in S[t & 1] (see s_row)
  auto read_operand = [&](const uint8_t* xl, int t, int st) {
    const int row = mw0 + 32 * t + l32;
    const int slot = (st == 0 ? h : st == 1 ? h + 4 : st == 2 ? h + 2 : h + 6) ^ act_swizzle(row);
    a[st] = *reinterpret_cast<const v4i*>(xl + row * 128 + (slot << 4));
  };
  auto read_scales = [&](const float* sl, int t, int buf) {
    S[buf] = sl[mw0 + 32 * t + s_row];
  };

  // prologue: groups 0 and 1 into stages 0 and 1, group 2 requested (it stays in registers
  // until the top of group 0), the weight ring filled, the first operands read
  load_sa3(0);
  if constexpr (WIDE) {
    dma_x(0, stage0);
    dma_x(1, stage1);
#pragma unroll
    for (int d = 0; d < NW; ++d) load_w(d, d);
    store_sa(0);
    store_sa(1);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
  } else {
    load_x(0);
    store_x(0);
    load_x(1);
#pragma unroll
    for (int d = 0; d < NW; ++d) load_w(d, d);
    store_x(1);
    load_x(2);
  }
  __syncthreads();
#pragma unroll
  for (int st = 0; st < 4; ++st) read_operand(stage0, 0, st);
  read_scales(scale0, 0, 0);

  // Timetable of the activations of group q + 2: requested from memory at the top of group
  // q - 1, widened into stage (q + 2) % 3 at the top of group q (a whole group after the
  // request, and with the rest of group q to land before anyone waits for them), published
  // by the barrier that ends group q, first read at the end of group q + 1 (the operands
  // of a group's first token tile are fetched under the last tile of the group before).
  auto group_body = [&](auto slot_c, int q) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_c)::value;
    const uint8_t* xl = stage_ptr(SLOT);
    const uint8_t* xl_next = stage_ptr((SLOT + 1) % NW);
    const float* sl = scale_ptr(SLOT);
    const float* sl_next = scale_ptr((SLOT + 1) % NW);
    if constexpr (WIDE) {
      // group q + 2 straight into its stage (last read in group q - 1); it has the whole of
      // this group to land, and the wait in front of this group's closing barrier counts the
      // loads issued after it: the scale triple (slot 0 only) and the ring refill
      dma_x(q + 2, stage_ptr((SLOT + 2) % NW));
      __builtin_amdgcn_sched_barrier(0);
      store_sa((SLOT + 2) % NW);
      if (SLOT == 0) load_sa3(q + 3);
    } else {
      store_x((SLOT + 2) % NW);                  // group q + 2; that stage was last read in group q - 1
      if (SLOT == 0) load_sa3(q + 3);            // (its last scale, of group q + 2, has just been used)
      load_x(q + 3);
    }
    __builtin_amdgcn_sched_barrier(0);

    // operands of this group: four B operands per 32-row pair, the lane's weight scale
    v4i b[PN][4];
    float swf[PN], swc[PN];
#pragma unroll
    for (int j = 0; j < PN; ++j) {
      const I8Pair lo = unpack_i8(wlo[SLOT][j]), hi = unpack_i8(whi[SLOT][j]);
      b[j][0] = lo.lo; b[j][1] = lo.hi; b[j][2] = hi.lo; b[j][3] = hi.hi;
      swf[j] = half_bits_to_float((uint16_t)sq[SLOT][j]);
      swc[j] = swf[j] * -12582912.0f;            // exact: 11 significant bits times 1.5 * 2^23
    }
    load_w(SLOT, q + NW);                        // the slot's contents are in b[] and swf[] now
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int idx = 0; idx < kTiles; ++idx) {
      const int t = idx / PN, j = idx % PN;
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        P[idx & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[st], b[j][st], st == 0 ? seed : P[idx & 1], 0, 0, 0);
        asm volatile("" : "+v"(P[idx & 1]));       // the MFMA is issued here, ahead of the rescaling below
        if (j == PN - 1) {
          // this step's operand of the next token tile: of this group, or the first tile of
          // the next group (whose stage the barrier before this group has published)
          if (t + 1 < PM) read_operand(xl, t + 1, st);
          else read_operand(xl_next, 0, st);
        }
        if (idx > 0) {
          rescale_quarter(P[(idx - 1) & 1], swf[(idx - 1) % PN], swc[(idx - 1) % PN], S[((idx - 1) / PN) & 1],
                          acc[(idx - 1) % PN][(idx - 1) / PN], st);
        } else {
          rescale_quarter(P[(kTiles - 1) & 1], pend_sw, pend_swc, pend_S, acc[PN - 1][PM - 1], st);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      // S[(t+1)&1] belonged to token tile t-1, whose last rescaling has just been issued
      if (j == 0 && t + 1 < PM) read_scales(sl, t + 1, (t + 1) & 1);
    }
    pend_sw = swf[PN - 1];
    pend_swc = swc[PN - 1];
    pend_S = S[(PM - 1) & 1];
    read_scales(sl_next, 0, 0);                  // S[0] was token tile PM-2's: released
    // (loads complete in order; no store may sit between them, so the kernel must compile
    // without register spills)
    if constexpr (WIDE) __builtin_amdgcn_s_waitcnt(waitcnt_vm(3 * PN + (SLOT == 0 ? 1 : 0)));
    __syncthreads();
  };

  // Three groups per trip (the ring slots are named statically), each a straight line;
  // the loop is left between groups (every block inside keeps a single predecessor, so
  // the compiler's wait-count bookkeeping stays exact).  Requests past the end of the
  // slice are out of range: zeros, no traffic.
  for (int q = 0; q < ng; q += NW) {
    group_body(std::integral_constant<int, 0>{}, q);
    if (q + 1 >= ng) break;
    group_body(std::integral_constant<int, 1>{}, q + 1);
    if (q + 2 >= ng) break;
    group_body(std::integral_constant<int, 2>{}, q + 2);
  }
#pragma unroll
  for (int part = 0; part < 4; ++part) rescale_quarter(P[(kTiles - 1) & 1], pend_sw, pend_swc, pend_S, acc[PN - 1][PM - 1], part);

  tile_store32<PN, PM, false>(p, tc, acc, n0, m0 + mw0);
}

}  // namespace qspec
