// Tiled draft-mode (W4A4) kernel for M > 32 on v_mfma_i32_32x32x32_i8 (paper
// Sec. 1 item (2): both operands stay 4-bit integers on the low-precision matrix
// units; Sec. 4.1: groups of 128).
//
// Per K group and 32 x 32 output tile: four MFMAs (32 k each) into a fresh int32
// tile P (exact), then  acc += float(P) * (sa[m,g] * 2^-8) * sw[n,g]  in fp32.
// Both int8 operands are 16*code (a nibble moved to the high half of a byte), so
// P is 256 times the true partial sum and 2^-8 rides on the activation scale.
// That epilogue is 3 VALU operations per output and group against 1/4 MFMA: the
// kernel is bound by vector arithmetic, not by the matrix unit, and the schedule
// below exists to keep the MFMAs and the LDS traffic hidden under it.
//
// A workgroup of WGN x WGM wavefronts owns BN x BM outputs (BN = 32*PN*WGN,
// BM = 32*PM*WGM) over a range of K groups.
//   - Activations: the BM x 64 B code block of a group and its BM scales go global
//     -> registers two groups ahead, are widened to int8 once per workgroup and
//     written to one of three LDS stages at the end of a group; one barrier per
//     group.  Row layout: 8 slots of 16 bytes (slot kb: low nibbles of k-block kb,
//     slot 4+kb: high nibbles), slot index xor-ed with (row/2)%8 so that 16
//     consecutive rows at one slot hit 16 different bank groups.
//   - Weights and their scales: straight into registers in MFMA operand layout
//     through a ring of three groups (slots named statically: the group loop is
//     unrolled three times, which also fixes the LDS stage of a group).
//
// A operand (32 rows x 32 k): lane l = (h = l / 32, row = l % 32) supplies 16 k of
// its row.  It fetches the 16 bytes of blob tile lane (row % 16, kb = h) ["lo"] and
// (row % 16, kb = h + 2) ["hi"] of the 16-row tile holding its row; each gives two
// operands (low nibbles, high nibbles), four MFMA steps in all.  The B operand of
// a step is, for lane (h, m = l % 32), the matching slot of token row m: kb = h or
// h + 2, low or high nibbles.  Any assignment of k to steps and lanes is valid as
// long as both operands use the same one: a group's dot product is order-free.
// D: lane holds column m = l % 32 and rows 8a + 4h + r (a, r = 0..3) in register
// 4a + r.
#pragma once
#include "gemm_tile16.hpp"

namespace qspec {

typedef int v16i __attribute__((ext_vector_type(16)));

template <int PN, int PM, int WGN, int WGM, int OCC>
__global__ __launch_bounds__(64 * WGN * WGM, OCC) void gemm_tile4w_kernel(TileArgs p) {
  constexpr int kWaves = WGN * WGM;
  constexpr int kThreads = 64 * kWaves;
  constexpr int BM = 32 * PM * WGM;
  constexpr int NW = 3;                              // weight ring = LDS stages
  constexpr int kActBytes = BM * 128;
  constexpr int kStageBytes = kActBytes + BM * 4;    // + sa[m] * 2^-8 of the group
  constexpr int kChunks = BM * 4;                    // 16-byte pieces of codes per group
  constexpr int U = (kChunks + kThreads - 1) / kThreads;
  static_assert(kChunks % kThreads == 0 || kChunks < kThreads, "whole passes, or one partial pass");
  static_assert(BM <= kThreads, "one thread per token row stages the activation scale");
  __shared__ __attribute__((aligned(16))) uint8_t lds[NW * kStageBytes];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wn = wave % WGN, wm = wave / WGN;
  const int m32 = lane & 31, h = lane >> 5;
  const int G = p.G;
  const TileCoord tc = tile_coord(p);
  const int g0 = tc.g0, g1 = tc.g1;
  const int ng = g1 - g0;
  const int n0 = (tc.nblk * (PN * WGN) + wn * PN) * 32;      // first output feature of this wave
  const int m0 = tc.mblk * BM;
  const int mw0 = wm * (PM * 32);

  const rsrc_t r_codes = make_rsrc(p.codes, (uint32_t)((size_t)p.N * p.K / 2));
  const rsrc_t r_scales = make_rsrc(p.scalesT, (uint32_t)((size_t)p.N * G * 2));
  const rsrc_t r_act = make_rsrc(p.act, (uint32_t)((size_t)p.M * p.K / 2));
  const rsrc_t r_sa = make_rsrc(p.sa, (uint32_t)((size_t)p.M * G * 4));
  // Work that does not exist gets bit 31 in its load offset (out of range: zeros, no
  // traffic), by arithmetic: a select between offsets tempts the compiler into a
  // branch around two load instructions, which ruins its wait-count bookkeeping.
  auto past_end = [&](int q) -> uint32_t { return (uint32_t)((ng - 1 - q) >> 31) << 31; };   // q >= ng ? bit 31 : 0

  // ---- activations: global -> registers (rows past M lie past the end of the buffer)
  uint4 xs[U];
  float sas = 0.0f;
  const uint32_t idle_sa = (uint32_t)((BM - 1 - tid) >> 31) << 31;                 // tid >= BM
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
    sas = buf_load_f32(r_sa, (((uint32_t)(m0 + tid) * G + g) * 4u) | gone | idle_sa);
  };
  auto store_x = [&](int stage) {
    uint8_t* base = lds + stage * kStageBytes;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = tid + u * kThreads;
      const int row = idx >> 2, c = idx & 3;
      if (kChunks % kThreads == 0 || idx < kChunks) {
        const I8Pair q = unpack_i8(xs[u]);
        const int sw = (row >> 1) & 7;
        *reinterpret_cast<v4i*>(base + row * 128 + ((c ^ sw) << 4)) = q.lo;
        *reinterpret_cast<v4i*>(base + row * 128 + (((c + 4) ^ sw) << 4)) = q.hi;
      }
    }
    if (tid < BM) *reinterpret_cast<float*>(base + kActBytes + tid * 4) = sas * 0.00390625f;   // 2^-8, exact
  };

  // ---- weights: ring of NW groups; per 32-row pair two 16-byte pieces and the
  // scales of the four runs of rows this lane's D registers cover
  uint4 wlo[NW][PN], whi[NW][PN];
  uint2 sq[NW][PN][4];
  const int n_lane = n0 + m32;          // this lane's weight row in pair 0
  const uint32_t w_voff = (uint32_t)(n_lane >> 4) * G * 1024u + (uint32_t)((n_lane & 15) + 16 * h) * 16u;
  auto load_w = [&](int d, int q) {
    const uint32_t gone = past_end(q);
    const int g = g0 + q;
#pragma unroll
    for (int j = 0; j < PN; ++j) {
      const uint32_t none = (uint32_t)((p.N - 1 - (n_lane + 32 * j)) >> 31) << 31;
      const uint32_t wo = w_voff + (uint32_t)(2 * j) * G * 1024u + (uint32_t)g * 1024u;
      wlo[d][j] = buf_load16(r_codes, wo | gone | none);
      whi[d][j] = buf_load16(r_codes, (wo + 512u) | gone | none);
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const int n = n0 + 32 * j + 8 * a + 4 * h;
        const uint32_t nonea = (uint32_t)((p.N - 1 - n) >> 31) << 31;
        sq[d][j][a] = buf_load8(r_scales, (((uint32_t)g * (uint32_t)p.N + (uint32_t)n) * 2u) | gone | nonea);
      }
    }
  };

  float acc[PN][PM][16];
#pragma unroll
  for (int j = 0; j < PN; ++j)
#pragma unroll
    for (int t = 0; t < PM; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][t][r] = 0.0f;

  // prologue: groups 0 and 1 into stages 0 and 1, the ring filled
  load_x(0);
  store_x(0);
  load_x(1);
#pragma unroll
  for (int d = 0; d < NW; ++d) load_w(d, d);
  store_x(1);
  __syncthreads();

  auto group_body = [&](auto slot_c, int q) __attribute__((always_inline)) {
    constexpr int SLOT = decltype(slot_c)::value;
    const uint8_t* xl = lds + SLOT * kStageBytes;
    load_x(q + 2);                               // lands in stage (SLOT + 2) % 3 at the end of this group
    __builtin_amdgcn_sched_barrier(0);

    // operands of this group: four A operands per 32-row pair, fp32 weight scales
    v4i a[PN][4];
    float swf[PN][16];
#pragma unroll
    for (int j = 0; j < PN; ++j) {
      const I8Pair lo = unpack_i8(wlo[SLOT][j]), hi = unpack_i8(whi[SLOT][j]);
      a[j][0] = lo.lo; a[j][1] = lo.hi; a[j][2] = hi.lo; a[j][3] = hi.hi;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        swf[j][4 * q4 + 0] = half_bits_to_float((uint16_t)(sq[SLOT][j][q4].x & 0xFFFF));
        swf[j][4 * q4 + 1] = half_bits_to_float((uint16_t)(sq[SLOT][j][q4].x >> 16));
        swf[j][4 * q4 + 2] = half_bits_to_float((uint16_t)(sq[SLOT][j][q4].y & 0xFFFF));
        swf[j][4 * q4 + 3] = half_bits_to_float((uint16_t)(sq[SLOT][j][q4].y >> 16));
      }
    }
    load_w(SLOT, q + NW);                        // the slot's contents are in a[] and swf[] now
    __builtin_amdgcn_sched_barrier(0);

    v4i b[2][4];                                 // B operands of token tile t live in b[t & 1]
    float sam[2];
    auto read_tile = [&](int t, int buf) {
      const int row = mw0 + 32 * t + m32;
      const int sw = (row >> 1) & 7;
      b[buf][0] = *reinterpret_cast<const v4i*>(xl + row * 128 + ((h ^ sw) << 4));
      b[buf][1] = *reinterpret_cast<const v4i*>(xl + row * 128 + (((h + 4) ^ sw) << 4));
      b[buf][2] = *reinterpret_cast<const v4i*>(xl + row * 128 + (((h + 2) ^ sw) << 4));
      b[buf][3] = *reinterpret_cast<const v4i*>(xl + row * 128 + (((h + 6) ^ sw) << 4));
      sam[buf] = *reinterpret_cast<const float*>(xl + kActBytes + row * 4);
    };
    v16i P[2];                                   // int32 tiles, alternating
    // scale-and-add of the tile finished one step ago, a quarter at a time
    auto epilogue_quarter = [&](int idx, int part) {
      const int t = idx / PN, j = idx % PN;
#pragma unroll
      for (int r = 4 * part; r < 4 * part + 4; ++r)
        acc[j][t][r] += (float)P[idx & 1][r] * (sam[t & 1] * swf[j][r]);
      // Pin the arithmetic here: nothing else uses these sums before the end of the
      // kernel, and instruction selection would otherwise park the whole epilogue of
      // every group at the bottom of the unrolled loop body (with every int32 tile
      // kept alive until then).
      asm volatile("" : "+v"(acc[j][t][4 * part]), "+v"(acc[j][t][4 * part + 1]), "+v"(acc[j][t][4 * part + 2]),
                        "+v"(acc[j][t][4 * part + 3]));
    };
    read_tile(0, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int idx = 0; idx < PN * PM; ++idx) {
      const int t = idx / PN, j = idx % PN;
      if (j == 0 && t + 1 < PM) {
        // operands of the next token tile, a whole tile ahead of their MFMAs (its
        // scale is fetched further down, once its register is free)
        const int row = mw0 + 32 * (t + 1) + m32;
        const int sw = (row >> 1) & 7;
        const int buf = (t + 1) & 1;
        b[buf][0] = *reinterpret_cast<const v4i*>(xl + row * 128 + ((h ^ sw) << 4));
        b[buf][1] = *reinterpret_cast<const v4i*>(xl + row * 128 + (((h + 4) ^ sw) << 4));
        b[buf][2] = *reinterpret_cast<const v4i*>(xl + row * 128 + (((h + 2) ^ sw) << 4));
        b[buf][3] = *reinterpret_cast<const v4i*>(xl + row * 128 + (((h + 6) ^ sw) << 4));
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        v16i c = P[idx & 1];
        if (st == 0) {
#pragma unroll
          for (int r = 0; r < 16; ++r) c[r] = 0;
        }
        P[idx & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[j][st], b[t & 1][st], c, 0, 0, 0);
        asm volatile("" : "+v"(P[idx & 1]));       // the MFMA is issued here, ahead of the epilogue below
        if (idx > 0) epilogue_quarter(idx - 1, st);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (j == PN - 1 && t + 1 < PM) {
        // sam[(t+1)&1] was the scale of token tile t-1, whose last epilogue has just been issued
        const int row = mw0 + 32 * (t + 1) + m32;
        sam[(t + 1) & 1] = *reinterpret_cast<const float*>(xl + kActBytes + row * 4);
      }
    }
#pragma unroll
    for (int part = 0; part < 4; ++part) epilogue_quarter(PN * PM - 1, part);

    store_x((SLOT + 2) % NW);
    __syncthreads();
  };

  // Straight-line body of three groups (no branch around a group: the compiler's
  // wait-count bookkeeping stays exact only without control flow).  Groups past the
  // end of the slice run on zeros: their loads are out of range.
  for (int q = 0; q < ng; q += NW) {
    group_body(std::integral_constant<int, 0>{}, q);
    group_body(std::integral_constant<int, 1>{}, q + 1);
    group_body(std::integral_constant<int, 2>{}, q + 2);
  }

  tile_store32<PN, PM>(p, tc, acc, n0, m0 + mw0);
}

}  // namespace qspec
