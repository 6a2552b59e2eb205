// One persistent launch for the MLP of a decoder block in the draft pass (paper Sec. 3.1,
// draft phase: gamma passes of small-M linear layers back to back; Sec. 3.2: the method's
// gain rests on the draft pass being fast):
//     gate/up projection (W4A4)  ->  SiLU(gate) * up, quantised to 4 bit  ->  down projection (W4A4)
// at M <= 32 tokens, where every one of these steps is bound by memory latency and launch
// cost rather than by arithmetic.  The grid is one workgroup of eight wavefronts per
// compute unit, all resident at once; a workgroup keeps its place through both projections.
//
//   stage 1   a workgroup streams its share of the gate/up weight tiles (the streaming
//             kernel's loop) and stores its fp16 outputs with write-through stores;
//   between   every quantisation group of 128 intermediate features has an arrival counter
//             that counts the 16 output tiles (8 gate, 8 up) it is made of.  The workgroup
//             whose tiles complete a group computes SiLU(gate) * up for it, quantises it
//             (all M tokens) and bumps the counter of finished groups.  Nobody waits here;
//   prefetch  then every workgroup copies ALL the down-projection weight tiles it owns into
//             LDS (loads that write LDS directly), so that HBM keeps streaming while the
//             few workgroups that quantise are still at work;
//   wait      thread 0 polls the counter of finished groups, a BOUNDED number of times; if
//             it gives up, the workgroup raises the caller's status word and leaves;
//   stage 2   the down projection from the weights in LDS and the quantised activations.
//
// Ordering between workgroups: data that another workgroup will read is either written
// with agent-scope write-through stores and published by "wait for vmcnt(0), barrier,
// counter increment" (the fp16 gate/up tensor; see exchange.hpp for why this equals a
// release here), or published by a counter increment with RELEASE semantics (the quantised
// activations, written with plain stores by the quantiser's shared code); readers execute
// an ACQUIRE fence at agent scope after they have seen the counter.
// All counters are zero on entry and zero again on exit (the last workgroup through the
// wait resets them); after a give-up the caller must clear them.
#pragma once
#include "exchange.hpp"
#include "gemm_stream.hpp"
#include "producers.hpp"

namespace qspec {

struct MlpArgs {
  // stage 1: gate/up projection, [N1 = 2 I] x [K1 = hidden]
  const uint4* codes1;
  const uint16_t* scales1T;
  const uint8_t* qa_h;       // quantised block input [M][K1/2]
  const float* sa_h;         // [M][G1]
  uint16_t* y_gu;            // out: fp16 [M][N1], gate in the first I columns
  // between the stages
  uint8_t* qa_i;             // out: quantised SiLU(gate)*up [M][I/2]
  float* sa_i;               // out: [M][I/128]
  // stage 2: down projection, [N2 = hidden] x [K2 = I]
  const uint4* codes2;
  const uint16_t* scales2T;
  uint16_t* y;               // out: fp16 [M][N2]
  unsigned* counters;        // [G2] tiles arrived per quantisation group, then [G2]: groups finished, [G2+1]: workgroups through the wait
  int* status;               // device word: set to 1 by a workgroup whose wait gave up
  int M, N1, K1, N2, K2;
  unsigned spin_limit;       // polls before a workgroup gives up
};

constexpr int kMlpWBufTiles = 96;          // down-projection weight tiles (1 KB each) a workgroup can hold in LDS
constexpr int kMlpRedTiles = 4;            // output tiles combined per reduction pass

// Combine the eight per-wave sums of the workgroup's output tiles (kMlpRedTiles per pass)
// and store fp16; WRITE_THROUGH: agent-scope stores that another workgroup will read.
template <int TM, int NT, bool WRITE_THROUGH>
__device__ __forceinline__ void mlp_reduce_store(float (&facc)[NT][TM][4], float* red_base, uint16_t* y, int N, int M,
                                                 int T0, int nt_valid, int wave, int lane) {
  constexpr int W = kStreamWaves;
  float (*red)[kMlpRedTiles * 4][kWave] = reinterpret_cast<float (*)[kMlpRedTiles * 4][kWave]>(red_base);
  const int r16 = lane & 15, kb = lane >> 4;
#pragma unroll
  for (int base = 0; base < NT * TM; base += kMlpRedTiles) {
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kMlpRedTiles; ++c) {
      const int o = base + c;
      if (o < NT * TM) {
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][c * 4 + r][lane] = facc[o / TM][o % TM][r];
      }
    }
    __syncthreads();
    const int o = base + wave;
    if (wave < kMlpRedTiles && o < NT * TM) {
      const int j = o / TM, t = o - j * TM;
      float s[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < W; ++w) v += red[w][wave * 4 + r][lane];
        s[r] = v;
      }
      const int m = 16 * t + r16;
      if (j < nt_valid && m < M) {
        const uint32_t lo = (uint32_t)float_to_half_bits(s[0]) | ((uint32_t)float_to_half_bits(s[1]) << 16);
        const uint32_t hi = (uint32_t)float_to_half_bits(s[2]) | ((uint32_t)float_to_half_bits(s[3]) << 16);
        uint16_t* dst = y + (size_t)m * N + (T0 + j) * 16 + 4 * kb;
        if (WRITE_THROUGH) {
          __hip_atomic_store(reinterpret_cast<uint64_t*>(dst), (uint64_t)lo | ((uint64_t)hi << 32), __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
        } else {
          *reinterpret_cast<uint2*>(dst) = uint2{lo, hi};
        }
      }
    }
  }
}

// The streaming loop of gemm_stream_kernel for one block of NT tiles over groups 0 .. G-1
// (wave w takes groups w, w + 8, ...), draft mode.
template <int TM, int NT>
__device__ __forceinline__ void mlp_stream(const StreamArgs& p, const StreamRsrc& rs, int T0, int nt_valid, int wave, int lane,
                                           float (&facc)[NT][TM][4], const uint8_t* wlds) {
  constexpr int W = kStreamWaves;
  const int n_g = max(0, (p.G - wave + W - 1) / W);
  if (n_g <= 0 || nt_valid <= 0) return;
  auto grp = [&](int it) { return wave + it * W; };
  GroupRegs<true, TM, NT> A, B;
  uint2 sw_cur = {0u, 0u}, sw_nxt = {0u, 0u};
  if (pair_scales(NT)) sw_cur = load_pair_scales<NT>(rs, p, grp(0), grp(1), true, 1 < n_g, T0, nt_valid, lane);
  load_group<true, TM, NT>(A, rs, p, grp(0), true, T0, nt_valid, lane, wlds);
  for (int it = 0; it < n_g; it += 2) {
    if (pair_scales(NT)) sw_nxt = load_pair_scales<NT>(rs, p, grp(it + 2), grp(it + 3), it + 2 < n_g, it + 3 < n_g, T0, nt_valid, lane);
    load_group<true, TM, NT>(B, rs, p, grp(it + 1), it + 1 < n_g, T0, nt_valid, lane, wlds);
    __builtin_amdgcn_sched_barrier(0);
    compute_group<true, TM, NT, 0>(A, sw_cur, facc, nullptr, lane);
    __builtin_amdgcn_sched_barrier(0);
    load_group<true, TM, NT>(A, rs, p, grp(it + 2), it + 2 < n_g, T0, nt_valid, lane, wlds);
    __builtin_amdgcn_sched_barrier(0);
    if (it + 1 < n_g) compute_group<true, TM, NT, 1>(B, sw_cur, facc, nullptr, lane);
    __builtin_amdgcn_sched_barrier(0);
    sw_cur = sw_nxt;
  }
}

typedef __attribute__((address_space(3))) void* mlp_lds_ptr_t;

template <int TM, int NT1, int NT2>
__global__ __launch_bounds__(kStreamWaves * 64, 1) void mlp_draft_kernel(MlpArgs p) {
  constexpr int W = kStreamWaves;
  __shared__ __attribute__((aligned(1024))) uint8_t wbuf[kMlpWBufTiles * 1024];     // stage-2 weights (written by direct loads)
  __shared__ __attribute__((aligned(16))) float red[W * kMlpRedTiles * 4 * kWave];  // reductions of both stages
  __shared__ int todo[8];
  __shared__ int n_todo, wait_ok;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nwg = gridDim.x, b = blockIdx.x;
  const int M = p.M;
  const int I = p.K2, G2 = p.K2 / kGroup;
  unsigned* const group_cnt = p.counters;
  unsigned* const done = p.counters + G2;
  unsigned* const seen = p.counters + G2 + 1;

  // ------------------------------------------------------------ stage 1: gate/up projection
  const int tiles1 = p.N1 / 16;
  const int t_lo = (int)((long long)b * tiles1 / nwg), t_hi = (int)((long long)(b + 1) * tiles1 / nwg);
  const int nt1 = t_hi - t_lo;                           // <= NT1 (checked on the host)
  {
    StreamArgs a{};
    a.M = M; a.N = p.N1; a.K = p.K1; a.G = p.K1 / kGroup; a.S = 1;
    StreamRsrc rs;
    rs.codes = make_rsrc(p.codes1, (uint32_t)((size_t)p.N1 * p.K1 / 2));
    rs.scales = make_rsrc(p.scales1T, (uint32_t)((size_t)p.N1 * a.G * 2));
    rs.act = make_rsrc(p.qa_h, (uint32_t)((size_t)M * p.K1 / 2));
    rs.sa = make_rsrc(p.sa_h, (uint32_t)((size_t)M * a.G * 4));
    float facc[NT1][TM][4];
#pragma unroll
    for (int j = 0; j < NT1; ++j)
#pragma unroll
      for (int t = 0; t < TM; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) facc[j][t][r] = 0.0f;
    mlp_stream<TM, NT1>(a, rs, t_lo, nt1, wave, lane, facc, nullptr);
    mlp_reduce_store<TM, NT1, false>(facc, red, p.y_gu, p.N1, M, t_lo, nt1, wave, lane);
  }
  // publish the tiles: plain stores (adjacent tiles merge into whole lines in L2; 8-byte
  // write-through stores were measured at 3 to 10 us for this step), the barrier, then
  // counter increments with RELEASE semantics (one L2 write-back per workgroup)
  __syncthreads();
  if (tid == 0) {
    // tile t (gate: t < I/16, up: the same index + I/16) belongs to quantisation group (t % (I/16)) / 8
    const int tilesI = I / 16;
    int n = 0, t = t_lo;
    if (t < t_hi) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    while (t < t_hi) {
      const int j = (t % tilesI) / 8;
      int c = 0;
      while (t < t_hi && (t % tilesI) / 8 == j) { ++c; ++t; }
      const unsigned old = __hip_atomic_fetch_add(&group_cnt[j], (unsigned)c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old + (unsigned)c == 16u) {
        __hip_atomic_store(&group_cnt[j], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (n < 8) todo[n++] = j;
      }
    }
    n_todo = n;
    if (n > 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  }
  __syncthreads();

  // ------------------------------------------------------------ SiLU(gate) * up + quantiser for the groups this workgroup completed
  // 16 lanes per (token, group): 32 such units per pass over the workgroup's 512 threads
  {
    const int n_units = M * n_todo;
    for (int u0 = 0; u0 < n_units; u0 += 32) {
      const int unit = u0 + (tid >> 4), l = tid & 15;
      const bool live = unit < n_units;
      const int gi = live ? unit / M : 0, m = live ? unit - gi * M : 0;
      const int j = todo[gi];
      uint4 graw = {0u, 0u, 0u, 0u}, uraw = {0u, 0u, 0u, 0u};
      if (live) {
        graw = *reinterpret_cast<const uint4*>(p.y_gu + (size_t)m * p.N1 + (size_t)j * kGroup + 8 * l);
        uraw = *reinterpret_cast<const uint4*>(p.y_gu + (size_t)m * p.N1 + (size_t)I + (size_t)j * kGroup + 8 * l);
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
      const size_t idx = (size_t)m * (size_t)(I / 8) + (size_t)j * 16 + l;   // word index in [M][I/8]
      finish_unit(v, false, live, idx, reinterpret_cast<uint32_t*>(p.qa_i), p.sa_i, nullptr);
    }
    if (n_todo > 0) {
      __syncthreads();                                     // the groups are written ...
      if (tid == 0) __hip_atomic_fetch_add(done, (unsigned)n_todo, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);   // ... and published
    }
  }

  // ------------------------------------------------------------ prefetch: this workgroup's down-projection weights -> LDS
  const int tiles2 = p.N2 / 16;
  const int u_lo = (int)((long long)b * tiles2 / nwg), u_hi = (int)((long long)(b + 1) * tiles2 / nwg);
  const int nt2 = u_hi - u_lo;                           // <= NT2, nt2 * G2 <= kMlpWBufTiles (checked on the host)
  {
    const rsrc_t r_codes2 = make_rsrc(p.codes2, (uint32_t)((size_t)p.N2 * p.K2 / 2));
    const int n_tg = nt2 * G2;
    for (int i = wave; i < n_tg; i += W) {
      const int j = i / G2, g = i - j * G2;
      const uint32_t off = ((uint32_t)(u_lo + j) * (uint32_t)G2 + (uint32_t)g) * 1024u + (uint32_t)lane * 16u;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r_codes2, (mlp_lds_ptr_t)(wbuf + (size_t)i * 1024), 16, off, 0, 0, 2);
    }
  }

  // ------------------------------------------------------------ bounded wait for the quantised activations
  if (tid == 0) {
    unsigned n = 0;
    bool ok = false;
    while (true) {
      if (__hip_atomic_load(done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= (unsigned)G2) { ok = true; break; }
      if (++n >= p.spin_limit) break;
      __builtin_amdgcn_s_sleep(2);
    }
    if (ok) {
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      const unsigned old = __hip_atomic_fetch_add(seen, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old == (unsigned)nwg - 1) {                      // everybody has seen it: back to zero for the next launch
        __hip_atomic_store(done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(seen, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    } else {
      *p.status = 1;
    }
    wait_ok = ok ? 1 : 0;
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);                    // vmcnt(0): this wave's copies into LDS have landed
  __syncthreads();
  if (!wait_ok) return;                                  // (the whole workgroup: uniform)

  // ------------------------------------------------------------ stage 2: down projection
  {
    StreamArgs a{};
    a.M = M; a.N = p.N2; a.K = p.K2; a.G = G2; a.S = 1;
    StreamRsrc rs;
    rs.codes = make_rsrc(p.codes2, (uint32_t)((size_t)p.N2 * p.K2 / 2));
    rs.scales = make_rsrc(p.scales2T, (uint32_t)((size_t)p.N2 * G2 * 2));
    rs.act = make_rsrc(p.qa_i, (uint32_t)((size_t)M * p.K2 / 2));
    rs.sa = make_rsrc(p.sa_i, (uint32_t)((size_t)M * G2 * 4));
    float facc[NT2][TM][4];
#pragma unroll
    for (int j = 0; j < NT2; ++j)
#pragma unroll
      for (int t = 0; t < TM; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) facc[j][t][r] = 0.0f;
    mlp_stream<TM, NT2>(a, rs, u_lo, nt2, wave, lane, facc, wbuf);
    mlp_reduce_store<TM, NT2, false>(facc, red, p.y, p.N2, M, u_lo, nt2, wave, lane);
  }
}

}  // namespace qspec
