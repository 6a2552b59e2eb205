// C ABI of the QSpec W4 linear layer for gfx950: argument validation, kernel
// selection by problem shape, launches on the caller's stream.  Declarations
// and the buffer layouts are in include/qspec.h.
#include "qspec.h"

#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "accept.hpp"
#include "common.hpp"
#include "gemm_generic.hpp"
#include "gemm_stream.hpp"
#include "gemm_tile16.hpp"
#include "gemm_tile4.hpp"
#include "mlp_chain.hpp"
#include "pack.hpp"
#include "producers.hpp"
#include "quant_act.hpp"

using namespace qspec;

// Scratch of qspec_gemm_w4a16_noalloc: arrival counters (first kTicketBytes) and K-slice
// partial sums, for callers that can neither allocate nor pass a workspace.  Every GPU
// the library runs on holds its own copy until the process ends.  In host code this name
// is only a handle for hipGetSymbolAddress; kernels and fills take the address that call
// returned for the current device (scratch_of_device below), never the name.
constexpr size_t kScratchBytes = ((size_t)32 << 20) + 16384;   // 32 MiB of partial sums + 16 KiB of counters
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

inline int check_shape(int M, int N, int K, int group) {
  if (group != kGroup) return QSPEC_ERR_SHAPE;
  if (K <= 0 || K % kGroup != 0) return QSPEC_ERR_SHAPE;
  if (N <= 0 || N % kTileRows != 0) return QSPEC_ERR_SHAPE;
  if (M < 1) return QSPEC_ERR_SHAPE;
  // 32-bit byte offsets are used inside the kernels: every buffer stays below 2 GiB
  if ((long long)N * K / 2 >= 0x7fffffffLL) return QSPEC_ERR_SHAPE;
  if ((long long)M * K * 2 >= 0x7fffffffLL) return QSPEC_ERR_SHAPE;
  return QSPEC_OK;
}

// The kernels use gfx950-only matrix instructions; refuse anything else.
int check_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return QSPEC_ERR_HIP;
  (void)hipGetLastError();
  static int verdict[64];   // 0 unknown, 1 ok, 2 unsupported
  if (dev < 0 || dev >= 64) return QSPEC_ERR_UNSUPPORTED;
  if (verdict[dev] == 0) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return QSPEC_ERR_HIP;
    verdict[dev] = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 2;
  }
  return verdict[dev] == 1 ? QSPEC_OK : QSPEC_ERR_UNSUPPORTED;
}

// QSPEC_ERR_HIP must mean "THIS call's launch failed": check_device(), which every entry
// point calls after validating its arguments and before launching, drops whatever error an
// unrelated earlier runtime call left behind; launch_status() then sees only this call's.
inline int launch_status() { return hipGetLastError() == hipSuccess ? QSPEC_OK : QSPEC_ERR_HIP; }

inline const uint16_t* blob_scales(const void* packed, int N, int K) {
  return reinterpret_cast<const uint16_t*>(static_cast<const uint8_t*>(packed) + (size_t)N * K / 2);
}

inline unsigned blocks_for(size_t n, unsigned per_block) { return (unsigned)((n + per_block - 1) / per_block); }

// tokens per workgroup: smallest of 16, 32, 64, 128 that covers M (128 at most)
inline int pick_tm(int M) { return M <= 16 ? 1 : M <= 32 ? 2 : M <= 64 ? 4 : 8; }

template <int TM>
void launch_w4a4(const GemmArgs& a, hipStream_t s) {
  dim3 grid(a.N / 16, (a.M + TM * 16 - 1) / (TM * 16));
  hipLaunchKernelGGL((gemm_w4a4_generic<TM, 4, false>), grid, dim3(256), 0, s, a);
}
template <int TM>
void launch_w4a16(const GemmArgs& a, hipStream_t s) {
  dim3 grid(a.N / 16, (a.M + TM * 16 - 1) / (TM * 16));
  hipLaunchKernelGGL((gemm_w4a16_generic<TM, 4>), grid, dim3(256), 0, s, a);
}


constexpr int kNumCU = 256;

// Plan overrides (benchmark A/B and tests only).  They are parsed ONCE: from the
// environment at the first use, and afterwards only through qspec_debug_set_plan.  The
// launch path reads plain integers; no entry point calls getenv.
//   QSPEC_KERNEL=generic            route M > 32 to the untiled reference kernels
//   QSPEC_STREAM_W4A4 / _W4A16      "NT,S" or "NT,S,MS": tiles per workgroup, K-slices, token-row blocks
//   QSPEC_STREAM_MAX_W4A4 / _W4A16  largest M of the streaming kernels without token-row blocks
//   QSPEC_TILE_W4A4 / _W4A16        "shape,S": workgroup shape index, K-slices
struct PlanOverrides {
  bool generic = false;
  int stream_fields[2] = {0, 0};      // [w4a4]: how many of nt, S, ms were given (0: no override)
  int stream[2][3] = {{0, 0, 0}, {0, 0, 0}};
  int stream_max[2] = {0, 0};         // 0: the default bound
  bool tile_set[2] = {false, false};
  int tile[2][2] = {{0, 0}, {0, 0}};
  unsigned mlp_spin = 0;              // 0: the default number of polls of the persistent MLP kernel's wait
};

// value == nullptr (or unparsable) clears the override named `name`; false: unknown name.
bool apply_override(PlanOverrides& o, const char* name, const char* value) {
  if (strcmp(name, "QSPEC_KERNEL") == 0) { o.generic = value && strcmp(value, "generic") == 0; return true; }
  if (strcmp(name, "QSPEC_MLP_SPIN") == 0) { o.mlp_spin = value ? (unsigned)strtoul(value, nullptr, 10) : 0u; return true; }
  for (int w4a4 = 0; w4a4 < 2; ++w4a4) {
    if (strcmp(name, w4a4 ? "QSPEC_STREAM_W4A4" : "QSPEC_STREAM_W4A16") == 0) {
      int* f = o.stream[w4a4];
      f[0] = f[1] = 0; f[2] = 1;
      const int nf = value ? sscanf(value, "%d,%d,%d", &f[0], &f[1], &f[2]) : 0;
      o.stream_fields[w4a4] = nf >= 2 ? nf : 0;
      if (nf < 3) f[2] = 1;
      return true;
    }
    if (strcmp(name, w4a4 ? "QSPEC_STREAM_MAX_W4A4" : "QSPEC_STREAM_MAX_W4A16") == 0) {
      const int v = value ? atoi(value) : 0;
      // the verify-mode streaming kernel exists for at most two 16-token tiles per workgroup
      o.stream_max[w4a4] = (v >= 32 && v <= (w4a4 ? 128 : 32)) ? v : 0;
      return true;
    }
    if (strcmp(name, w4a4 ? "QSPEC_TILE_W4A4" : "QSPEC_TILE_W4A16") == 0) {
      int* f = o.tile[w4a4];
      o.tile_set[w4a4] = value && sscanf(value, "%d,%d", &f[0], &f[1]) == 2;
      return true;
    }
  }
  return false;
}

constexpr const char* kOverrideNames[] = {"QSPEC_KERNEL", "QSPEC_STREAM_W4A4", "QSPEC_STREAM_W4A16",
                                          "QSPEC_STREAM_MAX_W4A4", "QSPEC_STREAM_MAX_W4A16",
                                          "QSPEC_TILE_W4A4", "QSPEC_TILE_W4A16", "QSPEC_MLP_SPIN"};

PlanOverrides& overrides() {
  static PlanOverrides o = [] {
    PlanOverrides init;
    for (const char* name : kOverrideNames)
      if (const char* e = getenv(name)) apply_override(init, name, e);
    return init;
  }();
  return o;
}

bool use_generic() { return overrides().generic; }

// ---------------------------------------------------------------- streaming (small-M) kernel
constexpr int kStreamMaxM = 32;
constexpr int kStreamMaxM4 = 64;

constexpr size_t kTicketBytes = 16384;                 // head of the workspace: arrival counters
constexpr int kMaxTickets = (int)(kTicketBytes / 4);

// Plan of the streaming kernel: NT adjacent n-tiles per workgroup, S K-slices, ms
// token-row blocks.  A pure function of (mode, M, N, K), so that qspec_workspace_bytes
// and the GEMM entry points agree.  QSPEC_STREAM_W4A4 / QSPEC_STREAM_W4A16 = "NT,S" or
// "NT,S,MS" override the heuristic (benchmark A/B only).
struct StreamPlan {
  int nt, S, blocks;
  int ms;       // token-row blocks (gridDim.y); block y owns rows y*16*tm .. (y+1)*16*tm - 1
  int tm;       // 16-token tiles per workgroup (the kernel's TM)
};
inline int stream_tm(int M) { return M <= 16 ? 1 : M <= 32 ? 2 : M <= 64 ? 4 : 8; }   // 16-token tiles that cover M rows
constexpr int kStreamNts[] = {1, 2, 3, 4, 6};
inline bool stream_nt_ok(int nt, int tm) {
  for (int v : kStreamNts) if (v == nt) return nt * tm <= 16;      // 4 accumulator registers per tile pair; beyond 64 the kernel spills
  return false;
}
// tiles per workgroup when the rows are dealt to ms blocks: ceil(M / ms) rows, in whole tiles
inline int stream_tm_split(int M, int ms) { return stream_tm(16 * (((M + ms - 1) / ms + 15) / 16)); }

// Largest M the streaming kernels take without token-row blocks: 32 verify-mode tokens, 64
// draft-mode tokens (a draft-mode activation operand is a quarter of a verify-mode one).
// The QSPEC_STREAM_MAX_* overrides replace the bound (benchmark A/B only).
int stream_base_max(bool w4a4) {
  const int forced = overrides().stream_max[w4a4 ? 1 : 0];
  return forced ? forced : (w4a4 ? kStreamMaxM4 : kStreamMaxM);
}

// Up to 128 tokens on layers no larger than 8192 x 8192 the streaming kernel with token-row
// blocks beats the tiled kernels when ONE round of workgroups covers the problem (the
// tiled kernels have too few output blocks to fill the chip there and fall back on
// K-slices): measured 4096 x 4096 at 128 tokens 16.0 -> 9.7 us (draft) and 15.5 -> 12.4 us
// (verify), 8192 x 8192 at 128 draft tokens 31.5 -> 27.1 us; with longer K or more than
// one round the tiled kernels win.  Picks tiles per workgroup, 16-token tiles per row
// block and the number of row blocks by the cost model of plan_stream; false: no such plan.
bool plan_wide_stream(bool w4a4, int M, int N, int K, int* nt_out, int* tm_out, int* ms_out) {
  if (M > 128 || N > 8192 || K > 8192) return false;
  const int tiles = N / 16;
  const double c = w4a4 ? 1.5 : 1.6;
  double best = 1e30;
  bool found = false;
  for (int tm = 1; tm <= (w4a4 ? 8 : 2); tm *= 2) {
    const int ms = (M + 16 * tm - 1) / (16 * tm);
    if (ms < 2 || ms > 8) continue;
    for (int v : kStreamNts) {
      if (!stream_nt_ok(v, tm)) continue;
      if (((tiles + v - 1) / v) * ms > kNumCU) continue;
      const double cost = v + c * tm;
      if (cost < best - 1e-9 || (cost < best + 1e-9 && v > *nt_out)) { best = cost; *nt_out = v; *tm_out = tm; *ms_out = ms; found = true; }
    }
  }
  return found;
}

StreamPlan plan_stream(bool w4a4, int M, int N, int K) {
  const int tiles = N / 16, G = K / kGroup;
  const PlanOverrides& ov = overrides();
  const int nf = ov.stream_fields[w4a4 ? 1 : 0];
  int nt = ov.stream[w4a4 ? 1 : 0][0], S = ov.stream[w4a4 ? 1 : 0][1], ms = ov.stream[w4a4 ? 1 : 0][2], tm_wide = 0;
  bool forced = nf >= 2 && S >= 1 && S <= G;
  if (nf < 3) ms = 1;
  if (forced && ms > 1) forced = S == 1 && (ms == 2 || ms == 4 || ms == 8);
  // a forced plan must have an instance and its row blocks must cover all M rows
  if (forced) forced = stream_nt_ok(nt, stream_tm_split(M, ms)) && (w4a4 || stream_tm_split(M, ms) <= 2) &&
                       (long long)ms * 16 * stream_tm_split(M, ms) >= M;
  if (!forced) { nt = 0; S = 0; ms = 1; }
  if (!forced && M > stream_base_max(w4a4)) {
    StreamPlan none{};                                   // nt == 0: no streaming plan, the tiled kernels take it
    if (!plan_wide_stream(w4a4, M, N, K, &nt, &tm_wide, &ms)) return none;
    S = 1;
  } else if (!forced) {
    // Cost of a plan, in units of one weight tile (1 KB from HBM) per wavefront:
    // rounds over the 256 compute units x groups per wavefront x (NT weight tiles +
    // the activation operand of the group, which comes from L2 and is re-used for
    // the NT tiles).  K-slices are never chosen here: measured on MI355X, the
    // exchange (write-through stores, a ticket, S dependent trips to memory) costs
    // 4 to 10 us, more than any of these launches saves; the path stays available
    // to the override and is covered by the tests.
    ms = 1;
    const int tm = stream_tm(M);
    const double act = w4a4 ? 0.4 * tm : 1.6 * tm;
    double best = 1e30;
    for (int s = 1; s <= 1; s *= 2) {
      for (int v : kStreamNts) {
        if (!stream_nt_ok(v, tm)) continue;
        const int blocks = (tiles + v - 1) / v;
        if (s > 1 && blocks > kMaxTickets) continue;
        const int rounds = (blocks * s + kNumCU - 1) / kNumCU;
        const int per_wave = ((G + s - 1) / s + kStreamWaves - 1) / kStreamWaves;
        const double cost = rounds * (per_wave * (v + act) + (s > 1 ? 0.25 * s * v * tm + 2.0 : 0.0));
        if (cost < best - 1e-9 || (cost < best + 1e-9 && v > nt)) { best = cost; nt = v; S = s; }
      }
    }
    // Two token-row blocks: with few tiles per workgroup the activation operand, not the
    // weights, is most of what a compute unit pulls through its L1 (every workgroup
    // reads ALL of x).  Dealing the rows to two workgroups that own twice the tiles
    // keeps the number of workgroups, halves that traffic, and lets the partner's
    // weight reads hit in L2 (both run on the same XCD: their ids differ by a multiple
    // of 8).  Measured on the 4096- and 5120-wide layers: 16-25 % less time where the
    // tile count per workgroup is below act/2 (act in weight-tile units: 1.6 per 16
    // verify-mode tokens, 1.5 per 16 draft-mode tokens for this decision), slower
    // on the wide layers, where the weights dominate already.
    if (tm >= 2) {
      const double act2 = (w4a4 ? 1.5 : 1.6) * tm;
      const int blocks1 = (tiles + nt - 1) / nt, blocks2 = ((tiles + 2 * nt - 1) / (2 * nt)) * 2;
      const bool same_rounds = (blocks2 + kNumCU - 1) / kNumCU <= (blocks1 + kNumCU - 1) / kNumCU;
      if (nt < act2 / 2 && stream_nt_ok(2 * nt, stream_tm_split(M, 2)) && same_rounds) { nt *= 2; ms = 2; }
    }
  }
  StreamPlan p{};
  p.nt = nt; p.S = S; p.blocks = (tiles + nt - 1) / nt; p.ms = ms;
  p.tm = tm_wide ? tm_wide : (ms > 1 ? stream_tm_split(M, ms) : stream_tm(M));
  return p;
}

inline size_t stream_ws_bytes(const StreamPlan& p) {
  return p.S > 1 ? kTicketBytes + (size_t)p.S * p.blocks * p.nt * p.tm * 1024 : 0;
}

bool tile_override(bool w4a4, int* shape, int* S);

bool use_stream(bool w4a4, int M, int N, int K) {
  if (M <= stream_base_max(w4a4)) {
    // Draft mode, 48 to 64 tokens, very wide layers (170 and more blocks of 128 outputs): the
    // tiled kernel is faster than the streaming one (22016 x 4096 at 64 tokens 26.8 -> 23.4 us,
    // 27648 x 5120: 36.4 -> 29.2, 57344 x 8192: 101.5 -> 68.4; at 48 tokens equal or better;
    // narrower layers stay with the streaming kernel: 12288 x 4096 at 64 tokens 13.7 vs 17.3 us)
    const PlanOverrides& ov = overrides();
    const bool wide_draft = w4a4 && M >= 48 && N >= 170 * 128 && ov.stream_fields[1] == 0 && ov.stream_max[1] == 0;
    return !wide_draft;
  }
  int shape, S;
  if (tile_override(w4a4, &shape, &S)) return false;      // a forced tile shape means the tiled kernel
  return plan_stream(w4a4, M, N, K).nt > 0;
}

// Launch the instance <mode, TM, NT> of a streaming plan.  A (TM, NT) pair that is not
// instantiated (a forced plan can name one) is refused: nothing is launched.
template <bool W4A4, int TM>
int launch_stream_tm(const StreamArgs& a, const StreamPlan& plan, hipStream_t s) {
  dim3 grid(plan.blocks * plan.S, plan.ms), block(kStreamWaves * 64);
  switch (plan.nt) {
    case 1: hipLaunchKernelGGL((gemm_stream_kernel<W4A4, TM, 1>), grid, block, 0, s, a); return QSPEC_OK;
    case 2: hipLaunchKernelGGL((gemm_stream_kernel<W4A4, TM, 2>), grid, block, 0, s, a); return QSPEC_OK;
    case 3:
      if constexpr (TM <= 4) { hipLaunchKernelGGL((gemm_stream_kernel<W4A4, TM, 3>), grid, block, 0, s, a); return QSPEC_OK; }
      return QSPEC_ERR_UNSUPPORTED;
    case 4:
      if constexpr (TM <= 4) { hipLaunchKernelGGL((gemm_stream_kernel<W4A4, TM, 4>), grid, block, 0, s, a); return QSPEC_OK; }
      return QSPEC_ERR_UNSUPPORTED;
    case 6:
      if constexpr (TM <= 2) { hipLaunchKernelGGL((gemm_stream_kernel<W4A4, TM, 6>), grid, block, 0, s, a); return QSPEC_OK; }
      return QSPEC_ERR_UNSUPPORTED;
    default: return QSPEC_ERR_UNSUPPORTED;
  }
}

template <bool W4A4>
int launch_stream(StreamArgs a, void* workspace, hipStream_t s) {
  const StreamPlan plan = plan_stream(W4A4, a.M, a.N, a.K);
  if ((long long)plan.ms * 16 * plan.tm < a.M) return QSPEC_ERR_UNSUPPORTED;      // the row blocks must cover M
  a.S = plan.S;
  a.tickets = static_cast<unsigned*>(workspace);
  a.ws = plan.S > 1 ? reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + kTicketBytes) : nullptr;
  switch (plan.tm) {
    case 1: return launch_stream_tm<W4A4, 1>(a, plan, s);
    case 2: return launch_stream_tm<W4A4, 2>(a, plan, s);
    case 4: if constexpr (W4A4) return launch_stream_tm<true, 4>(a, plan, s); else return QSPEC_ERR_UNSUPPORTED;
    case 8: if constexpr (W4A4) return launch_stream_tm<true, 8>(a, plan, s); else return QSPEC_ERR_UNSUPPORTED;
    default: return QSPEC_ERR_UNSUPPORTED;
  }
}

// ---------------------------------------------------------------- tiled (M > 32) kernels
// Workgroup shapes the tiled kernels are instantiated for: TN x TMW MFMA tiles per
// wavefront, WGN x WGM wavefronts per workgroup, weight ring of NW groups and NS
// activation stages (verify mode), OCC workgroups per compute unit (the register budget the compiler is held to).
struct TileShape { int TN, TMW, WGN, WGM, NW, NS, OCC; };
constexpr TileShape kShapes16[] = {     // verify mode (gemm_tile16w_kernel): TN, TMW count 32 x 32 tiles
    {1, 4, 4, 1, 4, 2, 2},   // 0: 128 outputs x 128 tokens
    {2, 2, 4, 1, 4, 4, 2},   // 1: 256 x 64, four activation stages
    {1, 2, 4, 1, 4, 2, 3},   // 2: 128 x 64, three workgroups per compute unit
    {1, 2, 4, 1, 4, 4, 2},   // 3: 128 x 64, four activation stages
    {1, 4, 8, 1, 4, 2, 1},   // 4: 256 x 128, eight wavefronts, one workgroup per compute unit
    {1, 4, 8, 1, 4, 4, 1},   // 5: 256 x 128, four activation stages
    {1, 2, 8, 1, 4, 4, 1},   // 6: 256 x 64, eight wavefronts, four activation stages
};
constexpr TileShape kShapes4[] = {      // draft mode (gemm_tile4w_kernel): TN, TMW count 32 x 32 tiles; NW = NS = 3
    {1, 4, 4, 1, 3, 3, 2},   // 0: 128 outputs x 128 tokens
    {1, 2, 4, 1, 3, 3, 2},   // 1: 128 x 64
    {1, 2, 2, 1, 3, 3, 2},   // 2: 64 x 64
    {1, 4, 8, 1, 3, 3, 1},   // 3: 256 x 128, eight wavefronts, one workgroup per compute unit
};
constexpr int kNumTileShapes = 4;
constexpr int kNumShapes16 = 7;
struct TilePlan {
  int shape;      // index into the mode's shape table
  int S;          // K-slices
  int nb, mb;     // output blocks
};

inline const TileShape& shape_of(bool w4a4, int i) { return w4a4 ? kShapes4[i] : kShapes16[i]; }

// QSPEC_TILE_W4A4 / QSPEC_TILE_W4A16 = "shape,S" override the heuristic (benchmark A/B only).
bool tile_override(bool w4a4, int* shape, int* S) {
  const PlanOverrides& ov = overrides();
  if (!ov.tile_set[w4a4 ? 1 : 0]) return false;
  *shape = ov.tile[w4a4 ? 1 : 0][0];
  *S = ov.tile[w4a4 ? 1 : 0][1];
  return *shape >= 0 && *shape < (w4a4 ? kNumTileShapes : kNumShapes16) && *S >= 1;
}

// Pure function of (mode, M, N, K): qspec_workspace_bytes and the GEMM entry points agree.
TilePlan plan_tile(bool w4a4, int M, int N, int K) {
  const int G = K / kGroup;
  TilePlan p{};
  int shape = 0, S = 1;
  if (!tile_override(w4a4, &shape, &S)) {
    // Both rules below come from sweeps over the Llama-shaped layers on the MI355X; the
    // figures quoted are microseconds per call before -> after the rule.
    bool s_chosen = false;
    if (w4a4) {
      // Two block sizes, 128 x 128 (a weight operand feeds four token tiles) and 128 x 64, and up
      // to four K-slices: the plan that comes closest to filling the 512 places of the chip
      // (two workgroups per compute unit) in ONE round wins.  From sweeps over the Llama-shaped
      // layers at 64 to 512 tokens: 13824 -> 5120 at 512 tokens 79.5 us (128 x 64, unsliced, 320
      // workgroups) -> 63.0 (128 x 128 in three slices, 480); 28672 -> 8192 at 384: 160 -> 140;
      // 10240 x 8192 at 256: 49.5 -> 44.9; at 128: 35.7 -> 28.4.  Ties go to the larger block when
      // its slices keep at least 48 groups, else to the plan with fewer slices (the exchange costs
      // 4-8 us).  Problems too large for one round run unsliced, on 128 x 128 blocks from 420
      // blocks on (27648 x 5120 at 256 tokens, 432 blocks: 70.0 -> 60.7 us).
      const int nb128 = (N + 127) / 128;
      const int blocks[2] = {nb128 * ((M + 127) / 128), nb128 * ((M + 63) / 64)};
      const int places = 2 * kNumCU;
      int sl[2] = {1, 1};
      double fill[2] = {-1.0, -1.0};
      for (int i = 0; i < 2; ++i) {
        if (blocks[i] > places || (i == 0 && M <= 64)) continue;       // (a 128-token block is half empty at 64 tokens)
        int c = places / blocks[i];
        if (c > 4) c = 4;
        // (slices of fewer than 20 groups lose to the unsliced plan even at half the fill: 4096 x
        // 4096 at 512 tokens, two slices of 16 groups 21.4 us, unsliced 18.8; 12288 x 4096 at 128:
        // 21.1 against 19.5; slices of 21 groups win: 10240 x 8192 at 128 tokens, three slices 29.0 us,
        // two 33.6, unsliced 39.3)
        while (c > 1 && G / c < 20) --c;
        // (but a chip left less than half full takes slices down to 12 groups, up to that half:
        // 4096 x 4096 at 256 tokens, 128 blocks: 18.6 us unsliced, 15.7 in two slices of 16)
        {
          int c2 = places / 2 / blocks[i];
          if (c2 > 4) c2 = 4;
          while (c2 > 1 && G / c2 < 12) --c2;
          if (c2 > c) c = c2;
        }
        sl[i] = c;
        fill[i] = (double)blocks[i] * c / places;
      }
      if (fill[0] < 0 && fill[1] < 0) {
        shape = (M > 64 && blocks[0] >= 420) ? 0 : 1;
        S = 1;
      } else if (fill[1] < 0) {
        shape = blocks[0] >= 420 ? 0 : 1;
        S = 1;
      } else if (fill[0] < 0) {
        shape = 1;
        S = sl[1];
      } else {
        const double d = fill[0] - fill[1];
        if (d > 0.05) shape = 0;
        else if (d < -0.05) shape = 1;
        else shape = (G / sl[0] >= 48 || sl[0] <= sl[1]) ? 0 : 1;
        S = sl[shape];
        // a very long K carries twice the slices even past one round (28672 -> 8192 at 384
        // tokens: two slices 148.7 us, four 139.8)
        if (fill[shape] <= 0.75 && S == 2 && G / 4 >= 48) S = 4;
      }
      // 256 x 128 blocks on eight wavefronts, one workgroup per compute unit: the activation
      // codes of a group are widened and staged once for twice the outputs, and half the
      // activation bytes enter the unit.  As in the verify mode a ragged round costs a whole
      // round, so (both plans timed alternately in one process): one round at least 60 % full
      // unsliced (57344 x 8192 at 128 tokens, 224 blocks: 115.4 -> 105.0 us; 10240 x 8192 at 512,
      // 160 blocks: 84.8 -> 72.7; 22016 x 4096 at 256, 172 blocks: 46.6 -> 40.9; 15360 x 5120 at
      // 384: 57.7 -> 50.0), or at least 90 % full in up to three K-slices of at least 21 groups
      // or four of at least 48 (28672 -> 8192 at 512 tokens, two slices: 179.6 -> 164.7; at 256,
      // four: 101.9 -> 93.8; 10240 x 8192 at 256, three: 47.4 -> 44.3; slices of 16 groups lose:
      // 12288 x 4096 at 256 tokens 31.6 -> 34.5), or up to two rounds at least 85 % full (57344 x
      // 8192 at 256 tokens: 188.3 -> 176.8; 1.3 rounds lose 6-8 %).
      const int mb128 = (M + 127) / 128;
      if (M > 96 && M * 4 >= mb128 * 128 * 3) {
        const int blocks3 = ((N + 255) / 256) * mb128;
        if (blocks3 <= kNumCU) {
          int c = kNumCU / blocks3;
          if (c > 4) c = 4;
          if (c == 4 && G / 4 < 48) c = 3;             // (four slices of 21 groups: 4096 x 11008 at 512 tokens 45.1 -> 47.1 us)
          while (c > 1 && G / c < 21) --c;
          const int full = blocks3 * c * 100;
          if (c == 1 ? full >= kNumCU * 60 : full >= kNumCU * 90) { shape = 3; S = c; }
        } else {
          // (from three rounds on 95 %: 57344 x 8192 at 512 tokens, 3.5 rounds, equal with packed
          // codes and 309 against 279 us on 128 x 128 blocks with the widened format)
          const int rounds3 = (blocks3 + kNumCU - 1) / kNumCU;
          if (blocks3 * 100 >= rounds3 * kNumCU * (rounds3 <= 2 ? 85 : 95)) { shape = 3; S = 1; }
        }
      }
      s_chosen = true;
    } else {
      const int blocks128 = ((N + 127) / 128) * ((M + 127) / 128);
      const int blocks64 = ((N + 127) / 128) * ((M + 63) / 64);
      // 128 x 64 blocks: with at most one workgroup per compute unit the instance with
      // four activation stages hides more latency (measured 23.5 -> 21.4 us at 128 tokens
      // on 12288 x 4096); with more workgroups than compute units the three-per-unit instance
      // (128 x 128 blocks also from 120 blocks on when K is long enough for the two K-slices that
      // then fill the chip: 28672 -> 8192 at 512 tokens 254 -> 236 us, at 256 tokens 141 -> 134 us;
      // 11008 -> 4096 at 512: 60.3 -> 58.8 us; 13824 -> 5120 at 384: 71.0 -> 68.9 us)
      // (and from one 128 x 128 block per compute unit on: 8192 x 8192 at 512 tokens, 256 blocks:
      // 74.1 us on 512 blocks of 128 x 64, 73.1 on 256 x 128 in two K-slices, 70.7 here)
      const bool big = M > 64 && (blocks128 >= 2 * kNumCU || (blocks128 >= 120 && G >= 86) || (M >= 128 && blocks128 >= kNumCU));
      shape = big ? 0 : (blocks64 <= kNumCU ? 3 : 2);
      // 256 x 128 blocks on eight wavefronts (one workgroup per compute unit) halve the
      // activation bytes a compute unit pulls per output (the global -> LDS transfers of x are
      // 19 % of the 128 x 128 instance's time), but with one workgroup per unit a ragged round
      // costs a whole round.  Taken when ONE round is at least 58 % full, counting the two
      // K-slices a long K allows (10240 x 8192 at 512 tokens, 160 blocks: 103.4 -> 94.5 us;
      // 15360 x 5120 at 384, 180 blocks: 70.8 -> 66.5; 12288 x 4096 at 512, 192 blocks: 59.6 ->
      // 57.5; 28672 -> 8192 at 512, 128 blocks in two slices: 241 -> 229; 128 blocks unsliced
      // lose: 8192 x 8192 at 512 tokens 75 -> 89 us), or when several rounds are at least 85 %
      // full (57344 x 8192 at 256 tokens, 448 blocks: 255 -> 236 us; at 512 tokens, 896 blocks
      // = 3.5 rounds: equal; 324 and 344 blocks lose 10 %).
      const int blocks256 = ((N + 255) / 256) * ((M + 127) / 128);
      const int rounds256 = (blocks256 + kNumCU - 1) / kNumCU;
      if (M >= 128) {                                  // (57344 x 8192 at 128 tokens, 224 blocks: 135 -> 123 us)
        int s256 = (M >= 256 && blocks256 * 2 <= kNumCU && G >= 64) ? 2 : 1;      // the slices the rule below will cut
        if (s256 == 2 && blocks128 >= kNumCU && G < 86) s256 = 1;                 // (unsliced 128 x 128 blocks fill the chip: see above)
        // (from three rounds on they must be 95 % full: 57344 x 8192 at 512 tokens, 3.5 rounds: 441 us, 128 x 128 blocks 435)
        const int need_pct = rounds256 <= 2 ? 85 : 95;
        if (rounds256 == 1 ? blocks256 * s256 >= 150 : blocks256 * 100 >= rounds256 * kNumCU * need_pct) shape = 4;
      }
    }
    // K-slices (measured: the exchange costs 4-8 us).  They pay while ALL workgroups
    // still run at once on compute units of their own: S = the largest count (not only
    // powers of two: slices are cut proportionally) with blocks * S <= 256 and at least 8
    // groups per slice.  Beyond that the extra workgroups queue behind the first ones
    // and only the exchange is added (172 blocks of a 22016-wide layer at 64 tokens:
    // 25.2 us unsliced, 29.6 us in two slices; 128 blocks of 8192 x 8192 at 128 tokens:
    // 40.9 -> 29.7 us).  With very long K (at least 43 groups per slice after doubling:
    // 11008 -> 4096 at 512 tokens 60.3 -> 58.8 us; 32 or 40 groups per slice lose, 8192 x 8192
    // at 512 tokens 70.7 -> 75.4, 8192 x 10240: 93.0 -> 97.0) doubling still pays while the
    // workgroups stay resident together (two per unit).
    if (!s_chosen) {
      const TileShape& t0 = shape_of(w4a4, shape);
      const int blocks = ((N + 32 * t0.TN * t0.WGN - 1) / (32 * t0.TN * t0.WGN)) * ((M + 32 * t0.TMW * t0.WGM - 1) / (32 * t0.TMW * t0.WGM));
      const int resident = t0.OCC >= 2 ? 2 * kNumCU : kNumCU;     // workgroups that run at once
      S = kNumCU / blocks;
      if (S > 8) S = 8;
      while (S > 1 && G / S < 8) --S;
      if (S < 1) S = 1;
      // (only while the doubled count still fits)
      while (S < 8 && blocks * S * 2 <= resident && G / (2 * S) >= 43) S *= 2;
    }
  }
  const TileShape& t = shape_of(w4a4, shape);
  const int edge = 32;                  // MFMA tile edge
  const int bn = edge * t.TN * t.WGN, bm = edge * t.TMW * t.WGM;
  p.shape = shape;
  p.nb = (N + bn - 1) / bn;
  p.mb = (M + bm - 1) / bm;
  if (S > G) S = G;
  if (p.nb * p.mb > kMaxTickets) S = 1;
  p.S = S;
  return p;
}

inline size_t plan_ws_bytes(bool w4a4, const TilePlan& p) {
  if (p.S <= 1) return 0;
  const TileShape& t = shape_of(w4a4, p.shape);
  const int edge = 32;
  const size_t block_floats = (size_t)(edge * t.TN * t.WGN) * (edge * t.TMW * t.WGM);   // whole blocks, ragged or not
  return kTicketBytes + (size_t)p.S * p.nb * p.mb * block_floats * 4;
}

template <int PN, int PM, int WGN, int WGM, int OCC>
int launch_tile4w_inst(const TileArgs& a, bool wide, hipStream_t s) {
  if (wide) hipLaunchKernelGGL((gemm_tile4w_kernel<PN, PM, WGN, WGM, OCC, true>), dim3(a.nb * a.mb * a.S),
                               dim3(64 * WGN * WGM), 0, s, a);
  else hipLaunchKernelGGL((gemm_tile4w_kernel<PN, PM, WGN, WGM, OCC, false>), dim3(a.nb * a.mb * a.S),
                          dim3(64 * WGN * WGM), 0, s, a);
  return QSPEC_OK;
}

template <int PN, int PM, int WGN, int WGM, int NW, int NS, int OCC>
int launch_tile16w_inst(const TileArgs& a, hipStream_t s) {
  hipLaunchKernelGGL((gemm_tile16w_kernel<PN, PM, WGN, WGM, NW, NS, OCC>), dim3(a.nb * a.mb * a.S),
                     dim3(64 * WGN * WGM), 0, s, a);
  return QSPEC_OK;
}

template <bool W4A4>
int launch_tile(const TilePlan& plan, TileArgs a, void* workspace, hipStream_t s, bool wide = false) {
  a.S = plan.S; a.nb = plan.nb; a.mb = plan.mb;
  a.tickets = static_cast<unsigned*>(workspace);
  a.ws = plan.S > 1 ? reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + kTicketBytes) : nullptr;
  if (W4A4) {
    switch (plan.shape) {
      case 0: return launch_tile4w_inst<1, 4, 4, 1, 2>(a, wide, s);
      case 1: return launch_tile4w_inst<1, 2, 4, 1, 2>(a, wide, s);
      case 2: return launch_tile4w_inst<1, 2, 2, 1, 2>(a, wide, s);
      default: return launch_tile4w_inst<1, 4, 8, 1, 1>(a, wide, s);
    }
  }
  switch (plan.shape) {
    case 0: return launch_tile16w_inst<1, 4, 4, 1, 4, 2, 2>(a, s);
    case 1: return launch_tile16w_inst<2, 2, 4, 1, 4, 4, 2>(a, s);
    case 2: return launch_tile16w_inst<1, 2, 4, 1, 4, 2, 3>(a, s);
    case 3: return launch_tile16w_inst<1, 2, 4, 1, 4, 4, 2>(a, s);
    case 4: return launch_tile16w_inst<1, 4, 8, 1, 4, 2, 1>(a, s);
    case 5: return launch_tile16w_inst<1, 4, 8, 1, 4, 4, 1>(a, s);
    default: return launch_tile16w_inst<1, 2, 8, 1, 4, 4, 1>(a, s);
  }
}

// ---------------------------------------------------------------- acceptance (after the verify pass)
// Chunks per logits row: about 4096 logits per workgroup, at most one chunk per lane
// of the second kernel.  A pure function of V.
struct ArgmaxPlan { int C, chunk; };
ArgmaxPlan plan_argmax(int V) {
  int C = (V + 4095) / 4096;
  if (C > kArgmaxMaxChunks) C = kArgmaxMaxChunks;
  if (C < 1) C = 1;
  int chunk = ((V + C - 1) / C + 7) & ~7;
  C = (V + chunk - 1) / chunk;
  return ArgmaxPlan{C, chunk};
}

// Device address of `scratch` on the current device, looked up once per device (with that
// device current) and kept.  nullptr: the lookup failed.
constexpr int kMaxDevices = 64;
void* scratch_of_device(int* status) {
  static void* ptr[kMaxDevices];
  static bool known[kMaxDevices];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { *status = QSPEC_ERR_HIP; return nullptr; }
  if (!known[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      *status = QSPEC_ERR_HIP;
      return nullptr;
    }
    ptr[dev] = p;
    known[dev] = true;
  }
  *status = QSPEC_OK;
  return ptr[dev];
}

// Zero the arrival counters at the head of a scratch area (a kernel, not a memset: the
// launch may be captured into a graph).
__global__ __launch_bounds__(256) void clear_tickets_kernel(unsigned* tickets, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) tickets[i] = 0u;
}

// ---------------------------------------------------------------- persistent draft-pass MLP
// Workgroups of the persistent launch: one per compute unit of the current device (looked up
// once per device).  0: the query failed.
int mlp_workgroups() {
  static int cus[kMaxDevices];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
  if (cus[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 0;
    cus[dev] = n;
  }
  return cus[dev];
}

constexpr size_t kMlpCounterBytes = 16384;
constexpr unsigned kMlpDefaultSpin = 200000;      // polls of about a microsecond each before a workgroup gives up

// Tiles per workgroup of the two projections for nwg workgroups; false: the shape does not fit the kernel.
bool mlp_plan(int M, int H, int I, int nwg, int* nt1, int* nt2) {
  if (M < 1 || M > 32 || nwg < 1) return false;
  const int tiles1 = 2 * I / 16, tiles2 = H / 16, G2 = I / kGroup;
  const int need1 = (tiles1 + nwg - 1) / nwg, need2 = (tiles2 + nwg - 1) / nwg;
  *nt1 = need1 <= 2 ? 2 : need1 <= 4 ? 4 : 6;
  *nt2 = need2 <= 1 ? 1 : 2;
  if (need1 > 6 || need2 > 2) return false;
  if (need2 * G2 > kMlpWBufTiles) return false;               // the down-projection tiles of a workgroup must fit LDS
  if ((size_t)(G2 + 2) * sizeof(unsigned) > kMlpCounterBytes) return false;
  return true;
}

template <int TM, int NT1>
int launch_mlp_nt2(const MlpArgs& a, int nt2, int nwg, hipStream_t s) {
  if (nt2 == 1) hipLaunchKernelGGL((mlp_draft_kernel<TM, NT1, 1>), dim3(nwg), dim3(kStreamWaves * 64), 0, s, a);
  else hipLaunchKernelGGL((mlp_draft_kernel<TM, NT1, 2>), dim3(nwg), dim3(kStreamWaves * 64), 0, s, a);
  return QSPEC_OK;
}
template <int TM>
int launch_mlp(const MlpArgs& a, int nt1, int nt2, int nwg, hipStream_t s) {
  switch (nt1) {
    case 2: return launch_mlp_nt2<TM, 2>(a, nt2, nwg, s);
    case 4: return launch_mlp_nt2<TM, 4>(a, nt2, nwg, s);
    case 6: return launch_mlp_nt2<TM, 6>(a, nt2, nwg, s);
    default: return QSPEC_ERR_UNSUPPORTED;
  }
}

inline bool misaligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) != 0; }

inline int check_accept_shape(int B, int gamma, int V) {
  if (B < 1 || gamma < 1 || V < 1) return QSPEC_ERR_SHAPE;
  if ((long long)B * (gamma + 1) > 65535) return QSPEC_ERR_SHAPE;        // one grid row per logits row
  return QSPEC_OK;
}

}  // namespace

extern "C" {

const char* qspec_status_string(int status) {
  switch (status) {
    case QSPEC_OK: return "ok";
    case QSPEC_ERR_NULL: return "null pointer";
    case QSPEC_ERR_SHAPE: return "unsupported shape or argument value (need group == 128, K % 128 == 0, N % 16 == 0, M >= 1, every buffer below 2 GiB; see the entry point for its other arguments)";
    case QSPEC_ERR_ALIGN: return "pointer not 16-byte aligned";
    case QSPEC_ERR_WORKSPACE: return "workspace too small";
    case QSPEC_ERR_HIP: return "HIP runtime error";
    case QSPEC_ERR_UNSUPPORTED: return "device is not gfx950, a forced plan names a kernel instance that does not exist, or the shape lies outside what this variant entry point takes";
    default: return "unknown status";
  }
}

int qspec_version(void) { return 1000; }

size_t qspec_packed_weight_bytes(int N, int K, int group) {
  if (check_shape(1, N, K, group) != QSPEC_OK) return 0;
  return (size_t)N * K / 2 + (size_t)N * (K / kGroup) * 2;
}

size_t qspec_workspace_bytes(int M, int N, int K, int group) {
  if (check_shape(M, N, K, group) != QSPEC_OK) return 0;
  // the larger of what the two modes need for this shape
  size_t need[2];
  for (int w4a4 = 0; w4a4 < 2; ++w4a4) {
    if (use_stream(w4a4 != 0, M, N, K)) need[w4a4] = stream_ws_bytes(plan_stream(w4a4 != 0, M, N, K));
    else if (use_generic()) need[w4a4] = 0;
    else need[w4a4] = plan_ws_bytes(w4a4 != 0, plan_tile(w4a4 != 0, M, N, K));
  }
  return need[0] > need[1] ? need[0] : need[1];
}

int qspec_pack_weights(const int8_t* codes, const void* scales_f16, int N, int K, int group,
                       void* packed, void* stream) {
  if (!codes || !scales_f16 || !packed) return QSPEC_ERR_NULL;
  if (int st = check_shape(1, N, K, group)) return st;
  if (misaligned(codes) || misaligned(scales_f16) || misaligned(packed)) return QSPEC_ERR_ALIGN;
  if (int st = check_device()) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int G = K / kGroup;
  const size_t n_words = (size_t)N * K / 8;
  hipLaunchKernelGGL(pack_codes_kernel, dim3(blocks_for(n_words, 256)), dim3(256), 0, s,
                     codes, static_cast<uint32_t*>(packed), N, K, G);
  uint16_t* sc_out = reinterpret_cast<uint16_t*>(static_cast<uint8_t*>(packed) + (size_t)N * K / 2);
  hipLaunchKernelGGL(transpose_scales_kernel, dim3(blocks_for((size_t)N * G, 256)), dim3(256), 0, s,
                     static_cast<const uint16_t*>(scales_f16), sc_out, N, G);
  return launch_status();
}

int qspec_unpack_weights(const void* packed, int N, int K, int group,
                         int8_t* codes, void* scales_f16, void* stream) {
  if (!codes || !scales_f16 || !packed) return QSPEC_ERR_NULL;
  if (int st = check_shape(1, N, K, group)) return st;
  if (misaligned(codes) || misaligned(scales_f16) || misaligned(packed)) return QSPEC_ERR_ALIGN;
  if (int st = check_device()) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int G = K / kGroup;
  const size_t n_words = (size_t)N * K / 8;
  hipLaunchKernelGGL(unpack_codes_kernel, dim3(blocks_for(n_words, 256)), dim3(256), 0, s,
                     static_cast<const uint32_t*>(packed), codes, N, K, G);
  // [G][N] -> [N][G] is the same transpose with the roles swapped
  hipLaunchKernelGGL(transpose_scales_kernel, dim3(blocks_for((size_t)N * G, 256)), dim3(256), 0, s,
                     blob_scales(packed, N, K), static_cast<uint16_t*>(scales_f16), G, N);
  return launch_status();
}

int qspec_quant_act(const void* x_f16, int M, int K, int group, uint8_t* qa, float* sa, void* stream) {
  if (!x_f16 || !qa || !sa) return QSPEC_ERR_NULL;
  if (int st = check_shape(M, kTileRows, K, group)) return st;
  if (misaligned(x_f16) || misaligned(qa) || misaligned(sa)) return QSPEC_ERR_ALIGN;
  if (int st = check_device()) return st;
  const size_t n_words = (size_t)M * K / 8;
  hipLaunchKernelGGL(quant_act_kernel, dim3(blocks_for(n_words, 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(x_f16),
                     reinterpret_cast<uint32_t*>(qa), sa, n_words);
  return launch_status();
}

int qspec_w4a4_takes_wide(int M, int N, int K, int group) {
  if (check_shape(M, N, K, group) != QSPEC_OK) return 0;
  return (!use_stream(true, M, N, K) && !use_generic()) ? 1 : 0;
}

int qspec_quant_act_wide(const void* x_f16, int M, int K, int group, int8_t* qa8, float* sa, void* stream) {
  if (!x_f16 || !qa8 || !sa) return QSPEC_ERR_NULL;
  if (int st = check_shape(M, kTileRows, K, group)) return st;
  if (misaligned(x_f16) || misaligned(qa8) || misaligned(sa)) return QSPEC_ERR_ALIGN;
  if (int st = check_device()) return st;
  const size_t n_words = (size_t)M * K / 8;
  hipLaunchKernelGGL(quant_act_wide_kernel, dim3(blocks_for(n_words, 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(x_f16),
                     reinterpret_cast<uint32_t*>(qa8), sa, n_words);
  return launch_status();
}

int qspec_rmsnorm_quant(const void* x_f16, const void* weight_f16, float eps, int M, int K, int group,
                        int rotate, uint8_t* qa, float* sa, void* h_f16, void* stream) {
  if (!x_f16 || !weight_f16 || !qa || !sa) return QSPEC_ERR_NULL;
  if (int st = check_shape(M, kTileRows, K, group)) return st;
  if (!(eps >= 0.0f) || !(eps <= 3.0e38f) || rotate < 0 || rotate > 3) return QSPEC_ERR_SHAPE;
  if (misaligned(x_f16) || misaligned(weight_f16) || misaligned(qa) || misaligned(sa) || misaligned(h_f16))
    return QSPEC_ERR_ALIGN;
  if (int st = check_device()) return st;
  const hipStream_t s = static_cast<hipStream_t>(stream);
  const uint4* x = static_cast<const uint4*>(x_f16);
  const uint4* w = static_cast<const uint4*>(weight_f16);
  uint32_t* words = reinterpret_cast<uint32_t*>(qa);
  uint4* h = static_cast<uint4*>(h_f16);
  // threads per row: one per 8 features up to 1024, whole wavefronts
  const int kw = K / 8;
  const int T = kw >= kRowMaxThreads ? kRowMaxThreads : (kw + 63) / 64 * 64;
  const int chunks = (kw + T - 1) / T;
  const double inv_K = 1.0 / (double)K;
  const dim3 grid(M), block(T);
  if (chunks <= 1) hipLaunchKernelGGL(rmsnorm_quant_kernel<1>, grid, block, 0, s, x, w, eps, K, inv_K, words, sa, h, rotate);
  else if (chunks <= 2) hipLaunchKernelGGL(rmsnorm_quant_kernel<2>, grid, block, 0, s, x, w, eps, K, inv_K, words, sa, h, rotate);
  else if (chunks <= 4) hipLaunchKernelGGL(rmsnorm_quant_kernel<4>, grid, block, 0, s, x, w, eps, K, inv_K, words, sa, h, rotate);
  else hipLaunchKernelGGL(rmsnorm_quant_kernel<0>, grid, block, 0, s, x, w, eps, K, inv_K, words, sa, h, rotate);
  return launch_status();
}

int qspec_silu_mul_quant(const void* gate_up_f16, int M, int I, int group,
                         int rotate, uint8_t* qa, float* sa, void* h_f16, void* stream) {
  if (!gate_up_f16 || !qa || !sa) return QSPEC_ERR_NULL;
  if (int st = check_shape(M, kTileRows, I, group)) return st;
  if (rotate < 0 || rotate > 3) return QSPEC_ERR_SHAPE;
  if (misaligned(gate_up_f16) || misaligned(qa) || misaligned(sa) || misaligned(h_f16)) return QSPEC_ERR_ALIGN;
  if (int st = check_device()) return st;
  const size_t n_words = (size_t)M * I / 8;
  hipLaunchKernelGGL(silu_mul_quant_kernel, dim3(blocks_for(n_words, 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(gate_up_f16), I / 8,
                     reinterpret_cast<uint32_t*>(qa), sa, static_cast<uint4*>(h_f16), n_words, rotate);
  return launch_status();
}

int qspec_hadamard_quant(const void* x_f16, int M, int K, int group,
                         uint8_t* qa, float* sa, void* h_f16, void* stream) {
  if (!x_f16 || !qa || !sa) return QSPEC_ERR_NULL;
  if (int st = check_shape(M, kTileRows, K, group)) return st;
  if (misaligned(x_f16) || misaligned(qa) || misaligned(sa) || misaligned(h_f16)) return QSPEC_ERR_ALIGN;
  if (int st = check_device()) return st;
  const size_t n_words = (size_t)M * K / 8;
  hipLaunchKernelGGL(hadamard_quant_kernel, dim3(blocks_for(n_words, 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(x_f16),
                     reinterpret_cast<uint32_t*>(qa), sa, static_cast<uint4*>(h_f16), n_words);
  return launch_status();
}

int qspec_reorder_quant(const void* x_f16, const int32_t* perm, int M, int K, int group,
                        int n_outlier_groups, uint8_t* qa, float* sa, void* h_f16, void* stream) {
  if (!x_f16 || !perm || !qa || !sa) return QSPEC_ERR_NULL;
  if (int st = check_shape(M, kTileRows, K, group)) return st;
  if (n_outlier_groups < 0 || n_outlier_groups > K / kGroup) return QSPEC_ERR_SHAPE;
  if (int st = check_shape(M, kTileRows, K + kGroup * n_outlier_groups, group)) return st;
  if (misaligned(x_f16) || misaligned(perm) || misaligned(qa) || misaligned(sa) || misaligned(h_f16))
    return QSPEC_ERR_ALIGN;
  if (int st = check_device()) return st;
  const size_t n_words = (size_t)M * K / 8;
  hipLaunchKernelGGL(reorder_quant_kernel, dim3(blocks_for(n_words, 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(x_f16), perm, K,
                     n_outlier_groups, reinterpret_cast<uint32_t*>(qa), sa, static_cast<uint4*>(h_f16), n_words);
  return launch_status();
}

int qspec_gemm_w4a4(const void* packed, const uint8_t* qa, const float* sa, int M, int N, int K, int group,
                    void* y_f16, void* workspace, size_t workspace_bytes, void* stream) {
  if (!packed || !qa || !sa || !y_f16) return QSPEC_ERR_NULL;
  if (int st = check_shape(M, N, K, group)) return st;
  if (misaligned(packed) || misaligned(qa) || misaligned(sa) || misaligned(y_f16)) return QSPEC_ERR_ALIGN;
  const size_t need = qspec_workspace_bytes(M, N, K, group);
  if (need > 0 && (!workspace || workspace_bytes < need)) return QSPEC_ERR_WORKSPACE;
  if (int st = check_device()) return st;
  GemmArgs a{};
  a.codes = static_cast<const uint4*>(packed);
  a.scalesT = blob_scales(packed, N, K);
  a.act = qa;
  a.sa = sa;
  a.y = static_cast<uint16_t*>(y_f16);
  a.M = M; a.N = N; a.K = K; a.G = K / kGroup;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (use_stream(true, M, N, K)) {
    StreamArgs st{};
    st.codes = a.codes; st.scalesT = a.scalesT; st.act = qa; st.sa = sa; st.y = a.y;
    st.M = M; st.N = N; st.K = K; st.G = a.G;
    if (int err = launch_stream<true>(st, workspace, s)) return err;
    return launch_status();
  }
  if (!use_generic()) {
    TileArgs t{};
    t.codes = a.codes; t.scalesT = a.scalesT; t.act = qa; t.sa = sa; t.y = a.y;
    t.M = M; t.N = N; t.K = K; t.G = a.G;
    if (int st = launch_tile<true>(plan_tile(true, M, N, K), t, workspace, s)) return st;
    return launch_status();
  }
  switch (pick_tm(M)) {
    case 1: launch_w4a4<1>(a, s); break;
    case 2: launch_w4a4<2>(a, s); break;
    case 4: launch_w4a4<4>(a, s); break;
    default: launch_w4a4<8>(a, s); break;
  }
  return launch_status();
}

int qspec_gemm_w4a4_wide(const void* packed, const int8_t* qa8, const float* sa, int M, int N, int K, int group,
                         void* y_f16, void* workspace, size_t workspace_bytes, void* stream) {
  if (!packed || !qa8 || !sa || !y_f16) return QSPEC_ERR_NULL;
  if (int st = check_shape(M, N, K, group)) return st;
  if (misaligned(packed) || misaligned(qa8) || misaligned(sa) || misaligned(y_f16)) return QSPEC_ERR_ALIGN;
  if (!qspec_w4a4_takes_wide(M, N, K, group)) return QSPEC_ERR_UNSUPPORTED;   // this shape runs on a kernel that reads packed codes
  const size_t need = qspec_workspace_bytes(M, N, K, group);
  if (need > 0 && (!workspace || workspace_bytes < need)) return QSPEC_ERR_WORKSPACE;
  if (int st = check_device()) return st;
  TileArgs t{};
  t.codes = static_cast<const uint4*>(packed);
  t.scalesT = blob_scales(packed, N, K);
  t.act = qa8;
  t.sa = sa;
  t.y = static_cast<uint16_t*>(y_f16);
  t.M = M; t.N = N; t.K = K; t.G = K / kGroup;
  if (int st = launch_tile<true>(plan_tile(true, M, N, K), t, workspace, static_cast<hipStream_t>(stream), true)) return st;
  return launch_status();
}

int qspec_gemm_w4a16(const void* packed, const void* x_f16, int M, int N, int K, int group,
                     void* y_f16, void* workspace, size_t workspace_bytes, void* stream) {
  if (!packed || !x_f16 || !y_f16) return QSPEC_ERR_NULL;
  if (int st = check_shape(M, N, K, group)) return st;
  if (misaligned(packed) || misaligned(x_f16) || misaligned(y_f16)) return QSPEC_ERR_ALIGN;
  const size_t need = qspec_workspace_bytes(M, N, K, group);
  if (need > 0 && (!workspace || workspace_bytes < need)) return QSPEC_ERR_WORKSPACE;
  if (int st = check_device()) return st;
  GemmArgs a{};
  a.codes = static_cast<const uint4*>(packed);
  a.scalesT = blob_scales(packed, N, K);
  a.act = x_f16;
  a.y = static_cast<uint16_t*>(y_f16);
  a.M = M; a.N = N; a.K = K; a.G = K / kGroup;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (use_stream(false, M, N, K)) {
    StreamArgs st{};
    st.codes = a.codes; st.scalesT = a.scalesT; st.act = x_f16; st.y = a.y;
    st.M = M; st.N = N; st.K = K; st.G = a.G;
    if (int err = launch_stream<false>(st, workspace, s)) return err;
    return launch_status();
  }
  if (!use_generic()) {
    TileArgs t{};
    t.codes = a.codes; t.scalesT = a.scalesT; t.act = x_f16; t.y = a.y;
    t.M = M; t.N = N; t.K = K; t.G = a.G;
    if (int st = launch_tile<false>(plan_tile(false, M, N, K), t, workspace, s)) return st;
    return launch_status();
  }
  switch (pick_tm(M)) {
    case 1: launch_w4a16<1>(a, s); break;
    case 2: launch_w4a16<2>(a, s); break;
    case 4: launch_w4a16<4>(a, s); break;
    default: launch_w4a16<8>(a, s); break;
  }
  return launch_status();
}

int qspec_gemm_w4a16_noalloc(const void* packed, const void* x_f16, int M, int N, int K, int group,
                             void* y_f16, void* stream) {
  if (!packed || !x_f16 || !y_f16) return QSPEC_ERR_NULL;
  if (int st = check_shape(M, N, K, group)) return st;
  if (misaligned(packed) || misaligned(x_f16) || misaligned(y_f16)) return QSPEC_ERR_ALIGN;
  const size_t need = qspec_workspace_bytes(M, N, K, group);
  if (need > kScratchBytes) return QSPEC_ERR_WORKSPACE;       // beyond the built-in scratch: use qspec_gemm_w4a16
  if (int st = check_device()) return st;
  int st = QSPEC_OK;
  void* ws = scratch_of_device(&st);
  if (!ws) return st;
  if (need > 0) {
    // the counters must start at zero whatever an earlier (possibly failed) call left
    hipLaunchKernelGGL(clear_tickets_kernel, dim3(kMaxTickets / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<unsigned*>(ws), kMaxTickets);
  }
  return qspec_gemm_w4a16(packed, x_f16, M, N, K, group, y_f16, ws, kScratchBytes, stream);
}

size_t qspec_mlp_draft_workspace_bytes(int M, int H, int I, int group) {
  if (check_shape(M, H, I, group) != QSPEC_OK || check_shape(M, 2 * I, H, group) != QSPEC_OK) return 0;
  return kMlpCounterBytes;
}

int qspec_mlp_draft(const void* packed_gate_up, const void* packed_down, const uint8_t* qa_h, const float* sa_h,
                    int M, int H, int I, int group, void* gate_up_f16, uint8_t* qa_i, float* sa_i, void* y_f16,
                    void* workspace, size_t workspace_bytes, int* status_word, void* stream) {
  if (!packed_gate_up || !packed_down || !qa_h || !sa_h || !gate_up_f16 || !qa_i || !sa_i || !y_f16 || !workspace || !status_word)
    return QSPEC_ERR_NULL;
  if (int st = check_shape(M, 2 * I, H, group)) return st;
  if (int st = check_shape(M, H, I, group)) return st;
  if (misaligned(packed_gate_up) || misaligned(packed_down) || misaligned(qa_h) || misaligned(sa_h) || misaligned(gate_up_f16) ||
      misaligned(qa_i) || misaligned(sa_i) || misaligned(y_f16) || misaligned(workspace) || misaligned4(status_word))
    return QSPEC_ERR_ALIGN;
  if (workspace_bytes < kMlpCounterBytes) return QSPEC_ERR_WORKSPACE;
  if (int st = check_device()) return st;
  const int nwg = mlp_workgroups();
  if (nwg <= 0) return QSPEC_ERR_HIP;
  int nt1 = 0, nt2 = 0;
  if (!mlp_plan(M, H, I, nwg, &nt1, &nt2)) return QSPEC_ERR_UNSUPPORTED;
  MlpArgs a{};
  a.codes1 = static_cast<const uint4*>(packed_gate_up);
  a.scales1T = blob_scales(packed_gate_up, 2 * I, H);
  a.qa_h = qa_h; a.sa_h = sa_h;
  a.y_gu = static_cast<uint16_t*>(gate_up_f16);
  a.qa_i = qa_i; a.sa_i = sa_i;
  a.codes2 = static_cast<const uint4*>(packed_down);
  a.scales2T = blob_scales(packed_down, H, I);
  a.y = static_cast<uint16_t*>(y_f16);
  a.counters = static_cast<unsigned*>(workspace);
  a.status = status_word;
  a.M = M; a.N1 = 2 * I; a.K1 = H; a.N2 = H; a.K2 = I;
  a.spin_limit = overrides().mlp_spin ? overrides().mlp_spin : kMlpDefaultSpin;   // QSPEC_MLP_SPIN: tests of the give-up path
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (int st = (M <= 16 ? launch_mlp<1>(a, nt1, nt2, nwg, s) : launch_mlp<2>(a, nt1, nt2, nwg, s))) return st;
  return launch_status();
}

int qspec_gemm_w4a4_partials(const void* packed, const uint8_t* qa, int M, int N, int K, int group,
                             int n0, int n_count, int32_t* partials, void* stream) {
  if (!packed || !qa || !partials) return QSPEC_ERR_NULL;
  if (int st = check_shape(M, N, K, group)) return st;
  if (n0 < 0 || n_count <= 0 || n0 % 16 || n_count % 16 || (long long)n0 + n_count > N) return QSPEC_ERR_SHAPE;
  if (misaligned(packed) || misaligned(qa) || misaligned(partials)) return QSPEC_ERR_ALIGN;
  if (int st = check_device()) return st;
  GemmArgs a{};
  a.codes = static_cast<const uint4*>(packed);
  a.scalesT = blob_scales(packed, N, K);
  a.act = qa;
  a.partials = partials;
  a.M = M; a.N = N; a.K = K; a.G = K / kGroup;
  a.n0 = n0; a.n_count = n_count;
  dim3 grid(n_count / 16, (M + 15) / 16);
  hipLaunchKernelGGL((gemm_w4a4_generic<1, 4, true>), grid, dim3(256), 0,
                     static_cast<hipStream_t>(stream), a);
  return launch_status();
}

size_t qspec_accept_workspace_bytes(int B, int gamma, int V) {
  if (check_accept_shape(B, gamma, V) != QSPEC_OK) return 0;
  return (size_t)B * (gamma + 1) * plan_argmax(V).C * sizeof(uint64_t);
}

int qspec_greedy_accept(const void* logits_f16, const int32_t* draft_tokens, int B, int gamma, int V,
                        int32_t* n_accept, int32_t* out_tokens,
                        void* workspace, size_t workspace_bytes, void* stream) {
  if (!logits_f16 || !draft_tokens || !n_accept || !out_tokens || !workspace) return QSPEC_ERR_NULL;
  if (int st = check_accept_shape(B, gamma, V)) return st;
  if (misaligned(logits_f16) || misaligned(workspace) || misaligned4(draft_tokens) || misaligned4(n_accept) ||
      misaligned4(out_tokens))
    return QSPEC_ERR_ALIGN;
  if (workspace_bytes < qspec_accept_workspace_bytes(B, gamma, V)) return QSPEC_ERR_WORKSPACE;
  if (int st = check_device()) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const ArgmaxPlan plan = plan_argmax(V);
  const int R = B * (gamma + 1);
  ArgmaxArgs a{static_cast<const uint16_t*>(logits_f16), static_cast<uint64_t*>(workspace), V, plan.C, plan.chunk};
  if (V % 8 == 0) hipLaunchKernelGGL((argmax_partial_kernel<true>), dim3(plan.C, R), dim3(kArgmaxThreads), 0, s, a);
  else hipLaunchKernelGGL((argmax_partial_kernel<false>), dim3(plan.C, R), dim3(kArgmaxThreads), 0, s, a);
  AcceptArgs f{static_cast<const uint64_t*>(workspace), draft_tokens, n_accept, out_tokens, gamma, plan.C};
  hipLaunchKernelGGL(accept_kernel, dim3(B), dim3(64), 0, s, f);
  return launch_status();
}

int qspec_kv_overwrite(const void* kv_verify_f16, const int32_t* n_accept, const int32_t* pos,
                       int B, int gamma, int D, int S, void* cache_f16, void* stream) {
  if (!kv_verify_f16 || !n_accept || !pos || !cache_f16) return QSPEC_ERR_NULL;
  if (B < 1 || gamma < 1 || S < 1 || D < 8 || D % 8 != 0) return QSPEC_ERR_SHAPE;
  if ((long long)B * (gamma + 1) > 0x7fffffffLL) return QSPEC_ERR_SHAPE;
  if (misaligned(kv_verify_f16) || misaligned(cache_f16) || misaligned4(n_accept) || misaligned4(pos))
    return QSPEC_ERR_ALIGN;
  if (int st = check_device()) return st;
  KvArgs a{static_cast<const uint4*>(kv_verify_f16), static_cast<uint4*>(cache_f16), n_accept, pos, gamma, D / 8, S};
  hipLaunchKernelGGL(kv_overwrite_kernel, dim3(B * (gamma + 1)), dim3(256), 0, static_cast<hipStream_t>(stream), a);
  return launch_status();
}

int qspec_debug_set_plan(const char* name, const char* value) {
  if (!name) return QSPEC_ERR_NULL;
  return apply_override(overrides(), name, value) ? QSPEC_OK : QSPEC_ERR_SHAPE;
}

int qspec_describe_kernel(int mode_w4a4, int M, int N, int K, int group, char* out, size_t cap) {
  if (!out || cap == 0) return QSPEC_ERR_NULL;
  if (int st = check_shape(M, N, K, group)) return st;
  const char* b = mode_w4a4 ? "true" : "false";
  if (use_stream(mode_w4a4 != 0, M, N, K)) {
    const StreamPlan sp = plan_stream(mode_w4a4 != 0, M, N, K);
    snprintf(out, cap, "gemm_stream_kernel<%s, %d, %d>", b, sp.tm, sp.nt);
  } else {
    if (!use_generic()) {
      const TileShape& t = shape_of(mode_w4a4 != 0, plan_tile(mode_w4a4 != 0, M, N, K).shape);
      if (mode_w4a4) snprintf(out, cap, "gemm_tile4w_kernel<%d, %d, %d, %d, %d, false>", t.TN, t.TMW, t.WGN, t.WGM, t.OCC);
      else snprintf(out, cap, "gemm_tile16w_kernel<%d, %d, %d, %d, %d, %d, %d>", t.TN, t.TMW, t.WGN, t.WGM, t.NW, t.NS, t.OCC);
    } else if (mode_w4a4) snprintf(out, cap, "gemm_w4a4_generic<%d, 4, false>", pick_tm(M));
    else snprintf(out, cap, "gemm_w4a16_generic<%d, 4>", pick_tm(M));
  }
  return QSPEC_OK;
}

}  // extern "C"
