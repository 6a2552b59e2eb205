// C ABI of the QSpec W4 linear layer for gfx950: argument validation, kernel
// selection by problem shape, launches on the caller's stream.  Declarations
// and the buffer layouts are in include/qspec.h.
#include "qspec.h"

#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "common.hpp"
#include "gemm_generic.hpp"
#include "gemm_small.hpp"
#include "gemm_stream.hpp"
#include "pack.hpp"
#include "quant_act.hpp"

using namespace qspec;

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
  static int verdict[64];   // 0 unknown, 1 ok, 2 unsupported
  if (dev < 0 || dev >= 64) return QSPEC_ERR_UNSUPPORTED;
  if (verdict[dev] == 0) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return QSPEC_ERR_HIP;
    verdict[dev] = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 2;
  }
  return verdict[dev] == 1 ? QSPEC_OK : QSPEC_ERR_UNSUPPORTED;
}

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


// ---------------------------------------------------------------- small-M plans
// A plan fixes the workgroup shape (WN x WK wavefronts), the number of
// K-chunks S and the LDS footprint.  It is a pure function of (mode, M, N, K),
// so qspec_workspace_bytes and the GEMM entry points always agree.
struct SmallPlan {
  bool use;        // false: fall back to the generic kernel
  int TM, WN, WK, S, gc_max;
  size_t lds_bytes;
};

constexpr int kLdsCap = 64 * 1024;
constexpr int kSmallMaxM = 32;

// QSPEC_PLAN_W4A4 / QSPEC_PLAN_W4A16 = "WN,WK,S" override the heuristic
// (benchmark A/B only; a plan that does not fit is ignored).
bool plan_override(bool w4a4, int* wn, int* wk, int* s) {
  const char* e = getenv(w4a4 ? "QSPEC_PLAN_W4A4" : "QSPEC_PLAN_W4A16");
  if (!e) return false;
  return sscanf(e, "%d,%d,%d", wn, wk, s) == 3;
}

// One staging pass must cover a chunk: kStageU 16-byte pieces per thread and
// row, one 8-byte scale piece per thread, two activation scales per thread.
template <bool W4A4>
bool small_stage_fits(int TM, int WN, int gc_max) {
  const int tpr = 512 / (TM * 16);
  if (gc_max * (W4A4 ? 4 : 16) > tpr * kStageU) return false;
  if (gc_max * WN * 4 > 512) return false;
  if (W4A4 && gc_max * TM * 16 > 1024) return false;
  return true;
}

template <bool W4A4>
size_t small_lds_bytes(int TM, int WN, int WK, int gc_max) {
  if (!small_stage_fits<W4A4>(TM, WN, gc_max)) return (size_t)1 << 30;
  size_t total = TM == 1 ? (size_t)SmallLds<W4A4, 1>(gc_max, WN).total : (size_t)SmallLds<W4A4, 2>(gc_max, WN).total;
  const size_t red = WK > 1 ? (size_t)WK * WN * TM * 4 * 64 * 4 : 0;
  return total > red ? total : red;
}

template <bool W4A4>
SmallPlan plan_small(int M, int N, int K) {
  SmallPlan p{};
  const int G = K / kGroup;
  if (M > kSmallMaxM) return p;
  p.TM = M <= 16 ? 1 : 2;
  int wn = W4A4 ? 1 : 8, wk = W4A4 ? 8 : 1, s = 0;
  const bool forced = plan_override(W4A4, &wn, &wk, &s);
  const bool shape_ok = (wn == 1 || wn == 2 || wn == 4 || wn == 8) && wn * wk == 8;
  if (!shape_ok) { wn = W4A4 ? 1 : 8; wk = 8 / wn; s = 0; }
  p.WN = wn; p.WK = wk;
  const int NB = (N / 16 + wn - 1) / wn;
  // smallest S whose chunk fits the LDS cap
  int s_min = 1;
  while (s_min < G && small_lds_bytes<W4A4>(p.TM, wn, wk, (G + s_min - 1) / s_min) > (size_t)kLdsCap) ++s_min;
  if (small_lds_bytes<W4A4>(p.TM, wn, wk, (G + s_min - 1) / s_min) > (size_t)kLdsCap) return p;
  if (!(forced && s >= s_min && s <= G)) {
    const int target = 512;                 // about two workgroups per CU
    s = (target + NB / 2) / NB;
    if (s < s_min) s = s_min;
    if (s > G) s = G;
    if (W4A4 && s_min == 1 && NB >= 256) s = 1;
  }
  p.S = s;
  p.gc_max = (G + s - 1) / s;
  p.lds_bytes = small_lds_bytes<W4A4>(p.TM, wn, wk, p.gc_max);
  p.use = true;
  return p;
}

template <bool W4A4, int TM, int WN, int WK>
void launch_small_inst(const SmallArgs& a, size_t lds, hipStream_t s) {
  dim3 grid((a.N / 16 + WN - 1) / WN, a.S);
  hipLaunchKernelGGL((gemm_small_kernel<W4A4, TM, WN, WK, 8>), grid, dim3(WN * WK * 64), lds, s, a);
}

template <bool W4A4, int TM>
void launch_small_tm(const SmallPlan& p, const SmallArgs& a, hipStream_t s) {
  switch (p.WN) {
    case 1: launch_small_inst<W4A4, TM, 1, 8>(a, p.lds_bytes, s); break;
    case 2: launch_small_inst<W4A4, TM, 2, 4>(a, p.lds_bytes, s); break;
    case 4: launch_small_inst<W4A4, TM, 4, 2>(a, p.lds_bytes, s); break;
    default: launch_small_inst<W4A4, TM, 8, 1>(a, p.lds_bytes, s); break;
  }
}

template <bool W4A4>
void launch_small(const SmallPlan& p, SmallArgs a, hipStream_t s) {
  a.S = p.S;
  a.gc_max = p.gc_max;
  if (p.TM == 1) launch_small_tm<W4A4, 1>(p, a, s); else launch_small_tm<W4A4, 2>(p, a, s);
  if (p.S > 1) {
    const size_t n_quads = (size_t)a.M * a.N / 4;
    hipLaunchKernelGGL(splitk_finish_kernel, dim3(blocks_for(n_quads, 256)), dim3(256), 0, s,
                       reinterpret_cast<const float4*>(a.ws), reinterpret_cast<uint2*>(a.y), n_quads, p.S);
  }
}


// ---------------------------------------------------------------- streaming (small-M) kernel
constexpr int kStreamMaxM = 32;
constexpr int kNumCU = 256;

// n-tiles per workgroup: minimise rounds x work per round over the 256 CUs, prefer
// the larger NT on a tie (the activation operand is re-used NT times).
// QSPEC_STREAM_NT=1..4 overrides (benchmark A/B only).
int stream_nt(int N) {
  const int tiles = N / 16;
  if (const char* e = getenv("QSPEC_STREAM_NT")) {
    const int v = atoi(e);
    if (v >= 1 && v <= 4) return v;
  }
  int best = 1, best_cost = 1 << 30;
  for (int nt = 1; nt <= 4; ++nt) {
    const int blocks = (tiles + nt - 1) / nt;
    const int cost = ((blocks + kNumCU - 1) / kNumCU) * nt;
    if (cost <= best_cost) { best_cost = cost; best = nt; }
  }
  return best;
}

bool use_stream(int M) {
  if (M > kStreamMaxM) return false;
  const char* e = getenv("QSPEC_KERNEL");
  return !(e && strcmp(e, "small") == 0);
}

template <bool W4A4, int TM>
void launch_stream_tm(const StreamArgs& a, int nt, hipStream_t s) {
  const int tiles = a.N / 16;
  dim3 grid((tiles + nt - 1) / nt), block(kStreamWaves * 64);
  switch (nt) {
    case 1: hipLaunchKernelGGL((gemm_stream_kernel<W4A4, TM, 1>), grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL((gemm_stream_kernel<W4A4, TM, 2>), grid, block, 0, s, a); break;
    case 3: hipLaunchKernelGGL((gemm_stream_kernel<W4A4, TM, 3>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((gemm_stream_kernel<W4A4, TM, 4>), grid, block, 0, s, a); break;
  }
}

template <bool W4A4>
void launch_stream(const StreamArgs& a, hipStream_t s) {
  const int nt = stream_nt(a.N);
  if (a.M <= 16) launch_stream_tm<W4A4, 1>(a, nt, s); else launch_stream_tm<W4A4, 2>(a, nt, s);
}

inline size_t plan_ws_bytes(const SmallPlan& p, int M, int N) {
  return p.use && p.S > 1 ? (size_t)p.S * M * N * 4 : 0;
}

}  // namespace

extern "C" {

const char* qspec_status_string(int status) {
  switch (status) {
    case QSPEC_OK: return "ok";
    case QSPEC_ERR_NULL: return "null pointer";
    case QSPEC_ERR_SHAPE: return "unsupported shape (need group == 128, K % 128 == 0, N % 16 == 0, M >= 1)";
    case QSPEC_ERR_ALIGN: return "pointer not 16-byte aligned";
    case QSPEC_ERR_WORKSPACE: return "workspace too small";
    case QSPEC_ERR_HIP: return "HIP runtime error";
    case QSPEC_ERR_UNSUPPORTED: return "device is not gfx950";
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
  if (use_stream(M)) return 0;
  const size_t a = plan_ws_bytes(plan_small<true>(M, N, K), M, N);
  const size_t b = plan_ws_bytes(plan_small<false>(M, N, K), M, N);
  return a > b ? a : b;
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
  if (use_stream(M)) {
    StreamArgs st{};
    st.codes = a.codes; st.scalesT = a.scalesT; st.act = qa; st.sa = sa; st.y = a.y;
    st.M = M; st.N = N; st.K = K; st.G = a.G;
    launch_stream<true>(st, s);
    return launch_status();
  }
  const SmallPlan plan = plan_small<true>(M, N, K);
  if (plan.use) {
    SmallArgs sa_{};
    sa_.codes = a.codes; sa_.scalesT = a.scalesT; sa_.act = qa; sa_.sa = sa; sa_.y = a.y;
    sa_.ws = static_cast<float*>(workspace);
    sa_.M = M; sa_.N = N; sa_.K = K; sa_.G = a.G;
    launch_small<true>(plan, sa_, s);
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
  if (use_stream(M)) {
    StreamArgs st{};
    st.codes = a.codes; st.scalesT = a.scalesT; st.act = x_f16; st.y = a.y;
    st.M = M; st.N = N; st.K = K; st.G = a.G;
    launch_stream<false>(st, s);
    return launch_status();
  }
  const SmallPlan plan = plan_small<false>(M, N, K);
  if (plan.use) {
    SmallArgs sa_{};
    sa_.codes = a.codes; sa_.scalesT = a.scalesT; sa_.act = x_f16; sa_.y = a.y;
    sa_.ws = static_cast<float*>(workspace);
    sa_.M = M; sa_.N = N; sa_.K = K; sa_.G = a.G;
    launch_small<false>(plan, sa_, s);
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

int qspec_describe_kernel(int mode_w4a4, int M, int N, int K, int group, char* out, size_t cap) {
  if (!out || cap == 0) return QSPEC_ERR_NULL;
  if (int st = check_shape(M, N, K, group)) return st;
  const char* b = mode_w4a4 ? "true" : "false";
  if (use_stream(M)) {
    snprintf(out, cap, "gemm_stream_kernel<%s, %d, %d>", b, M <= 16 ? 1 : 2, stream_nt(N));
  } else {
    const SmallPlan p = mode_w4a4 ? plan_small<true>(M, N, K) : plan_small<false>(M, N, K);
    if (p.use) snprintf(out, cap, "gemm_small_kernel<%s, %d, %d, %d, 8>", b, p.TM, p.WN, p.WK);
    else if (mode_w4a4) snprintf(out, cap, "gemm_w4a4_generic<%d, 4, false>", pick_tm(M));
    else snprintf(out, cap, "gemm_w4a16_generic<%d, 4>", pick_tm(M));
  }
  return QSPEC_OK;
}

}  // extern "C"
