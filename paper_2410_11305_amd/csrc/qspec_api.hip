// C ABI of the QSpec W4 linear layer for gfx950: argument validation, kernel
// selection by problem shape, launches on the caller's stream.  Declarations
// and the buffer layouts are in include/qspec.h.
#include "qspec.h"

#include <hip/hip_runtime.h>
#include <string.h>

#include "common.hpp"
#include "gemm_generic.hpp"
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
  // 32-bit tile / row indices are used inside the kernels
  if ((long long)N * (K / kGroup) > 0x7fffffffLL) return QSPEC_ERR_SHAPE;
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
  return 0;   // every current kernel combines its K-splits inside the workgroup
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

}  // extern "C"
