// Weight blob construction and its inverse (paper Sec. 3: one 4-bit weight
// tensor shared by the draft and verify modes; Sec. 4.1: group size 128).
// Pure bit moves: canonical int8 codes [N,K] + fp16 scales [N,G] <-> blob.
#pragma once
#include "common.hpp"

namespace qspec {

// One thread builds one 32-bit word (8 codes).  Words are enumerated in blob
// order so the stores are fully coalesced; the 8-byte reads are strided.
__global__ __launch_bounds__(256) void pack_codes_kernel(const int8_t* __restrict__ codes,
                                                         uint32_t* __restrict__ blob_words,
                                                         int N, int K, int G) {
  const size_t total = (size_t)N * K / 8;
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= total) return;
  const int i = (int)(o & 3);              // word within the lane's 16 bytes
  const int lane = (int)((o >> 2) & 63);
  const size_t tile = o >> 8;              // T*G + g
  const int g = (int)(tile % G);
  const int T = (int)(tile / G);
  const int n = T * kTileRows + (lane & 15);
  const int k0 = g * kGroup + i * 32 + (lane >> 4) * 8;   // word i of k-block kb covers 32i + 8kb ..
  const uint2 raw = *reinterpret_cast<const uint2*>(codes + (size_t)n * K + k0);
  uint32_t w = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t byte = ((e < 4 ? raw.x : raw.y) >> (8 * (e & 3))) & 0xFu;
    w |= byte << (4 * nibble_pos(e));
  }
  blob_words[o] = w;
}

// scales [N][G] -> [G][N]
__global__ __launch_bounds__(256) void transpose_scales_kernel(const uint16_t* __restrict__ in,
                                                               uint16_t* __restrict__ out,
                                                               int rows, int cols) {
  const size_t total = (size_t)rows * cols;
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // index into out [cols][rows]
  if (o >= total) return;
  const int r = (int)(o % rows);
  const int c = (int)(o / rows);
  out[o] = in[(size_t)r * cols + c];
}

__global__ __launch_bounds__(256) void unpack_codes_kernel(const uint32_t* __restrict__ blob_words,
                                                           int8_t* __restrict__ codes,
                                                           int N, int K, int G) {
  const size_t total = (size_t)N * K / 8;
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= total) return;
  const int i = (int)(o & 3);
  const int lane = (int)((o >> 2) & 63);
  const size_t tile = o >> 8;
  const int g = (int)(tile % G);
  const int T = (int)(tile / G);
  const int n = T * kTileRows + (lane & 15);
  const int k0 = g * kGroup + i * 32 + (lane >> 4) * 8;   // word i of k-block kb covers 32i + 8kb ..
  const uint32_t w = blob_words[o];
  uint2 raw = {0u, 0u};
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int c = ((int)((w >> (4 * nibble_pos(e))) << 28)) >> 28;     // sign-extend 4 bits
    const uint32_t byte = (uint32_t)c & 0xFFu;
    if (e < 4) raw.x |= byte << (8 * e); else raw.y |= byte << (8 * (e - 4));
  }
  *reinterpret_cast<uint2*>(codes + (size_t)n * K + k0) = raw;
}

}  // namespace qspec
