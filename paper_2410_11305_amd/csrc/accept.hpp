// The two steps that follow the verify pass (paper Sec. 3.1): the greedy
// acceptance policy and the KV-cache overwrite.
//
// Acceptance: the verify pass returns gamma + 1 rows of fp16 logits per sequence;
// a drafted token is accepted exactly when it equals the top-1 token of the
// verify distribution at its position, the first rejection discards the later
// drafts, and the token at that position (or, when every draft is accepted, one
// extra token) is the verify pass's own top-1.  Ties go to the lowest token id.
//
// Two launches, no atomics, no state: argmax_partial_kernel scans one chunk of
// one row per workgroup (HBM-bound: every logit is read once, 16 bytes per
// lane) and leaves a 64-bit key per chunk in the workspace; accept_kernel (one
// wavefront per sequence) reduces the keys of each row and walks the drafts in
// order.  A key is (order-preserving image of the fp16 value) << 32 | ~index,
// so that the unsigned maximum is the largest value and, among equals, the
// lowest index.
#pragma once
#include "buffer.hpp"
#include "common.hpp"

namespace qspec {

constexpr int kArgmaxThreads = 256;
constexpr int kArgmaxMaxChunks = 64;        // one lane of the second kernel per chunk

// fp16 bits -> 16-bit unsigned whose order is the order of the values
// (-0 and +0 compare equal, as they do as numbers; NaN is not handled).
__device__ inline uint32_t half_order_key(uint32_t bits) {
  bits &= 0xFFFFu;
  if (bits == 0x8000u) bits = 0u;
  return (bits & 0x8000u) ? (bits ^ 0xFFFFu) : (bits | 0x8000u);
}

__device__ inline uint64_t wave_max_u64(uint64_t k) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)k, off, 64);
    const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(k >> 32), off, 64);
    const uint64_t o = ((uint64_t)hi << 32) | lo;
    k = o > k ? o : k;
  }
  return k;
}

struct ArgmaxArgs {
  const uint16_t* logits;   // fp16 [R][V]
  uint64_t* keys;           // [R][C]
  int V, C, chunk;          // chunk: elements per chunk (a multiple of 8 when VEC)
};

// grid (C, R).  VEC: V % 8 == 0, rows are 16-byte aligned, 8 logits per load.
template <bool VEC>
__global__ __launch_bounds__(kArgmaxThreads) void argmax_partial_kernel(ArgmaxArgs p) {
  const int c = blockIdx.x, r = blockIdx.y;
  const int begin = c * p.chunk;
  const int end = min(p.V, begin + p.chunk);
  const uint16_t* row = p.logits + (size_t)r * p.V;
  uint32_t best = 0u, best_i = 0xFFFFFFFFu;          // key 0 is below every real key (the lowest is 0x0000 only for NaN patterns)
  bool have = false;
  if (VEC) {
    for (int i = begin + (int)threadIdx.x * 8; i < end; i += kArgmaxThreads * 8) {
      const uint4 q = *reinterpret_cast<const uint4*>(row + i);
      const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t k = half_order_key(w[e >> 1] >> ((e & 1) * 16));
        // indices rise inside a thread: a strict comparison keeps the lowest index of equal values
        if (!have || k > best) { best = k; best_i = (uint32_t)(i + e); have = true; }
      }
    }
  } else {
    for (int i = begin + (int)threadIdx.x; i < end; i += kArgmaxThreads) {
      const uint32_t k = half_order_key(row[i]);
      if (!have || k > best) { best = k; best_i = (uint32_t)i; have = true; }
    }
  }
  uint64_t key = have ? (((uint64_t)best << 32) | (uint64_t)(~best_i)) : 0ull;
  key = wave_max_u64(key);
  __shared__ uint64_t part[kArgmaxThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = key;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint64_t k = part[0];
#pragma unroll
    for (int w = 1; w < kArgmaxThreads / 64; ++w) k = part[w] > k ? part[w] : k;
    p.keys[(size_t)r * p.C + c] = k;
  }
}

struct AcceptArgs {
  const uint64_t* keys;     // [B*(gamma+1)][C]
  const int32_t* draft;     // [B][gamma]
  int32_t* n_accept;        // [B]
  int32_t* out_tokens;      // [B][gamma+1]
  int gamma, C;
};

// One wavefront per sequence (grid B, 64 threads).
__global__ __launch_bounds__(64) void accept_kernel(AcceptArgs p) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int rows = p.gamma + 1;
  int n = 0;
  bool open = true;                       // no draft rejected so far
  for (int j = 0; j < rows; ++j) {
    uint64_t k = lane < p.C ? p.keys[((size_t)b * rows + j) * p.C + lane] : 0ull;
    k = wave_max_u64(k);
    const int32_t top = (int32_t)(~(uint32_t)k);
    int32_t emit = -1;
    if (open) {
      if (j < p.gamma && p.draft[(size_t)b * p.gamma + j] == top) {
        emit = top;                       // accepted draft
        n = j + 1;
      } else {
        emit = top;                       // the verify pass's own token: correction, or the extra one
        open = false;
      }
    }
    if (lane == 0) p.out_tokens[(size_t)b * rows + j] = emit;
  }
  if (lane == 0) p.n_accept[b] = n;
}

struct KvArgs {
  const uint4* src;         // fp16 [B][gamma+1][D]
  uint4* cache;             // fp16 [B][S][D]
  const int32_t* n_accept;  // [B]
  const int32_t* pos;       // [B]
  int gamma, D8, S;         // D8 = D / 8 (16-byte pieces per row)
};

// grid B*(gamma+1): row j of sequence b goes to cache row pos[b] + j when j <= n_accept[b]
// (and the target lies inside the cache).
__global__ __launch_bounds__(256) void kv_overwrite_kernel(KvArgs p) {
  const int rows = p.gamma + 1;
  const int b = blockIdx.x / rows, j = blockIdx.x - b * rows;
  const int a = min(max(p.n_accept[b], 0), p.gamma);
  const long long s = (long long)p.pos[b] + j;
  if (j > a || s < 0 || s >= p.S) return;
  const uint4* src = p.src + ((size_t)b * rows + j) * p.D8;
  uint4* dst = p.cache + ((size_t)b * p.S + (size_t)s) * p.D8;
  for (int i = threadIdx.x; i < p.D8; i += 256) dst[i] = src[i];
}

}  // namespace qspec
