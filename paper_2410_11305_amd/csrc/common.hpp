// Shared device-side definitions for the gfx950 kernels of the QSpec W4 linear
// layer: vector types, the packed-word format and the two unpackers (nibbles
// -> int8 for the draft mode, nibbles -> fp16 for the verify mode).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qspec {

constexpr int kGroup = 128;        // quantisation group along K (paper Sec. 4.1)
constexpr int kTileRows = 16;      // output rows per weight tile
constexpr int kTileBytes = 1024;   // 16 rows x 128 codes x 4 bit
constexpr int kWave = 64;

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));

// Bit position (in nibbles) of code e of an 8-code run inside its 32-bit word.
// Chosen so that masking with 0x000F000F / 0x00F000F0 (before and after a
// shift by 8) yields the fp16 pairs (c0,c1) (c2,c3) (c4,c5) (c6,c7) in order,
// while 0xF0F0F0F0 masks yield four int8 values per register.
__device__ __host__ inline constexpr int nibble_pos(int e) { return (e & 1) * 4 + (e >> 1); }

// ---- int8 operands -------------------------------------------------------
// Each nibble is moved to the HIGH half of a byte, so the byte read as int8
// equals 16 * code (two's complement does the sign extension for free).  A
// product of two such operands is 256 * the true integer partial sum.
struct I8Pair { v4i lo, hi; };

__device__ inline I8Pair unpack_i8(uint4 w) {
  I8Pair r;
  r.hi = v4i{(int)(w.x & 0xF0F0F0F0u), (int)(w.y & 0xF0F0F0F0u),
             (int)(w.z & 0xF0F0F0F0u), (int)(w.w & 0xF0F0F0F0u)};
  r.lo = v4i{(int)((w.x << 4) & 0xF0F0F0F0u), (int)((w.y << 4) & 0xF0F0F0F0u),
             (int)((w.z << 4) & 0xF0F0F0F0u), (int)((w.w << 4) & 0xF0F0F0F0u)};
  return r;
}

// ---- fp16 operands -------------------------------------------------------
// One word (8 codes) -> 8 fp16 values equal to the integer codes, exactly.
// 0x6400 is fp16 1024.0 whose mantissa LSB is 1: OR-ing an offset-binary
// nibble u = code + 8 into mantissa bits 0..3 gives 1024 + u, into bits 4..7
// gives 1024 + 16u; (1024 + u) - 1032 and (1024 + 16u)/16 - 72 are both the
// code, with no rounding.
__device__ inline v8h dequant_word(uint32_t w) {
  // (w & mask) ^ c is one three-input bit operation: the xor constant flips
  // the nibble's sign bit (two's complement -> offset binary) and plants the
  // 0x6400 exponent in the bits the mask cleared.
  const uint32_t w8 = w >> 8;
  const uint32_t b0 = (w & 0x000F000Fu) ^ 0x64086408u;
  const uint32_t b1 = (w & 0x00F000F0u) ^ 0x64806480u;
  const uint32_t b2 = (w8 & 0x000F000Fu) ^ 0x64086408u;
  const uint32_t b3 = (w8 & 0x00F000F0u) ^ 0x64806480u;
  const v2h k1032 = {(_Float16)1032.0f, (_Float16)1032.0f};
  const v2h k72 = {(_Float16)72.0f, (_Float16)72.0f};
  const v2h k16th = {(_Float16)0.0625f, (_Float16)0.0625f};
  const v2h h0 = __builtin_bit_cast(v2h, b0) - k1032;
  const v2h h1 = __builtin_bit_cast(v2h, b1) * k16th - k72;
  const v2h h2 = __builtin_bit_cast(v2h, b2) - k1032;
  const v2h h3 = __builtin_bit_cast(v2h, b3) * k16th - k72;
  return v8h{h0.x, h0.y, h1.x, h1.y, h2.x, h2.y, h3.x, h3.y};
}

__device__ inline float half_bits_to_float(uint16_t b) {
  return (float)__builtin_bit_cast(_Float16, b);
}

__device__ inline uint16_t float_to_half_bits(float f) {
  return __builtin_bit_cast(uint16_t, (_Float16)f);   // round-to-nearest-even
}

}  // namespace qspec
