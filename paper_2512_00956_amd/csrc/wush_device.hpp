// Device-side helpers shared by the gfx950 kernels: vector types, the E8M0
// scale rule on FP32 bit patterns, and E2M1 packing through the hardware
// convert.  (Quantizer: RTN with AbsMax scales per group of 32 -- paper,
// Methodology, "Block-independent constraint".)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wush {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

constexpr int kBlock = 32;  // transform block = quantization group

// E8M0 byte for a group whose largest magnitude is `amax` (>= 0, finite).
//   rule 0 (no saturation): smallest e with amax <= 6 * 2^e.  6 * 2^e is
//   1.5 * 2^(e+2), so e = exponent(amax) - 2, plus one when the significand
//   exceeds 1.5; adding 0x3FFFFF to the bit pattern carries into the exponent
//   field exactly in that case.
//   rule 1 (OCP floor): e = exponent(amax) - 2.
// Zero and FP32 denormals fall through to byte 0.
__device__ __forceinline__ int scale_byte_f32(float amax, int rule) {
  const uint32_t bits = __float_as_uint(amax);
  const int biased = rule == 0 ? (int)((bits + 0x3FFFFFu) >> 23) : (int)(bits >> 23);
  return min(max(biased - 2, 0), 254);
}

// The power of two 2^(byte-127) as an FP32 bit pattern.  Byte 0 (2^-127) is
// an FP32 denormal; the fp4 convert only looks at the exponent field of its
// scale operand, where an all-zero field already means 2^-127.
__device__ __forceinline__ float scale_as_f32(int byte) {
  return __uint_as_float((uint32_t)byte << 23);
}

// Round two FP32 values divided by the power-of-two `scale` to E2M1 (nearest,
// ties to even, saturating, sign of zero kept) and place the byte
// (first value = low nibble) at byte position SEL of `word`.
template <int SEL>
__device__ __forceinline__ uint32_t pack2_e2m1(uint32_t word, float a, float b, float scale) {
  return __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(word, a, b, scale, SEL);
}

// Eight FP32 values -> one 32-bit word of E2M1 codes, element i in nibble i.
__device__ __forceinline__ uint32_t pack8_e2m1(const float* v, float scale) {
  uint32_t w = 0;
  w = pack2_e2m1<0>(w, v[0], v[1], scale);
  w = pack2_e2m1<1>(w, v[2], v[3], scale);
  w = pack2_e2m1<2>(w, v[4], v[5], scale);
  w = pack2_e2m1<3>(w, v[6], v[7], scale);
  return w;
}

// Scale byte from an FP64 AbsMax; same rule as scale_byte_f32 on the 11-bit
// exponent (re-biased to E8M0) and the 52-bit fraction.
__device__ __forceinline__ int scale_byte_f64(double amax, int rule) {
  const uint64_t bits = (uint64_t)__double_as_longlong(amax);
  if (amax == 0.0) return 0;
  const int e11 = (int)(bits >> 52);
  const uint64_t frac = bits & 0xFFFFFFFFFFFFFull;
  int biased = e11 - 1023 + 127 - 2;
  if (rule == 0 && frac > 0x8000000000000ull) biased += 1;
  return min(max(biased, 0), 254);
}

// |v| (already divided by the group scale) -> E2M1 magnitude code, nearest,
// ties to the even code, saturating.
__device__ __forceinline__ uint32_t e2m1_code_f64(double a) {
  uint32_t c = 0;
  c += a > 0.25;
  c += a >= 0.75;
  c += a > 1.25;
  c += a >= 1.75;
  c += a > 2.5;
  c += a >= 3.5;
  c += a > 5.0;
  return c;
}

// ---------------------------------------------------------------------------
// Tiled ("MFMA fragment order") layout of packed codes and scales, used between
// the quantizers and the tiled GEMM.  Needs K % 256 == 0; buffers are padded to a
// multiple of 256 rows.  With rb = row/32, r = row%32, and the 32-element group g of a
// row split as kt = g/8 (K tile of 256), kh = (g%8)/4, kk = g%4:
//   codes : the 16-byte chunk of (row, g) sits at
//           ((((rb*KT + kt)*4 + kk)*64) + kh*32 + r) * 16
//           i.e. [row block][K tile][issue kk][lane = kh*32 + r][16 B]: one
//           (row block, K tile, kk) fragment is 1 KiB, contiguous, in the lane
//           order of the scaled 32x32x64 MFMA operand;
//   scales: the dword holding groups 4kh..4kh+3 of tile kt of the row sits at
//           ((rb*KT + kt)*64 + kh*32 + r) * 4, byte kk = group 4kh + kk.
// ---------------------------------------------------------------------------
__host__ __device__ __forceinline__ int64_t tiled_chunk_offset(int row, int g, int KT) {
  const int rb = row >> 5, r = row & 31, kt = g >> 3, kh = (g >> 2) & 1, kk = g & 3;
  return ((((int64_t)rb * KT + kt) * 4 + kk) * 64 + kh * 32 + r) * 16;
}

__host__ __device__ __forceinline__ int64_t tiled_scale_offset(int row, int g, int KT) {
  const int rb = row >> 5, r = row & 31, kt = g >> 3, kh = (g >> 2) & 1, kk = g & 3;
  return (((int64_t)rb * KT + kt) * 64 + kh * 32 + r) * 4 + kk;
}

// Workgroup id -> tile id such that every XCD (the hardware deals workgroup ids round-robin over the
// eight XCDs, each with an L2 of its own) works on one contiguous range of tile ids: XCD x takes
// total / 8 ids, one more if x < total % 8.
__device__ __forceinline__ int xcd_contiguous_id(int id, int total) {
  const int xcd = id & 7, pos = id >> 3, base = total >> 3, rem = total & 7;
  return xcd * base + min(xcd, rem) + pos;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
  return __uint_as_float((uint32_t)b << 16);
}

// FP32 -> BF16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// FP64 -> BF16 bits, round to nearest even, for finite values in BF16's normal range.
__device__ __forceinline__ uint16_t f64_to_bf16_bits(double v) {
  const uint64_t u = (uint64_t)__double_as_longlong(v);
  const uint32_t sign = (uint32_t)(u >> 63) << 15;
  const int e11 = (int)((u >> 52) & 0x7FF);
  if (e11 == 0) return (uint16_t)sign;               // zero (FP64 denormals flush)
  const int e8 = e11 - 1023 + 127;
  if (e8 <= 0) return (uint16_t)sign;                 // below BF16's normal range
  if (e8 >= 255) return (uint16_t)(sign | 0x7F80);    // overflow -> inf
  const uint64_t frac = u & 0xFFFFFFFFFFFFFull;       // 52 bits
  uint32_t mag = ((uint32_t)e8 << 7) | (uint32_t)(frac >> 45);
  const uint64_t rest = frac & ((1ull << 45) - 1), half = 1ull << 44;
  if (rest > half || (rest == half && (mag & 1))) mag += 1;  // carry may bump the exponent: still correct
  return (uint16_t)(sign | mag);
}

}  // namespace wush
