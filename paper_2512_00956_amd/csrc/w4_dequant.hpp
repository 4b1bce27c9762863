// Exact dequantization of the two 4-bit formats without a block-scaled MFMA path to FP16, the
// operand type of v_mfma_f32_32x32x16_f16: NVFP4 (E2M1 element x E4M3 scale per 16: at most 2 + 4
// significant bits, range 2^-10 .. 2688) and INT4 (two's-complement code x BF16 scale per 32: at
// most 3 + 8 significant bits, exact while the scale lies in FP16's normal range).  Shared by the
// tiled GEMM kernels and the weight-streaming kernel for few tokens.
#pragma once
#include "wush_device.hpp"

namespace wush {

typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

// Two E4M3 scale bytes (word `HI` of the row's scale dword) -> two FP16 values, by the
// hardware FP8 convert (gfx950 reads FP8 as OCP E4M3); every finite E4M3 value is an
// FP16 normal, so the conversion is exact.
template <bool HI>
__device__ __forceinline__ v2h e4m3x2_to_f16(uint32_t scales) {
  return __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(scales, 1.0f, HI);
}

// Eight codes (one dword, element i in nibble i) times the group scale -> 8 FP16.
__device__ __forceinline__ v4u dequant8(uint32_t w, v2h s) {
  const float one = 1.0f;
  union { v2h h[4]; v4u u; } c;
  c.h[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, one, 0) * s;
  c.h[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, one, 1) * s;
  c.h[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, one, 2) * s;
  c.h[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, one, 3) * s;
  return c.u;
}

// Eight two's-complement INT4 codes times the group scale -> 8 FP16.  With the sign bits flipped a
// nibble n' = n ^ 8 holds code + 8.  OR-ed into the fraction of an FP16 constant where it stands, it
// becomes 1024 + n' (nibble in bits 0-3 of a half: unit 2^0 in the binade of 1024) or 64 + n' (bits
// 4-7: unit 2^-6 * 64); subtracting 1032 or 72 leaves the signed code, exactly; code * scale has at
// most 3 + 8 significant bits: exact in FP16 too.  One shift by 8 brings the other four nibbles to the
// same two positions, so the eight codes come out in the order 0 4 | 1 5 | 2 6 | 3 7: both operands
// of the GEMM go through this function, and the MFMA's sum over k does not care about the order.
constexpr uint32_t kInt4Mask[2] = {0x000F000Fu, 0x00F000F0u}, kInt4Magic[2] = {0x64006400u, 0x54005400u};
__device__ __forceinline__ v2h int4_pair(uint32_t x, int pos) {   // pos = 0: nibbles at bits 0-3, 1: bits 4-7
  union { uint32_t u; v2h h; } t;
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(t.u) : "v"(x), "s"(kInt4Mask[pos]), "v"(kInt4Magic[pos]));
  return t.h;
}
__device__ __forceinline__ v2h int4_bias(int pos) {
  const _Float16 b = pos ? (_Float16)72.0f : (_Float16)1032.0f;
  return (v2h){b, b};
}
__device__ __forceinline__ v4u dequant8_int4(uint32_t w, v2h s) {
  const uint32_t x = w ^ 0x88888888u, y = x >> 8;
  union { v2h h[4]; v4u u; } c;
#pragma unroll
  for (int i = 0; i < 4; ++i) c.h[i] = (int4_pair(i < 2 ? x : y, i & 1) - int4_bias(i & 1)) * s;
  return c.u;
}

constexpr int kNvfp4 = 0, kInt4 = 1;

// The scales of a lane's 32 W codes of a K step as FP16: bytes 2h, 2h+1 of the row's scale dword,
// h = the lane's half.  NVFP4: two E4M3 bytes, [0] for groups 0 and 1, [1] for groups 2 and 3.
// INT4: one BF16 number, in both.  sel = 0x05040C0C + 0x02020000 h (byte selector that moves the
// two bytes to the top of a dword).
template <int FMT>
__device__ __forceinline__ v2h w_step_scales(uint32_t sdw, int h, uint32_t sel) {
  if constexpr (FMT == kNvfp4) return e4m3x2_to_f16<false>(sdw >> (16 * h));
  else {
    const _Float16 sc = (_Float16)__uint_as_float(__builtin_amdgcn_perm(sdw, sdw, sel));
    return (v2h){sc, sc};
  }
}

}  // namespace wush
