// Pieces shared by the weight-streaming GEMM kernels for few tokens (MXFP4: layer_decode.hip; NVFP4 and
// INT4: w4_gemm_skinny.hip): a workgroup of four waves owns 32 output channels at a time, its waves
// split K into four contiguous ranges and their partial 32 x 32 tiles are summed through LDS in a
// fixed order (deterministic).
#pragma once
#include "wush_device.hpp"

namespace wush {
namespace skinny {

constexpr int kWaves = 4;

// Sum the four waves' partial tiles of column block j (fixed order 0,1,2,3), multiply by `scale` if
// SCALED (the product of the tensor scales of a format that has them), and store.  Accumulator e of lane (r, kh), row block rb is token 32*rb + r, output
// channel 32*j + 8*(e/4) + 4*kh + e%4; wave w finishes the quads e/4 == w.
template <int RB, bool OUT_F32, bool SCALED = false>
__device__ __forceinline__ void reduce_store_block(const v16f (&acc)[RB], float (*red)[RB][16][64], int j, int M, int N,
                                                   void* __restrict__ Y, int64_t ldy, int vec_store, int lane, int wave,
                                                   float scale = 1.0f) {
  const int r = lane & 31, kh = lane >> 5;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int e = 0; e < 16; ++e) red[wave][rb][e][lane] = acc[rb][e];
  __syncthreads();
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float v[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int e = 4 * wave + t;
      v[t] = ((red[0][rb][e][lane] + red[1][rb][e][lane]) + red[2][rb][e][lane]) + red[3][rb][e][lane];
      if (SCALED) v[t] *= scale;
    }
    const int row = 32 * rb + r;
    const int col = 32 * j + 8 * wave + 4 * kh;
    if (row < M && col < N) {
      if (OUT_F32) {
        float* y = reinterpret_cast<float*>(Y) + (int64_t)row * ldy + col;
        if (vec_store) {
          *reinterpret_cast<v4f*>(y) = (v4f){v[0], v[1], v[2], v[3]};
        } else {
#pragma unroll
          for (int t = 0; t < 4; ++t)
            if (col + t < N) y[t] = v[t];
        }
      } else {
        uint16_t* y = reinterpret_cast<uint16_t*>(Y) + (int64_t)row * ldy + col;
        if (vec_store) {
          v2u two;
          two[0] = (uint32_t)f32_to_bf16_bits(v[0]) | ((uint32_t)f32_to_bf16_bits(v[1]) << 16);
          two[1] = (uint32_t)f32_to_bf16_bits(v[2]) | ((uint32_t)f32_to_bf16_bits(v[3]) << 16);
          *reinterpret_cast<v2u*>(y) = two;
        } else {
#pragma unroll
          for (int t = 0; t < 4; ++t)
            if (col + t < N) y[t] = f32_to_bf16_bits(v[t]);
        }
      }
    }
  }
  __syncthreads();   // red is rewritten by the next column block
}

// Contiguous K-tile range of a wave: the four waves split KT as evenly as possible.
__device__ __forceinline__ void wave_k_range(int KT, int wave, int& kt0, int& kt1) {
  const int q = (KT + kWaves - 1) / kWaves;
  kt0 = min(wave * q, KT);
  kt1 = min(kt0 + q, KT);
}

// 8-byte (BF16) / 16-byte (FP32) stores of four consecutive channels
inline int decode_vec_store(const void* Y, int64_t N, int64_t ldy, int out_f32) {
  const uintptr_t a = reinterpret_cast<uintptr_t>(Y);
  return (N % 4 == 0) && (ldy % 4 == 0) && (a % (out_f32 ? 16 : 8) == 0);
}

}  // namespace skinny
}  // namespace wush
