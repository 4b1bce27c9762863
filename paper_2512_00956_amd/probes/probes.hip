// Measurement aid, not part of the layer path: the block-scaled FP4 MFMA
// (v_mfma_scale_f32_32x32x64_f8f6f4) in a register-only loop, the ceiling the
// MXFP4 GEMM is compared against.  One wave per SIMD, 64 independent MFMAs per
// trip (the GEMM's 8 x 2 accumulator tiles x 4 issues), operands loaded once from
// a caller-provided buffer so that the caller decides the bit patterns: the
// sustained rate depends on them (the shader clock drops with switching
// activity), which is the point of the measurement.  Every workgroup reports its
// shader-clock cycles and 100 MHz real-time ticks.
#include "wush_device.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

__global__ __launch_bounds__(256) void mfma_probe_kernel(const int* __restrict__ in, int iters,
                                                         unsigned long long* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  v16f acc[8][2];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = (v16f){0};
  v4i af[8], bf[2][4];
  int sa[8], sb[2];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    af[i] = *reinterpret_cast<const v4i*>(in + 4 * (64 * i + lane));           // 8 KiB of X-side fragments
    sa[i] = 0x7f7f7f7f;                                                         // scale 1.0
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) bf[j][kk] = *reinterpret_cast<const v4i*>(in + 2048 + 4 * (64 * (4 * j + kk) + lane));
    sb[j] = 0x7f7f7f7f;
  }
  __builtin_amdgcn_sched_barrier(0);
  const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  __builtin_amdgcn_sched_barrier(0);
  for (int it = 0; it < iters; ++it) {
#define WUSH_PROBE_ISSUE(KK)                                                                                          \
  _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                                     \
    const v8i A = {af[i][0], af[i][1], af[i][2], af[i][3], 0, 0, 0, 0};                                               \
    _Pragma("unroll") for (int j = 0; j < 2; ++j) {                                                                   \
      const v8i B = {bf[j][KK][0], bf[j][KK][1], bf[j][KK][2], bf[j][KK][3], 0, 0, 0, 0};                             \
      acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(B, A, acc[i][j], 4, 4, KK, sb[j], KK, sa[i]);       \
    }                                                                                                                 \
  }
    WUSH_PROBE_ISSUE(0)
    WUSH_PROBE_ISSUE(1)
    WUSH_PROBE_ISSUE(2)
    WUSH_PROBE_ISSUE(3)
#undef WUSH_PROBE_ISSUE
  }
  __builtin_amdgcn_sched_barrier(0);
  const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  float r = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) r += acc[i][j][e];
  if (threadIdx.x == 0) {
    out[2 * blockIdx.x] = c1 - c0 + (r == 1.2345f ? 1 : 0);   // keeps the accumulators live
    out[2 * blockIdx.x + 1] = r1 - r0;
  }
}

// The same for the FP16 MFMA (v_mfma_f32_32x32x16_f16), the instruction of the NVFP4 GEMM:
// 4 x 4 accumulator tiles x 4 K steps = 64 independent MFMAs per trip.  `in` = 16 KiB of FP16:
// X-side fragments [4 steps][4 row blocks][64 lanes][8], then the W side likewise.
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(256) void mfma_f16_probe_kernel(const v8h* __restrict__ in, int iters,
                                                             unsigned long long* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  v16f acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = (v16f){0};
  // 8 KiB per side = 8 fragments of 1 KiB: two K steps x 4 row blocks, reused for steps 2 and 3
  v8h a[2][4], b[2][4];
#pragma unroll
  for (int g = 0; g < 2; ++g)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a[g][i] = in[(4 * g + i) * 64 + lane];
      b[g][i] = in[512 + (4 * g + i) * 64 + lane];
    }
  __builtin_amdgcn_sched_barrier(0);
  const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  __builtin_amdgcn_sched_barrier(0);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[g & 1][i], b[g & 1][j], acc[i][j], 0, 0, 0);
  }
  __builtin_amdgcn_sched_barrier(0);
  const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  float r = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) r += acc[i][j][e];
  if (threadIdx.x == 0) {
    out[2 * blockIdx.x] = c1 - c0 + (r == 1.2345f ? 1 : 0);   // keeps the accumulators live
    out[2 * blockIdx.x + 1] = r1 - r0;
  }
}

}  // namespace

hipError_t launch_mfma_f16_probe(const void* operand_bits, int iters, int blocks, void* out, hipStream_t stream) {
  mfma_f16_probe_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(static_cast<const v8h*>(operand_bits), iters,
                                                                        static_cast<unsigned long long*>(out));
  return hipGetLastError();
}

hipError_t launch_mfma_probe(const void* operand_bits, int iters, int blocks, void* out, hipStream_t stream) {
  mfma_probe_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(static_cast<const int*>(operand_bits), iters,
                                                                    static_cast<unsigned long long*>(out));
  return hipGetLastError();
}

}  // namespace wush
