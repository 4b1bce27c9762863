// MXFP4 x MXFP4 GEMM, FP32 accumulation, on CDNA4 block-scaled MFMA
// (v_mfma_scale_f32_32x32x64_f8f6f4 with both operands E2M1 and one E8M0 scale
// per 32 elements): Y = deq(Xq,Xs) . deq(Wq,Ws)^T, the sum over blocks of the
// layer forward-pass equation ("FP4-MatMul" in section "GPU Kernel Support").
//
// Operand mapping of the instruction (verified on hardware): for a 32x64
// operand tile, lane l holds row l%32 and the 32 consecutive K elements of
// half l/32 -- 16 bytes of the canonical packed layout -- plus the one scale
// byte of exactly that group.  Accumulator r of lane l is output row
// 8*(r/4) + 4*(l/32) + r%4, column l%32.
#include "wush_device.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

__device__ __forceinline__ void store_out(void* Y, int64_t ldy, int row, int col, float v, int out_f32) {
  if (out_f32) reinterpret_cast<float*>(Y)[(int64_t)row * ldy + col] = v;
  else reinterpret_cast<uint16_t*>(Y)[(int64_t)row * ldy + col] = f32_to_bf16_bits(v);
}

// Reference-grade kernel: one wavefront per 32x32 output tile, operands straight
// from global memory.  Handles every shape (ragged M, N, odd K/32).
__global__ __launch_bounds__(256) void gemm_simple_kernel(
    const uint8_t* __restrict__ Xq, const uint8_t* __restrict__ Xs,
    const uint8_t* __restrict__ Wq, const uint8_t* __restrict__ Ws,
    int M, int N, int K, int out_f32, void* __restrict__ Y, int64_t ldy) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int tiles_n = (N + 31) / 32;
  const int64_t tile = (int64_t)blockIdx.x * 4 + wave;
  const int tm = (int)(tile / tiles_n), tn = (int)(tile % tiles_n);
  if (tm * 32 >= M) return;  // wave-uniform
  const int r = lane & 31, kh = lane >> 5;
  const int C = K / 32;
  const int arow = min(tm * 32 + r, M - 1);
  const int brow = min(tn * 32 + r, N - 1);
  const uint8_t* ap = Xq + (int64_t)arow * (K / 2);
  const uint8_t* bp = Wq + (int64_t)brow * (K / 2);
  const uint8_t* as = Xs + (int64_t)arow * C;
  const uint8_t* bs = Ws + (int64_t)brow * C;
  v16f acc = {0};
  for (int g = 0; g < C; g += 2) {
    const int gg = g + kh;
    v4i a = {0, 0, 0, 0}, b = {0, 0, 0, 0};
    int sa = 127, sb = 127;
    if (gg < C) {
      a = *reinterpret_cast<const v4i*>(ap + 16 * gg);
      b = *reinterpret_cast<const v4i*>(bp + 16 * gg);
      sa = as[gg];
      sb = bs[gg];
    }
    const v8i A = {a[0], a[1], a[2], a[3], 0, 0, 0, 0};
    const v8i B = {b[0], b[1], b[2], b[3], 0, 0, 0, 0};
    acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, acc, 4, 4, 0, sa, 0, sb);
  }
  const int col = tn * 32 + r;
  if (col < N) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = tm * 32 + 8 * (i >> 2) + 4 * kh + (i & 3);
      if (row < M) store_out(Y, ldy, row, col, acc[i], out_f32);
    }
  }
}

}  // namespace

hipError_t launch_mxfp4_gemm(const void* Xq, const void* Xs, const void* Wq, const void* Ws,
                             int64_t M, int64_t N, int64_t K, int out_f32, void* Y, int64_t ldy,
                             hipStream_t stream) {
  const int64_t tiles = ((M + 31) / 32) * ((N + 31) / 32);
  gemm_simple_kernel<<<dim3((unsigned)((tiles + 3) / 4)), dim3(256), 0, stream>>>(
      (const uint8_t*)Xq, (const uint8_t*)Xs, (const uint8_t*)Wq, (const uint8_t*)Ws,
      (int)M, (int)N, (int)K, out_f32, Y, ldy);
  return hipGetLastError();
}

}  // namespace wush
