// Offline construction of the per-block WUSH transforms on the GPU
// (Alg. 2, RTN case, first two steps, and Alg. 1):
//   M_W = d_out^-1 W_(i) W_(i)^T,  M_X = d_batch^-1 X_(i) X_(i)^T     (per block i)
//   W' W'^T = M_W + lambda d^-1 tr(M_W) I,  X' X'^T = likewise         (Cholesky)
//   U S V^T = W'^T X'                                                  (SVD)
//   T_wush = H S^(-1/2) U^T W'^T                                       (the WUSH construction equation)
// Everything is FP64.  Products of two BF16 inputs are exact, so the second
// moments differ from an FP64 reference only in summation order.
//
//   1. second_moment_kernel: grid (block, row split, {W, X}); a workgroup
//      streams its rows of one 32-channel block through LDS and accumulates the
//      32x32 moment, each thread a 2x2 patch; partial sums go to the workspace
//      (fixed split -> fixed summation order, no atomics).
//   2. wush_block_kernel: one wavefront per block: reduce the partials, damp,
//      Cholesky of both moments side by side (lanes 0..31 / 32..63), A = W'^T X',
//      one-sided Jacobi SVD on the columns of A (16 disjoint column pairs per
//      round, 4 lanes per pair; V is never needed), sort, sign convention
//      (largest-magnitude entry of each column of U positive), then
//      T = H diag(s^-1/2) U^T W'^T, rounded to BF16 (nearest even, straight from
//      FP64).
#include "wush_block.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

constexpr int kRowsPerStep = 128;

__global__ __launch_bounds__(256) void second_moment_kernel(
    const uint16_t* __restrict__ W, int64_t ldw, int N, const uint16_t* __restrict__ X, int64_t ldx, int Mc,
    int rows_per_split_w, int rows_per_split_x, int S, int C, double* __restrict__ partial) {
  __shared__ float tile[kRowsPerStep][34];
  const int b = blockIdx.x, s = blockIdx.y, z = blockIdx.z;
  const uint16_t* A = z == 0 ? W : X;
  const int64_t ld = z == 0 ? ldw : ldx;
  const int rows = z == 0 ? N : Mc;
  const int per = z == 0 ? rows_per_split_w : rows_per_split_x;
  const int r_begin = min(s * per, rows), r_end = min(r_begin + per, rows);
  const int ti = threadIdx.x >> 4, tj = threadIdx.x & 15;
  double a00 = 0, a01 = 0, a10 = 0, a11 = 0;
  for (int r0 = r_begin; r0 < r_end; r0 += kRowsPerStep) {
    __syncthreads();
    // 128 rows x 4 chunks of 8 BF16: two chunks per thread
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int idx = threadIdx.x + 256 * u;
      const int rr = idx >> 2, ch = idx & 3;
      const int row = r0 + rr;
      v4u raw = {0, 0, 0, 0};
      if (row < r_end) raw = *reinterpret_cast<const v4u*>(A + (int64_t)row * ld + 32 * b + 8 * ch);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        tile[rr][8 * ch + 2 * i] = __uint_as_float(raw[i] << 16);
        tile[rr][8 * ch + 2 * i + 1] = __uint_as_float(raw[i] & 0xFFFF0000u);
      }
    }
    __syncthreads();
#pragma unroll 8
    for (int rr = 0; rr < kRowsPerStep; ++rr) {
      const float2 a = *reinterpret_cast<const float2*>(&tile[rr][2 * ti]);
      const float2 c = *reinterpret_cast<const float2*>(&tile[rr][2 * tj]);
      const double ax = a.x, ay = a.y, cx = c.x, cy = c.y;
      a00 = fma(ax, cx, a00);
      a01 = fma(ax, cy, a01);
      a10 = fma(ay, cx, a10);
      a11 = fma(ay, cy, a11);
    }
  }
  double* out = partial + (((int64_t)z * S + s) * C + b) * 1024;
  out[(2 * ti) * 32 + 2 * tj] = a00;
  out[(2 * ti) * 32 + 2 * tj + 1] = a01;
  out[(2 * ti + 1) * 32 + 2 * tj] = a10;
  out[(2 * ti + 1) * 32 + 2 * tj + 1] = a11;
}

__global__ __launch_bounds__(64) void wush_block_kernel(const double* __restrict__ partial, int S, int C, int N,
                                                        int Mc, double lambda, uint16_t* __restrict__ T_out,
                                                        double* __restrict__ T_f64, int* __restrict__ status) {
  const int b = blockIdx.x;
  // reduce the partial moments in a fixed order and normalize
  auto moment = [&](int half, int r, int c) {
    const double* p = partial + ((int64_t)half * S * C + b) * 1024;
    double acc = 0.0;
    for (int s = 0; s < S; ++s) acc += p[(int64_t)s * C * 1024 + r * 32 + c];
    return acc * (1.0 / (double)(half ? Mc : N));
  };
  wush_block_wave<32>(moment, lambda, T_out + (int64_t)b * 1024, T_f64 ? T_f64 + (int64_t)b * 1024 : nullptr, nullptr,
                      status);
}

// The same for 16 x 16 blocks (the NVFP4 variant: transform block = quantization group of 16).  The
// moments of block b are the diagonal 16 x 16 sub-block (b & 1) of the 32-channel moments of block b / 2.
__global__ __launch_bounds__(64) void wush_block16_kernel(const double* __restrict__ partial, int S, int C, int N,
                                                          int Mc, double lambda, uint16_t* __restrict__ T_out,
                                                          double* __restrict__ T_f64, int* __restrict__ status) {
  const int b = blockIdx.x, b32 = b >> 1, off = 16 * (b & 1);
  auto moment = [&](int half, int r, int c) {
    const double* p = partial + ((int64_t)half * S * C + b32) * 1024;
    double acc = 0.0;
    for (int s = 0; s < S; ++s) acc += p[(int64_t)s * C * 1024 + (off + r) * 32 + off + c];
    return acc * (1.0 / (double)(half ? Mc : N));
  };
  wush_block_wave<16>(moment, lambda, T_out + (int64_t)b * 256, T_f64 ? T_f64 + (int64_t)b * 256 : nullptr, nullptr,
                      status);
}

__global__ void reset_bt_status_kernel(int* status) {
  if (threadIdx.x < 4) status[threadIdx.x] = 0;
}

int splits_for(int64_t C) {
  int64_t s = 2048 / C;
  if (s < 1) s = 1;
  if (s > 256) s = 256;
  return (int)s;
}

}  // namespace

size_t build_transforms_status_offset(int64_t K) {
  const int64_t C = K / 32;
  return (size_t)(2 * splits_for(C) * C) * 1024 * sizeof(double);
}

size_t build_transforms_workspace_bytes(int64_t K) { return build_transforms_status_offset(K) + 16; }

hipError_t launch_build_transforms(const void* W, int64_t N, int64_t ldw, const void* X, int64_t Mc, int64_t ldx,
                                   int64_t K, double lambda, int block, void* T_out, double* T_f64, void* workspace,
                                   hipStream_t stream) {
  const int C = (int)(K / 32);
  const int S = splits_for(C);
  double* partial = reinterpret_cast<double*>(workspace);
  int* status = reinterpret_cast<int*>(reinterpret_cast<char*>(workspace) + build_transforms_status_offset(K));
  reset_bt_status_kernel<<<dim3(1), dim3(64), 0, stream>>>(status);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  auto per = [&](int64_t rows) { return (int)(((rows + S - 1) / S + kRowsPerStep - 1) / kRowsPerStep * kRowsPerStep); };
  second_moment_kernel<<<dim3(C, S, 2), dim3(256), 0, stream>>>((const uint16_t*)W, ldw, (int)N, (const uint16_t*)X,
                                                               ldx, (int)Mc, per(N), per(Mc), S, C, partial);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (block == 16)
    wush_block16_kernel<<<dim3(2 * C), dim3(64), 0, stream>>>(partial, S, C, (int)N, (int)Mc, lambda, (uint16_t*)T_out,
                                                              T_f64, status);
  else
    wush_block_kernel<<<dim3(C), dim3(64), 0, stream>>>(partial, S, C, (int)N, (int)Mc, lambda, (uint16_t*)T_out, T_f64,
                                                        status);
  return hipGetLastError();
}

}  // namespace wush
