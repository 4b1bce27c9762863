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
//      32x32 moment on the FP64 MFMA, each wave every fourth group of 4 rows; partial
//      sums go to the workspace (fixed split -> fixed summation order, no atomics).
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

typedef double v4d __attribute__((ext_vector_type(4)));

// Row of the 16 x 16 result block that accumulator element v of a lane holds (v_mfma_f64_16x16x4_f64;
// its column is lane % 16).  Checked by the parity tests of the transforms: the other candidate,
// 4 (lane / 16) + v, gives moments that are not positive definite.
__device__ __forceinline__ int mfma_f64_row(int lane, int v) { return (lane >> 4) + 4 * v; }

__global__ __launch_bounds__(256) void second_moment_kernel(
    const uint16_t* __restrict__ W, int64_t ldw, int N, const uint16_t* __restrict__ X, int64_t ldx, int Mc,
    int rows_per_split_w, int rows_per_split_x, int S, int C, double* __restrict__ partial) {
  // 2 * 1024 FP64 flop per row and block against 64 bytes read: arithmetic bound, so the products run
  // on the FP64 MFMA (16 x 16 x 4: four rows of the block at a time).  With A[i][k] = x[row k][channel i]
  // and B[k][j] = x[row k][channel j] a lane feeds both operands from the element (row lane / 16,
  // channel lane % 16) of a 16-channel half; the moment is symmetric, so the two diagonal 16 x 16
  // blocks and one off-diagonal block are computed (3 MFMAs per 4 rows) and the fourth is its mirror.
  // A wave takes every fourth group of 4 rows; the four waves' sums are added at the end in wave order.
  __shared__ __attribute__((aligned(16))) float tile[kRowsPerStep][48];   // row stride 48: the 4-row reads hit 32 distinct banks per half wave
  __shared__ double red[3][768];
  const int b = blockIdx.x, s = blockIdx.y, z = blockIdx.z;
  const uint16_t* A = z == 0 ? W : X;
  const int64_t ld = z == 0 ? ldw : ldx;
  const int rows = z == 0 ? N : Mc;
  const int per = z == 0 ? rows_per_split_w : rows_per_split_x;
  const int r_begin = min(s * per, rows), r_end = min(r_begin + per, rows);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int k = lane >> 4, c = lane & 15;
  v4d acc00 = {0, 0, 0, 0}, acc01 = {0, 0, 0, 0}, acc11 = {0, 0, 0, 0};
  // 128 rows x 4 chunks of 8 BF16 per step: two chunks per thread (rows past the end contribute zeros);
  // the chunks of the next step are fetched while this one is multiplied
  const int rr0 = threadIdx.x >> 2, ch = threadIdx.x & 3;
  v4u raw[2];
  auto fetch = [&](int r0) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int row = r0 + rr0 + 64 * u;
      raw[u] = (v4u){0, 0, 0, 0};
      if (row < r_end) raw[u] = *reinterpret_cast<const v4u*>(A + (int64_t)row * ld + 32 * b + 8 * ch);
    }
  };
  fetch(r_begin);
  for (int r0 = r_begin; r0 < r_end; r0 += kRowsPerStep) {
    __syncthreads();
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      float4 lo, hi;
      lo.x = __uint_as_float(raw[u][0] << 16); lo.y = __uint_as_float(raw[u][0] & 0xFFFF0000u);
      lo.z = __uint_as_float(raw[u][1] << 16); lo.w = __uint_as_float(raw[u][1] & 0xFFFF0000u);
      hi.x = __uint_as_float(raw[u][2] << 16); hi.y = __uint_as_float(raw[u][2] & 0xFFFF0000u);
      hi.z = __uint_as_float(raw[u][3] << 16); hi.w = __uint_as_float(raw[u][3] & 0xFFFF0000u);
      *reinterpret_cast<float4*>(&tile[rr0 + 64 * u][8 * ch]) = lo;
      *reinterpret_cast<float4*>(&tile[rr0 + 64 * u][8 * ch + 4]) = hi;
    }
    __syncthreads();
    if (r0 + kRowsPerStep < r_end) fetch(r0 + kRowsPerStep);
#pragma unroll
    for (int t = 0; t < kRowsPerStep / 16; ++t) {
      const int rr = 4 * (wave + 4 * t) + k;
      const double x0 = tile[rr][c], x1 = tile[rr][16 + c];
      acc00 = __builtin_amdgcn_mfma_f64_16x16x4f64(x0, x0, acc00, 0, 0, 0);
      acc01 = __builtin_amdgcn_mfma_f64_16x16x4f64(x0, x1, acc01, 0, 0, 0);
      acc11 = __builtin_amdgcn_mfma_f64_16x16x4f64(x1, x1, acc11, 0, 0, 0);
    }
  }
  // waves 1..3 hand their sums to wave 0, which adds them in wave order and writes the 32 x 32 partial
  if (wave > 0) {
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      red[wave - 1][4 * lane + v] = acc00[v];
      red[wave - 1][256 + 4 * lane + v] = acc01[v];
      red[wave - 1][512 + 4 * lane + v] = acc11[v];
    }
  }
  __syncthreads();
  if (wave == 0) {
    double* out = partial + (((int64_t)z * S + s) * C + b) * 1024;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int e = 4 * lane + v, i = mfma_f64_row(lane, v);
      const double m00 = ((acc00[v] + red[0][e]) + red[1][e]) + red[2][e];
      const double m01 = ((acc01[v] + red[0][256 + e]) + red[1][256 + e]) + red[2][256 + e];
      const double m11 = ((acc11[v] + red[0][512 + e]) + red[1][512 + e]) + red[2][512 + e];
      out[i * 32 + c] = m00;
      out[i * 32 + 16 + c] = m01;
      out[(16 + c) * 32 + i] = m01;
      out[(16 + i) * 32 + 16 + c] = m11;
    }
  }
}

__global__ __launch_bounds__(64) void wush_block_kernel(const double* __restrict__ partial, int S, int C, int N,
                                                        int Mc, double lambda, uint16_t* __restrict__ T_out,
                                                        double* __restrict__ T_f64, int* __restrict__ status) {
  const int b = blockIdx.x;
  // reduce the partial moments in a fixed order and normalize
  auto moment = [&](int half, int r, int c) {
    const double* p = partial + ((int64_t)half * S * C + b) * 1024;
    return ordered_sum(p + r * 32 + c, (int64_t)C * 1024, S) * (1.0 / (double)(half ? Mc : N));
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
    return ordered_sum(p + (off + r) * 32 + off + c, (int64_t)C * 1024, S) * (1.0 / (double)(half ? Mc : N));
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
