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
#include "wush_device.hpp"
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

__global__ __launch_bounds__(64) void wush_block_kernel(const double* __restrict__ partial, int S, int C, int N,
                                                        int Mc, double lambda, uint16_t* __restrict__ T_out,
                                                        double* __restrict__ T_f64, int* __restrict__ status) {
  __shared__ double LW[32][33];   // M_W, then W' (lower triangle)
  __shared__ double LX[32][33];   // M_X, then X'
  __shared__ double A[32][33];    // W'^T X', then U S (columns), then B
  __shared__ double U[32][33];
  __shared__ double sv[32];
  __shared__ int order[32];
  __shared__ int conv;
  const int b = blockIdx.x, lane = threadIdx.x;
  const int half = lane >> 5, r = lane & 31;
  double (*L)[33] = half ? LX : LW;

  // ---- reduce partial moments (fixed order), normalize, damp
  {
    const double inv_n = 1.0 / (double)(half ? Mc : N);
    const double* p = partial + ((int64_t)half * S * C + b) * 1024;
    double tr = 0.0;
    for (int c = 0; c < 32; ++c) {
      double acc = 0.0;
      for (int s = 0; s < S; ++s) acc += p[(int64_t)s * C * 1024 + r * 32 + c];
      acc *= inv_n;
      L[r][c] = acc;
    }
    __syncthreads();
    for (int c = 0; c < 32; ++c) tr += L[c][c];
    L[r][r] += lambda * tr / 32.0;
    __syncthreads();
  }
  // ---- Cholesky (lower), both matrices at once: lane r owns row r of its matrix
  bool bad = false;
  for (int j = 0; j < 32; ++j) {
    double d = L[j][j];
    for (int k = 0; k < j; ++k) d -= L[j][k] * L[j][k];
    if (!(d > 0.0)) { bad = true; d = 1.0; }
    const double dj = sqrt(d);
    double v = 0.0;
    if (r > j) {
      v = L[r][j];
      for (int k = 0; k < j; ++k) v -= L[r][k] * L[j][k];
      v /= dj;
    }
    __syncthreads();
    if (r == j) L[j][j] = dj;
    else if (r > j) L[r][j] = v;
    else L[r][j] = 0.0;                                // zero the upper triangle
    __syncthreads();
  }
  if (__any(bad)) {
    if (lane == 0) atomicExch(status, 1);
  }
  // ---- A = W'^T X':  A[i][j] = sum_k W'[k][i] X'[k][j]   (16 outputs per lane)
  for (int o = lane; o < 1024; o += 64) {
    const int i = o >> 5, j = o & 31;
    double acc = 0.0;
    for (int k = max(i, j); k < 32; ++k) acc = fma(LW[k][i], LX[k][j], acc);
    A[i][j] = acc;
  }
  __syncthreads();
  // ---- one-sided Jacobi on the columns of A (right rotations): A V = U S
  const int pr = lane >> 2, sub = lane & 3;            // pair slot 0..15, 8 rows per lane
  for (int sweep = 0; sweep < 40; ++sweep) {
    if (lane == 0) conv = 1;
    __syncthreads();
    for (int rnd = 0; rnd < 31; ++rnd) {
      // circle method: position 0 fixed, the other 31 rotate
      const int pos_p = pr, pos_q = 31 - pr;
      const int p = pos_p == 0 ? 0 : 1 + (pos_p - 1 + rnd) % 31;
      const int q = 1 + (pos_q - 1 + rnd) % 31;
      double al = 0.0, be = 0.0, ga = 0.0;
      double ap[8], aq[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        ap[i] = A[8 * sub + i][p];
        aq[i] = A[8 * sub + i][q];
        al = fma(ap[i], ap[i], al);
        be = fma(aq[i], aq[i], be);
        ga = fma(ap[i], aq[i], ga);
      }
      al += __shfl_xor(al, 1, 64); be += __shfl_xor(be, 1, 64); ga += __shfl_xor(ga, 1, 64);
      al += __shfl_xor(al, 2, 64); be += __shfl_xor(be, 2, 64); ga += __shfl_xor(ga, 2, 64);
      if (fabs(ga) > 1e-15 * sqrt(al * be) && ga != 0.0) {
        const double zeta = (be - al) / (2.0 * ga);
        const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
        const double c = 1.0 / sqrt(1.0 + t * t), s = c * t;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          A[8 * sub + i][p] = c * ap[i] - s * aq[i];
          A[8 * sub + i][q] = s * ap[i] + c * aq[i];
        }
        conv = 0;
      }
      __syncthreads();
    }
    if (conv) break;
    __syncthreads();
  }
  // ---- singular values, descending order, U with the sign convention
  if (lane < 32) {
    double n2 = 0.0;
    for (int i = 0; i < 32; ++i) n2 = fma(A[i][lane], A[i][lane], n2);
    sv[lane] = sqrt(n2);
  }
  __syncthreads();
  if (lane < 32) {
    int rank = 0;
    for (int k = 0; k < 32; ++k) rank += (sv[k] > sv[lane]) || (sv[k] == sv[lane] && k < lane);
    order[rank] = lane;
  }
  __syncthreads();
  double s_mine = 0.0;
  if (lane < 32) {
    const int src = order[lane];
    s_mine = sv[src];
    double best = -1.0, bestv = 1.0;
    for (int i = 0; i < 32; ++i) {
      const double v = A[i][src] / s_mine;
      U[i][lane] = v;
      if (fabs(v) > best) { best = fabs(v); bestv = v; }
    }
    if (bestv < 0.0)
      for (int i = 0; i < 32; ++i) U[i][lane] = -U[i][lane];
  }
  __syncthreads();
  if (lane < 32) sv[lane] = s_mine;
  __syncthreads();
  // ---- B = diag(s^-1/2) U^T W'^T :  B[i][k] = s_i^-1/2 sum_m U[m][i] W'[k][m]
  for (int o = lane; o < 1024; o += 64) {
    const int i = o >> 5, k = o & 31;
    double acc = 0.0;
    for (int m = 0; m <= k; ++m) acc = fma(U[m][i], LW[k][m], acc);
    A[i][k] = acc / sqrt(sv[i]);
  }
  __syncthreads();
  // ---- T = H B with the normalized Sylvester matrix H[j][i] = (-1)^popcount(j & i) / sqrt(32)
  const double hn = 1.0 / sqrt(32.0);
  for (int o = lane; o < 1024; o += 64) {
    const int j = o >> 5, k = o & 31;
    double acc = 0.0;
    for (int i = 0; i < 32; ++i) acc += (__popc(j & i) & 1) ? -A[i][k] : A[i][k];
    acc *= hn;
    T_out[(int64_t)b * 1024 + o] = f64_to_bf16_bits(acc);
    if (T_f64) T_f64[(int64_t)b * 1024 + o] = acc;
  }
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
                                   int64_t K, double lambda, void* T_out, double* T_f64, void* workspace,
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
  wush_block_kernel<<<dim3(C), dim3(64), 0, stream>>>(partial, S, C, (int)N, (int)Mc, lambda, (uint16_t*)T_out, T_f64,
                                                      status);
  return hipGetLastError();
}

}  // namespace wush
