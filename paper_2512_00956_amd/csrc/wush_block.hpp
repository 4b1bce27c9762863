// Wave-level FP64 pieces of the transform construction shared by the RTN-case
// and the GPTQ-case kernels: Alg. 1 on one block.
#pragma once
#include "wush_device.hpp"

namespace wush {

// Alg. 1 for one D x D block (D = 32, or 16 for the NVFP4 variant), by ONE wavefront (64 lanes, all active):
//   W' W'^T = M_W + lambda d^-1 tr(M_W) I,  X' X'^T likewise  (Cholesky, side by side)
//   U S V^T = W'^T X'  (one-sided Jacobi on the columns; V never needed)
//   T = H S^(-1/2) U^T W'^T, singular values descending, the entry of largest
//   magnitude of every column of U positive.
// moment(h, r, c): entry (r, c) of the normalized, undamped second moment, h = 0
// for M_W, 1 for M_X.  T goes out as BF16 bits (T_bits) and, where the pointers
// are non-null, as FP64 before rounding (T_f64) and as the FP64 value of the
// rounded matrix (T_rounded), each [D][D] row-major.  A moment that is not
// positive definite sets *status.
template <int D, class MomentFn>
__device__ __forceinline__ void wush_block_wave(MomentFn moment, double lambda, uint16_t* __restrict__ T_bits,
                                                double* __restrict__ T_f64, double* __restrict__ T_rounded,
                                                int* __restrict__ status) {
  static_assert(D == 32 || D == 16, "block size");
  constexpr int kPairs = D / 2;          // disjoint column pairs per Jacobi round
  constexpr int kLpp = 64 / kPairs;      // lanes per pair
  constexpr int kRpl = D / kLpp;         // rows of a column pair per lane
  __shared__ double LW[D][D + 1];   // M_W, then W' (lower triangle)
  __shared__ double LX[D][D + 1];   // M_X, then X'
  __shared__ double A[D][D + 1];    // W'^T X', then U S (columns), then B
  __shared__ double U[D][D + 1];
  __shared__ double sv[D];
  __shared__ int order[D];
  __shared__ int conv;
  const int lane = threadIdx.x & 63;
  // lanes 0..D-1 own the rows of M_W, the next D those of M_X; with D = 16 the upper 32 lanes
  // repeat the lower ones (same values to the same addresses)
  const int half = (lane / D) & 1, r = lane % D;
  double (*L)[D + 1] = half ? LX : LW;
  {
    double tr = 0.0;
    for (int c = 0; c < D; ++c) L[r][c] = moment(half, r, c);
    __syncthreads();
    for (int c = 0; c < D; ++c) tr += L[c][c];
    L[r][r] += lambda * tr / (double)D;
    __syncthreads();
  }
  // ---- Cholesky (lower), both matrices at once: lane r owns row r of its matrix
  bool bad = false;
  for (int j = 0; j < D; ++j) {
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
  for (int o = lane; o < D * D; o += 64) {
    const int i = o / D, j = o % D;
    double acc = 0.0;
    for (int k = max(i, j); k < D; ++k) acc = fma(LW[k][i], LX[k][j], acc);
    A[i][j] = acc;
  }
  __syncthreads();
  // ---- one-sided Jacobi on the columns of A (right rotations): A V = U S
  const int pr = lane / kLpp, sub = lane % kLpp;       // pair slot, kRpl rows per lane
  for (int sweep = 0; sweep < 40; ++sweep) {
    if (lane == 0) conv = 1;
    __syncthreads();
    for (int rnd = 0; rnd < D - 1; ++rnd) {
      // circle method: position 0 fixed, the other D - 1 rotate
      const int pos_p = pr, pos_q = D - 1 - pr;
      const int p = pos_p == 0 ? 0 : 1 + (pos_p - 1 + rnd) % (D - 1);
      const int q = 1 + (pos_q - 1 + rnd) % (D - 1);
      double al = 0.0, be = 0.0, ga = 0.0;
      double ap[kRpl], aq[kRpl];
#pragma unroll
      for (int i = 0; i < kRpl; ++i) {
        ap[i] = A[kRpl * sub + i][p];
        aq[i] = A[kRpl * sub + i][q];
        al = fma(ap[i], ap[i], al);
        be = fma(aq[i], aq[i], be);
        ga = fma(ap[i], aq[i], ga);
      }
#pragma unroll
      for (int m = 1; m < kLpp; m <<= 1) {
        al += __shfl_xor(al, m, 64); be += __shfl_xor(be, m, 64); ga += __shfl_xor(ga, m, 64);
      }
      if (fabs(ga) > 1e-15 * sqrt(al * be) && ga != 0.0) {
        const double zeta = (be - al) / (2.0 * ga);
        const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
        const double c = 1.0 / sqrt(1.0 + t * t), s = c * t;
#pragma unroll
        for (int i = 0; i < kRpl; ++i) {
          A[kRpl * sub + i][p] = c * ap[i] - s * aq[i];
          A[kRpl * sub + i][q] = s * ap[i] + c * aq[i];
        }
        conv = 0;
      }
      __syncthreads();
    }
    if (conv) break;
    __syncthreads();
  }
  // ---- singular values, descending order, U with the sign convention
  if (lane < D) {
    double n2 = 0.0;
    for (int i = 0; i < D; ++i) n2 = fma(A[i][lane], A[i][lane], n2);
    sv[lane] = sqrt(n2);
  }
  __syncthreads();
  if (lane < D) {
    int rank = 0;
    for (int k = 0; k < D; ++k) rank += (sv[k] > sv[lane]) || (sv[k] == sv[lane] && k < lane);
    order[rank] = lane;
  }
  __syncthreads();
  double s_mine = 0.0;
  if (lane < D) {
    const int src = order[lane];
    s_mine = sv[src];
    double best = -1.0, bestv = 1.0;
    for (int i = 0; i < D; ++i) {
      const double v = A[i][src] / s_mine;
      U[i][lane] = v;
      if (fabs(v) > best) { best = fabs(v); bestv = v; }
    }
    if (bestv < 0.0)
      for (int i = 0; i < D; ++i) U[i][lane] = -U[i][lane];
  }
  __syncthreads();
  if (lane < D) sv[lane] = s_mine;
  __syncthreads();
  // ---- B = diag(s^-1/2) U^T W'^T :  B[i][k] = s_i^-1/2 sum_m U[m][i] W'[k][m]
  for (int o = lane; o < D * D; o += 64) {
    const int i = o / D, k = o % D;
    double acc = 0.0;
    for (int m = 0; m <= k; ++m) acc = fma(U[m][i], LW[k][m], acc);
    A[i][k] = acc / sqrt(sv[i]);
  }
  __syncthreads();
  // ---- T = H B with the normalized Sylvester matrix H[j][i] = (-1)^popcount(j & i) / sqrt(D)
  const double hn = 1.0 / sqrt((double)D);
  for (int o = lane; o < D * D; o += 64) {
    const int j = o / D, k = o % D;
    double acc = 0.0;
    for (int i = 0; i < D; ++i) acc += (__popc(j & i) & 1) ? -A[i][k] : A[i][k];
    acc *= hn;
    const uint16_t bits = f64_to_bf16_bits(acc);
    T_bits[o] = bits;
    if (T_f64) T_f64[o] = acc;
    if (T_rounded) T_rounded[o] = (double)bf16_bits_to_f32(bits);
  }
}

}  // namespace wush

