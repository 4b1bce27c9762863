// Wave-level FP64 pieces of the transform construction shared by the RTN-case
// and the GPTQ-case kernels: Alg. 1 on one block.
#pragma once
#include "wush_device.hpp"

namespace wush {

// Sum of the S values p[0], p[stride], ..., in ascending order (a fixed summation order), with the loads
// of eight terms in flight at a time: one at a time, each waits out a full memory latency.
__device__ __forceinline__ double ordered_sum(const double* __restrict__ p, int64_t stride, int S) {
  double acc = 0.0;
  for (int s0 = 0; s0 < S; s0 += 8) {
    double v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = s0 + u < S ? p[(int64_t)(s0 + u) * stride] : 0.0;
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u];
  }
  return acc;
}

// 1 / sqrt(x) for a positive normal x: the hardware estimate and two Newton steps (relative error of a
// few 2^-53; not correctly rounded, which the Jacobi rotations below do not need).
__device__ __forceinline__ double rsqrt_newton(double x) {
  double y = __builtin_amdgcn_rsq(x);
  const double hx = 0.5 * x;
  y = fma(y, fma(-hx * y, y, 0.5), y);
  y = fma(y, fma(-hx * y, y, 0.5), y);
  return y;
}

// The value of x in another lane of the same row of 16, chosen by a DPP control word (no LDS round trip).
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x) {
  const long long b = __double_as_longlong(x);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)b, CTRL, 0xF, 0xF, true);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xF, 0xF, true);
  return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
// Sum of x over the LANES adjacent lanes (4 or 8, aligned) that share a column pair, the same in each of
// them: partner lane ^ 1, then lane ^ 2 (quad permutes), then the mirrored lane of the other quad.
template <int LANES>
__device__ __forceinline__ double group_sum(double x) {
  static_assert(LANES == 4 || LANES == 8, "lanes per column pair");
  x += dpp_f64<0xB1>(x);    // quad_perm [1, 0, 3, 2]
  x += dpp_f64<0x4E>(x);    // quad_perm [2, 3, 0, 1]
  if (LANES == 8) x += dpp_f64<0x141>(x);   // row_half_mirror: lane i <-> 7 - i
  return x;
}

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
    // consecutive lanes fetch consecutive entries of a row (the moments come from global memory),
    // four entries per lane at a time so that their loads overlap
    constexpr int kPerLane = 2 * D * D / 64;
#pragma unroll 1
    for (int i0 = 0; i0 < kPerLane; i0 += 4) {
      double v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int e = lane + 64 * (i0 + u);
        v[u] = moment(e / (D * D), (e % (D * D)) / D, e % D);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int e = lane + 64 * (i0 + u);
        (e / (D * D) ? LX : LW)[(e % (D * D)) / D][e % D] = v[u];
      }
    }
    __syncthreads();
    double tr = 0.0;
    for (int c = 0; c < D; ++c) tr += L[c][c];
    const double damped = L[r][r] + lambda * tr / (double)D;
    __syncthreads();
    L[r][r] = damped;
    __syncthreads();
  }
  // ---- Cholesky (lower), both matrices at once: lane r owns row r of its matrix
  bool bad = false;
  for (int j = 0; j < D; ++j) {
    double d = L[j][j];
#pragma unroll 4
    for (int k = 0; k < j; ++k) d -= L[j][k] * L[j][k];
    if (!(d > 0.0)) { bad = true; d = 1.0; }
    const double dj = sqrt(d);
    double v = 0.0;
    if (r > j) {
      v = L[r][j];
#pragma unroll 4
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
#pragma unroll 4
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
      al = group_sum<kLpp>(al);
      be = group_sum<kLpp>(be);
      ga = group_sum<kLpp>(ga);
      if (ga * ga > 1e-30 * (al * be)) {             // |ga| > 1e-15 sqrt(al be)
        // The rotation by the angle of smaller magnitude that makes the two columns orthogonal:
        // tan(2 theta) = 2 ga / (be - al), |theta| <= pi / 4.  From cos(2 theta) = |be - al| / h and
        // sin(2 theta) = |2 ga| / h, h = hypot(be - al, 2 ga):  c^2 = (1 + cos 2 theta) / 2,
        // |s| = sin 2 theta / (2 c) -- two reciprocal square roots, no division, no cancellation.
        const double dd = be - al, g2 = 2.0 * ga;
        const double ih = rsqrt_newton(fma(dd, dd, g2 * g2));
        const double c2 = fma(0.5 * fabs(dd), ih, 0.5);
        const double ic = rsqrt_newton(c2);
        const double c = c2 * ic;
        const bool pos = dd == 0.0 || (dd > 0.0) == (g2 > 0.0);
        const double sa = 0.5 * fabs(g2) * ih * ic;
        const double s = pos ? sa : -sa;
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

