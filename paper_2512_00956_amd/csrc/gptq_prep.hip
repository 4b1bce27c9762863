// Offline weight path, GPTQ case of Alg. 2: WUSH transforms interleaved with
// GPTQ's intra-block and inter-block error propagation.  Everything is FP64; the
// path runs once per layer and is written for agreement with an FP64 reference.
//
// The paper's schedule uses L, the lower Cholesky factor of the inverse of the
// damped Hessian Hd = H + lambda tr(H)/d_in I, through three quantities per
// block i: (L_ii L_ii^T)^-1, and L_ji L_ii^-1 for j > i.  This file never
// inverts Hd.  With the reverse Cholesky factorization Hd = U U^T (U upper
// triangular) one has L = U^-T, hence
//     (L_ii L_ii^T)^-1       = U_ii U_ii^T
//     (L_ji L_ii^-1)^T       = U_ii (U^-1)_ij          (j > i)
// so the work is: H, its reverse Cholesky factor in place (blocked, right-
// looking from the last block), V = U^-1 (blocked, one workgroup per block row),
// and then the sequential loop over blocks:
//     M_W of the UPDATED weight block, Alg. 1 -> T_i (rounded to BF16),
//     Wbar = W_i inv(T_i),  Hbar = (T_i U_ii)(T_i U_ii)^T,
//     R = inverse of the reverse Cholesky factor of Hbar (R^T R = inv(Hbar)),
//     GPTQ subroutine on Wbar with R: per output channel, 32 steps of
//       quantize (static group scale), err = (w - q)/R[r][r], w[r'] -= err R[r][r'],
//     E = deq T_i - W_i,  W_rest += E (U_ii V_i,rest).
// Summation orders are fixed (no atomics), so the result is reproducible.
#include "wush_block.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

constexpr double kPivotFloor = 1e-290;

// ------------------------------------------------------------------ Hessian
// H = Xc^T Xc / M, 64 x 64 output tile per workgroup (tiles on or above the
// diagonal; the mirror image is written too).  Products of BF16 values are exact.
__global__ __launch_bounds__(256) void gptq_hessian_kernel(const uint16_t* __restrict__ X, int64_t ldx, int Mc, int K,
                                                           double* __restrict__ H) {
  const int ti = blockIdx.y, tj = blockIdx.x;
  if (tj < ti) return;
  __shared__ float a[32][65], b[32][65];
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  double acc[4][4] = {};
  const int lr = threadIdx.x >> 3, lc = (threadIdx.x & 7) * 8;   // one 16-byte chunk per thread and side
  for (int m0 = 0; m0 < Mc; m0 += 32) {
    __syncthreads();
#pragma unroll
    for (int side = 0; side < 2; ++side) {
      const int col = 64 * (side ? tj : ti) + lc;
      v4u raw = {0, 0, 0, 0};
      if (m0 + lr < Mc && col < K) raw = *reinterpret_cast<const v4u*>(X + (int64_t)(m0 + lr) * ldx + col);
      float (*dst)[65] = side ? b : a;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        dst[lr][lc + 2 * i] = __uint_as_float(raw[i] << 16);
        dst[lr][lc + 2 * i + 1] = __uint_as_float(raw[i] & 0xFFFF0000u);
      }
    }
    __syncthreads();
    for (int r = 0; r < 32; ++r) {
      double av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = a[r][4 * ty + i]; bv[i] = b[r][4 * tx + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fma(av[i], bv[j], acc[i][j]);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r = 64 * ti + 4 * ty + i, c = 64 * tj + 4 * tx + j;
      if (r < K && c < K) {
        const double v = acc[i][j] / (double)Mc;
        H[(int64_t)r * K + c] = v;
        H[(int64_t)c * K + r] = v;
      }
    }
}

// tr(H) in a fixed order, then: keep the undamped diagonal blocks (the M_X of
// every block) and add lambda tr(H)/K to the diagonal.
__global__ __launch_bounds__(256) void gptq_trace_kernel(const double* __restrict__ H, int K, double* __restrict__ tr_out) {
  __shared__ double part[256];
  double s = 0.0;
  for (int d = threadIdx.x; d < K; d += 256) s += H[(int64_t)d * K + d];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w >= 1; w >>= 1) {
    if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) tr_out[0] = part[0];
}

__global__ __launch_bounds__(256) void gptq_damp_kernel(double* __restrict__ H, int K, double lambda,
                                                        const double* __restrict__ tr, double* __restrict__ MX) {
  const int b = blockIdx.x;
  const double add = lambda * tr[0] / (double)K;
  for (int o = threadIdx.x; o < 1024; o += 256) {
    const int r = o >> 5, c = o & 31;
    const int64_t idx = (int64_t)(32 * b + r) * K + 32 * b + c;
    const double v = H[idx];
    MX[(int64_t)b * 1024 + o] = v;
    if (r == c) H[idx] = v + add;
  }
}

// ------------------------------------------------- 32 x 32 building blocks
// (one wavefront; matrices in LDS with a padded row)

// U upper triangular with U U^T = S (S symmetric positive definite, overwritten:
// upper triangle = U, strict lower triangle = 0).  Lane r < 32 owns row r.
__device__ __forceinline__ bool reverse_cholesky32(double (*S)[33], int lane) {
  bool bad = false;
  const int r = lane & 31;
  for (int j = 31; j >= 0; --j) {
    double d = S[j][j];
#pragma unroll 4
    for (int l = j + 1; l < 32; ++l) d -= S[j][l] * S[j][l];
    if (!(d > 0.0)) { bad = true; d = 1.0; }
    const double dj = sqrt(d);
    double v = 0.0;
    if (r < j) {
      v = S[r][j];
#pragma unroll 4
      for (int l = j + 1; l < 32; ++l) v -= S[r][l] * S[j][l];
      v /= dj;
    }
    __syncthreads();
    if (lane < 32) {
      if (r == j) S[j][j] = dj;
      else if (r < j) S[r][j] = v;
      else S[r][j] = 0.0;
    }
    __syncthreads();
  }
  return bad;
}

// Vout = inverse of the upper triangular U (both [32][33] in LDS); lane c < 32
// computes column c by back substitution.
__device__ __forceinline__ void upper_inverse32(const double (*U)[33], double (*Vout)[33], int lane) {
  if (lane < 32) {
    const int c = lane;
    double x[32];
#pragma unroll
    for (int r = 31; r >= 0; --r) {
      double acc = (r == c) ? 1.0 : 0.0;
#pragma unroll
      for (int l = r + 1; l < 32; ++l) acc -= U[r][l] * x[l];
      x[r] = (r <= c) ? acc / U[r][r] : 0.0;
    }
#pragma unroll
    for (int r = 0; r < 32; ++r) Vout[r][c] = x[r];
  }
  __syncthreads();
}

// ------------------------------------------------ reverse Cholesky of Hd
__global__ __launch_bounds__(64) void gptq_rchol_diag_kernel(double* __restrict__ H, int K, int i, int* __restrict__ status) {
  __shared__ double S[32][33];
  const int lane = threadIdx.x;
  for (int o = lane; o < 1024; o += 64) S[o >> 5][o & 31] = H[(int64_t)(32 * i + (o >> 5)) * K + 32 * i + (o & 31)];
  __syncthreads();
  const bool bad = reverse_cholesky32(S, lane);
  if (__any(bad) && lane == 0) atomicExch(status, 1);
  for (int o = lane; o < 1024; o += 64) H[(int64_t)(32 * i + (o >> 5)) * K + 32 * i + (o & 31)] = S[o >> 5][o & 31];
}

// rows above block i: U_ki = S_ki U_ii^-T, one thread per row (x U_ii^T = s by back substitution)
__global__ __launch_bounds__(256) void gptq_rchol_panel_kernel(double* __restrict__ H, int K, int i) {
  __shared__ double U[32][33];
  for (int o = threadIdx.x; o < 1024; o += 256) U[o >> 5][o & 31] = H[(int64_t)(32 * i + (o >> 5)) * K + 32 * i + (o & 31)];
  __syncthreads();
  const int row = blockIdx.x * 256 + threadIdx.x;
  if (row >= 32 * i) return;
  double* p = H + (int64_t)row * K + 32 * i;
  double x[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) x[j] = p[j];
#pragma unroll
  for (int j = 31; j >= 0; --j) {
    double acc = x[j];
#pragma unroll
    for (int l = j + 1; l < 32; ++l) acc -= x[l] * U[j][l];
    x[j] = acc / U[j][j];
  }
#pragma unroll
  for (int j = 0; j < 32; ++j) p[j] = x[j];
}

// trailing update: S_kl -= U_ki U_li^T for block pairs k <= l < i (one 32 x 32 block per workgroup)
__global__ __launch_bounds__(256) void gptq_rchol_update_kernel(double* __restrict__ H, int K, int i) {
  const int k = blockIdx.y, l = blockIdx.x;
  if (k > l) return;
  __shared__ double pk[32][33], pl[32][33];
  for (int o = threadIdx.x; o < 1024; o += 256) {
    pk[o >> 5][o & 31] = H[(int64_t)(32 * k + (o >> 5)) * K + 32 * i + (o & 31)];
    pl[o >> 5][o & 31] = H[(int64_t)(32 * l + (o >> 5)) * K + 32 * i + (o & 31)];
  }
  __syncthreads();
  const int r = threadIdx.x >> 3, c0 = (threadIdx.x & 7) * 4;
  double acc[4] = {0, 0, 0, 0};
  for (int m = 0; m < 32; ++m) {
    const double a = pk[r][m];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = fma(a, pl[c0 + t][m], acc[t]);
  }
  double* out = H + (int64_t)(32 * k + r) * K + 32 * l + c0;
#pragma unroll
  for (int t = 0; t < 4; ++t) out[t] -= acc[t];
}

// ------------------------------------------------------------ V = U^-1
__global__ __launch_bounds__(64) void gptq_triinv_diag_kernel(const double* __restrict__ H, int K, double* __restrict__ V) {
  __shared__ double U[32][33], Vi[32][33];
  const int i = blockIdx.x, lane = threadIdx.x;
  for (int o = lane; o < 1024; o += 64) U[o >> 5][o & 31] = H[(int64_t)(32 * i + (o >> 5)) * K + 32 * i + (o & 31)];
  __syncthreads();
  upper_inverse32(U, Vi, lane);
  for (int o = lane; o < 1024; o += 64) V[(int64_t)(32 * i + (o >> 5)) * K + 32 * i + (o & 31)] = Vi[o >> 5][o & 31];
}

// block row i of V: V_ij = -(sum_{k=i}^{j-1} V_ik U_kj) V_jj for j = i+1 .. C-1.
// The workgroup reads back what it wrote for smaller j; the workgroup barrier orders that.
// The 32 x 32 block products run on the FP64 MFMA (16 x 16 x 4), one 16 x 16 output tile per wave:
// with scalar FMAs the kernel was bound by its LDS reads (five per four FMAs), and its longest chain
// (block row 0: C^2 / 2 products one after the other) is the whole kernel's duration.
typedef double v4d_t __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void gptq_triinv_rows_kernel(const double* __restrict__ H, int K, int C,
                                                               double* __restrict__ V) {
  __shared__ double va[32][33], ub[32][33], acc_s[32][33];
  const int i = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tr = 16 * (wave >> 1), tc = 16 * (wave & 1);      // this wave's output tile
  const int l16 = lane & 15, l4 = lane >> 4;
  // A[row l16][k l4] and B[k l4][column l16] of the MFMA; accumulator element v is (row l4 + 4 v, column l16)
  auto product = [&](const double (*a)[33], const double (*b)[33], v4d_t acc) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[tr + l16][4 * kk + l4], b[4 * kk + l4][tc + l16], acc, 0, 0, 0);
    return acc;
  };
  // the blocks of step k + 1 travel from memory into registers while step k is multiplied
  double rv[4], ru[4];
  auto fetch = [&](int k, int j) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int o = threadIdx.x + 256 * u;
      rv[u] = V[(int64_t)(32 * i + (o >> 5)) * K + 32 * k + (o & 31)];
      ru[u] = H[(int64_t)(32 * k + (o >> 5)) * K + 32 * j + (o & 31)];
    }
  };
  for (int j = i + 1; j < C; ++j) {
    v4d_t acc = {0, 0, 0, 0};
    fetch(i, j);
    for (int k = i; k < j; ++k) {
      __syncthreads();
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int o = threadIdx.x + 256 * u;
        va[o >> 5][o & 31] = rv[u];
        ub[o >> 5][o & 31] = ru[u];
      }
      __syncthreads();
      if (k + 1 < j) fetch(k + 1, j);
      acc = product(va, ub, acc);
    }
    __syncthreads();
#pragma unroll
    for (int v = 0; v < 4; ++v) acc_s[tr + l4 + 4 * v][tc + l16] = acc[v];
    for (int o = threadIdx.x; o < 1024; o += 256)
      ub[o >> 5][o & 31] = V[(int64_t)(32 * j + (o >> 5)) * K + 32 * j + (o & 31)];   // V_jj
    __syncthreads();
    const v4d_t out = product(acc_s, ub, (v4d_t){0, 0, 0, 0});
#pragma unroll
    for (int v = 0; v < 4; ++v) V[(int64_t)(32 * i + tr + l4 + 4 * v) * K + 32 * j + tc + l16] = -out[v];
    __threadfence_block();
  }
}

// ------------------------------------------------------ per-block kernels
__global__ __launch_bounds__(256) void gptq_widen_kernel(const uint16_t* __restrict__ W, int64_t ldw, int N, int K,
                                                         double* __restrict__ Wf) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)N * K) return;
  const int n = (int)(idx / K), k = (int)(idx % K);
  Wf[idx] = (double)bf16_bits_to_f32(W[(int64_t)n * ldw + k]);
}

// partial second moments of the current weight block: split s sums its rows
__global__ __launch_bounds__(256) void gptq_moment_kernel(const double* __restrict__ Wf, int N, int K, int i,
                                                          int rows_per_split, double* __restrict__ partial) {
  __shared__ double tile[64][33];
  const int s = blockIdx.x;
  const int r_begin = min(s * rows_per_split, N), r_end = min(r_begin + rows_per_split, N);
  const int ti = threadIdx.x >> 4, tj = threadIdx.x & 15;
  double a00 = 0, a01 = 0, a10 = 0, a11 = 0;
  for (int r0 = r_begin; r0 < r_end; r0 += 64) {
    __syncthreads();
    for (int o = threadIdx.x; o < 64 * 32; o += 256) {
      const int rr = o >> 5, c = o & 31;
      tile[rr][c] = (r0 + rr < r_end) ? Wf[(int64_t)(r0 + rr) * K + 32 * i + c] : 0.0;
    }
    __syncthreads();
    for (int rr = 0; rr < 64; ++rr) {
      const double ax = tile[rr][2 * ti], ay = tile[rr][2 * ti + 1], cx = tile[rr][2 * tj], cy = tile[rr][2 * tj + 1];
      a00 = fma(ax, cx, a00);
      a01 = fma(ax, cy, a01);
      a10 = fma(ay, cx, a10);
      a11 = fma(ay, cy, a11);
    }
  }
  double* out = partial + (int64_t)s * 1024;
  out[(2 * ti) * 32 + 2 * tj] = a00;
  out[(2 * ti) * 32 + 2 * tj + 1] = a01;
  out[(2 * ti + 1) * 32 + 2 * tj] = a10;
  out[(2 * ti + 1) * 32 + 2 * tj + 1] = a11;
}

// Alg. 1 on (M_W of the updated block, M_X = diagonal block of H): T_i
__global__ __launch_bounds__(64) void gptq_wush_kernel(const double* __restrict__ partial, int S, int N,
                                                       const double* __restrict__ MX_i, double lambda,
                                                       uint16_t* __restrict__ T_bits_i, double* __restrict__ Tb,
                                                       int* __restrict__ status) {
  auto moment = [&](int half, int r, int c) {
    if (half) return MX_i[r * 32 + c];
    return ordered_sum(partial + r * 32 + c, 1024, S) / (double)N;
  };
  wush_block_wave<32>(moment, lambda, T_bits_i, nullptr, Tb, status);
}

// identity / fixed transforms for comparisons: T_i given, only widen it
__global__ __launch_bounds__(64) void gptq_fixed_transform_kernel(const uint16_t* __restrict__ T_bits_i,
                                                                  double* __restrict__ Tb) {
  for (int o = threadIdx.x; o < 1024; o += 64) Tb[o] = (double)bf16_bits_to_f32(T_bits_i[o]);
}

// From T_i (BF16-valued) and U_ii: inv(T_i) (Gauss-Jordan, partial pivoting) and
// R = inverse of the reverse Cholesky factor of Hbar = (T_i U_ii)(T_i U_ii)^T.
__global__ __launch_bounds__(64) void gptq_block_mats_kernel(const double* __restrict__ Tb, const double* __restrict__ H,
                                                             int K, int i, double* __restrict__ Tinv,
                                                             double* __restrict__ R, int* __restrict__ status) {
  __shared__ double a[32][65];
  __shared__ double B[32][33], Hb[32][33], Rm[32][33];
  const int lane = threadIdx.x;
  // ---- inverse of T_i
  for (int r = 0; r < 32; ++r) a[r][lane] = lane < 32 ? Tb[r * 32 + lane] : ((lane - 32 == r) ? 1.0 : 0.0);
  __syncthreads();
  bool singular = false;
  for (int p = 0; p < 32; ++p) {
    const int rr = lane & 31;
    double mag = (rr >= p) ? fabs(a[rr][p]) : -1.0;
    int idx = rr;
    for (int off = 16; off >= 1; off >>= 1) {
      const double omag = __shfl_xor(mag, off, 64);
      const int oidx = __shfl_xor(idx, off, 64);
      if (omag > mag || (omag == mag && oidx < idx)) { mag = omag; idx = oidx; }
    }
    if (!(mag > kPivotFloor)) { singular = true; break; }   // uniform across the wave
    if (idx != p) {
      const double t0 = a[p][lane];
      a[p][lane] = a[idx][lane];
      a[idx][lane] = t0;
    }
    __syncthreads();
    const double inv_piv = 1.0 / a[p][p];
    __syncthreads();
    const double prow = a[p][lane] * inv_piv;
    a[p][lane] = prow;
    __syncthreads();
    // column p (the factors) is read whole before any lane touches it: lane p updates it below
    double f[32];
#pragma unroll
    for (int r = 0; r < 32; ++r) f[r] = a[r][p];
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 32; ++r)
      if (r != p) a[r][lane] -= f[r] * prow;
    __syncthreads();
  }
  if (singular && lane == 0) atomicExch(status, 1);
  for (int r = 0; r < 32; ++r)
    if (lane >= 32) Tinv[r * 32 + (lane - 32)] = singular ? 0.0 : a[r][lane];
  // ---- B = T_i U_ii (U_ii upper triangular), Hbar = B B^T
  for (int o = lane; o < 1024; o += 64) {
    Rm[o >> 5][o & 31] = H[(int64_t)(32 * i + (o >> 5)) * K + 32 * i + (o & 31)];
    Hb[o >> 5][o & 31] = Tb[o];                       // T_i, until Hbar takes its place
  }
  __syncthreads();
  for (int o = lane; o < 1024; o += 64) {
    const int r = o >> 5, c = o & 31;
    double acc = 0.0;
#pragma unroll 4
    for (int m = 0; m <= c; ++m) acc = fma(Hb[r][m], Rm[m][c], acc);
    B[r][c] = acc;
  }
  __syncthreads();
  for (int o = lane; o < 1024; o += 64) {
    const int r = o >> 5, c = o & 31;
    double acc = 0.0;
#pragma unroll 8
    for (int m = 0; m < 32; ++m) acc = fma(B[r][m], B[c][m], acc);
    Hb[r][c] = acc;
  }
  __syncthreads();
  const bool bad = reverse_cholesky32(Hb, lane);
  if (__any(bad) && lane == 0) atomicExch(status, 1);
  upper_inverse32(Hb, Rm, lane);
  for (int o = lane; o < 1024; o += 64) R[o] = Rm[o >> 5][o & 31];
}

// P = U_ii V[block row i][columns past block i]: the inter-block propagation matrix, [32][K]
__global__ __launch_bounds__(256) void gptq_pmat_kernel(const double* __restrict__ H, const double* __restrict__ V,
                                                        int K, int i, double* __restrict__ P) {
  __shared__ double U[32][33];
  for (int o = threadIdx.x; o < 1024; o += 256) U[o >> 5][o & 31] = H[(int64_t)(32 * i + (o >> 5)) * K + 32 * i + (o & 31)];
  __syncthreads();
  const int c = 32 * (i + 1) + blockIdx.x * 256 + threadIdx.x;
  if (c >= K) return;
  double v[32];
#pragma unroll
  for (int m = 0; m < 32; ++m) v[m] = V[(int64_t)(32 * i + m) * K + c];
#pragma unroll
  for (int r = 0; r < 32; ++r) {
    double acc = 0.0;
#pragma unroll
    for (int m = r; m < 32; ++m) acc = fma(U[r][m], v[m], acc);
    P[(int64_t)r * K + c] = acc;
  }
}

// The GPTQ subroutine on the transformed block, one thread per output channel,
// the codes and scale of the block, and the error in the original space.
__global__ __launch_bounds__(64) void gptq_quant_kernel(const double* __restrict__ Wf, int N, int K, int i,
                                                         const double* __restrict__ Tb, const double* __restrict__ Tinv,
                                                         const double* __restrict__ R, int rule, int tiled,
                                                         uint8_t* __restrict__ Wq, uint8_t* __restrict__ Ws,
                                                         double* __restrict__ E) {
  __shared__ double ti[32][32], tb[32][32], rm[32][32];
  for (int o = threadIdx.x; o < 1024; o += 64) {
    ti[o >> 5][o & 31] = Tinv[o];
    tb[o >> 5][o & 31] = Tb[o];
    rm[o >> 5][o & 31] = R[o];
  }
  __syncthreads();
  const int n = blockIdx.x * 64 + threadIdx.x;
  if (n >= N) return;
  double w[32], y[32];
  const double* wp = Wf + (int64_t)n * K + 32 * i;
#pragma unroll
  for (int k = 0; k < 32; ++k) w[k] = wp[k];
  double amax = 0.0;
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    double acc = 0.0;
#pragma unroll
    for (int k = 0; k < 32; ++k) acc = fma(w[k], ti[k][j], acc);
    y[j] = acc;
    amax = fmax(amax, fabs(acc));
  }
  const int byte = scale_byte_f64(amax, rule);   // static group scale: taken before any update
  const double inv_scale = __longlong_as_double((int64_t)(uint64_t)(1023 + 127 - byte) << 52);   // 2^(127-byte)
  const double scale = __longlong_as_double((int64_t)(uint64_t)(1023 - 127 + byte) << 52);       // 2^(byte-127)
  double dq[32];
  uint32_t words[4] = {0, 0, 0, 0};
#pragma unroll
  for (int r = 0; r < 32; ++r) {
#pragma clang fp contract(off)   // the reference subtracts a rounded product: no fused multiply-add here
    const double v = y[r];
    const uint32_t sign = (uint32_t)(((uint64_t)__double_as_longlong(v)) >> 63);
    const uint32_t code = e2m1_code_f64(fabs(v) * inv_scale);
    words[r >> 3] |= ((sign << 3) | code) << (4 * (r & 7));
    const double mag = (code < 4 ? 0.5 * (double)code : (code == 4 ? 2.0 : (code == 5 ? 3.0 : (code == 6 ? 4.0 : 6.0)))) * scale;
    dq[r] = sign ? -mag : mag;
    const double err = (v - dq[r]) / rm[r][r];
#pragma unroll
    for (int rp = r + 1; rp < 32; ++rp) y[rp] = y[rp] - err * rm[r][rp];
  }
  const v4u chunk = {words[0], words[1], words[2], words[3]};
  if (tiled) {
    *reinterpret_cast<v4u*>(Wq + tiled_chunk_offset(n, i, K >> 8)) = chunk;
    Ws[tiled_scale_offset(n, i, K >> 8)] = (uint8_t)byte;
  } else {
    *reinterpret_cast<v4u*>(Wq + (int64_t)n * (K / 2) + 16 * i) = chunk;
    Ws[(int64_t)n * (K / 32) + i] = (uint8_t)byte;
  }
  double* e = E + (int64_t)n * 32;
#pragma unroll
  for (int k = 0; k < 32; ++k) {
    double acc = 0.0;
#pragma unroll
    for (int j = 0; j < 32; ++j) acc = fma(dq[j], tb[j][k], acc);
    e[k] = acc - wp[k];   // read again rather than kept in registers through the recurrence
  }
}

// W[:, columns past block i] += E P, 64 x 64 tile per workgroup
__global__ __launch_bounds__(256) void gptq_propagate_kernel(double* __restrict__ Wf, int N, int K, int i,
                                                             const double* __restrict__ E, const double* __restrict__ P) {
  __shared__ double es[64][33], ps[32][65];
  const int n0 = blockIdx.y * 64, c0 = 32 * (i + 1) + blockIdx.x * 64;
  for (int o = threadIdx.x; o < 64 * 32; o += 256) {
    const int r = o >> 5, m = o & 31;
    es[r][m] = (n0 + r < N) ? E[(int64_t)(n0 + r) * 32 + m] : 0.0;
  }
  for (int o = threadIdx.x; o < 32 * 64; o += 256) {
    const int m = o >> 6, c = o & 63;
    ps[m][c] = (c0 + c < K) ? P[(int64_t)m * K + c0 + c] : 0.0;
  }
  __syncthreads();
  // rank-32 update on the FP64 MFMA (16 x 16 x 4): wave w owns rows 16 w .. 16 w + 15 of the tile and its
  // four 16-column blocks; A[row l16][k l4] is shared by the four, B[k l4][column l16] differs
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l16 = lane & 15, l4 = lane >> 4;
  // accumulator element v of column block tc: row l4 + 4 v, column l16.  The weights it updates are
  // requested before the products, so that the kernel runs at the rate of its memory traffic.
  double w[4][4];
#pragma unroll
  for (int tc = 0; tc < 4; ++tc)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int n = n0 + 16 * wave + l4 + 4 * v, c = c0 + 16 * tc + l16;
      w[tc][v] = (n < N && c < K) ? Wf[(int64_t)n * K + c] : 0.0;
    }
  double ev[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) ev[kk] = es[16 * wave + l16][4 * kk + l4];
#pragma unroll
  for (int tc = 0; tc < 4; ++tc) {
    v4d_t acc = {0, 0, 0, 0};
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      acc = __builtin_amdgcn_mfma_f64_16x16x4f64(ev[kk], ps[4 * kk + l4][16 * tc + l16], acc, 0, 0, 0);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int n = n0 + 16 * wave + l4 + 4 * v, c = c0 + 16 * tc + l16;
      if (n < N && c < K) Wf[(int64_t)n * K + c] = w[tc][v] + acc[v];
    }
  }
}

__global__ void gptq_reset_status_kernel(int* status) {
  if (threadIdx.x < 4) status[threadIdx.x] = 0;
}

constexpr int kMomentSplits = 64;

struct Layout {
  size_t H, V, Wf, MX, partial, Tb, Tinv, R, P, E, tr, status, total;
};

Layout layout(int64_t N, int64_t K) {
  Layout L{};
  size_t off = 0;
  auto take = [&](size_t doubles) { const size_t o = off; off += (doubles * sizeof(double) + 255) / 256 * 256; return o; };
  const size_t C = (size_t)(K / 32);
  L.H = take((size_t)K * K);
  L.V = take((size_t)K * K);
  L.Wf = take((size_t)N * K);
  L.MX = take(C * 1024);
  L.partial = take((size_t)kMomentSplits * 1024);
  L.Tb = take(1024);
  L.Tinv = take(1024);
  L.R = take(1024);
  L.P = take((size_t)32 * K);
  L.E = take((size_t)N * 32);
  L.tr = take(4);
  L.status = take(4);
  L.total = off;
  return L;
}

}  // namespace

size_t gptq_prep_workspace_bytes(int64_t N, int64_t K) { return layout(N, K).total; }
size_t gptq_prep_status_offset(int64_t N, int64_t K) { return layout(N, K).status; }

#define WUSH_GPTQ_CHECK()                 \
  {                                       \
    const hipError_t e_ = hipGetLastError(); \
    if (e_ != hipSuccess) return e_;      \
  }

hipError_t launch_gptq_prep(const void* W, int64_t N, int64_t K, int64_t ldw, const void* Xc, int64_t Mc, int64_t ldx,
                            double lambda, int transform_given, int rule, int tiled, void* T_blocks, void* Wq, void* Ws,
                            void* workspace, hipStream_t st) {
  const Layout L = layout(N, K);
  char* base = static_cast<char*>(workspace);
  auto D = [&](size_t off) { return reinterpret_cast<double*>(base + off); };
  double *H = D(L.H), *V = D(L.V), *Wf = D(L.Wf), *MX = D(L.MX), *partial = D(L.partial), *Tb = D(L.Tb),
         *Tinv = D(L.Tinv), *R = D(L.R), *P = D(L.P), *E = D(L.E), *tr = D(L.tr);
  int* status = reinterpret_cast<int*>(base + L.status);
  const int C = (int)(K / 32), Ki = (int)K, Ni = (int)N;
  uint16_t* Tbits = static_cast<uint16_t*>(T_blocks);

  gptq_reset_status_kernel<<<1, 64, 0, st>>>(status);
  WUSH_GPTQ_CHECK()
  gptq_widen_kernel<<<(unsigned)(((int64_t)N * K + 255) / 256), 256, 0, st>>>((const uint16_t*)W, ldw, Ni, Ki, Wf);
  WUSH_GPTQ_CHECK()
  const unsigned t64 = (unsigned)((K + 63) / 64);
  gptq_hessian_kernel<<<dim3(t64, t64), 256, 0, st>>>((const uint16_t*)Xc, ldx, (int)Mc, Ki, H);
  WUSH_GPTQ_CHECK()
  gptq_trace_kernel<<<1, 256, 0, st>>>(H, Ki, tr);
  WUSH_GPTQ_CHECK()
  gptq_damp_kernel<<<C, 256, 0, st>>>(H, Ki, lambda, tr, MX);
  WUSH_GPTQ_CHECK()
  // reverse Cholesky, last block first
  for (int i = C - 1; i >= 0; --i) {
    gptq_rchol_diag_kernel<<<1, 64, 0, st>>>(H, Ki, i, status);
    WUSH_GPTQ_CHECK()
    if (i > 0) {
      gptq_rchol_panel_kernel<<<(unsigned)((32 * i + 255) / 256), 256, 0, st>>>(H, Ki, i);
      WUSH_GPTQ_CHECK()
      gptq_rchol_update_kernel<<<dim3(i, i), 256, 0, st>>>(H, Ki, i);
      WUSH_GPTQ_CHECK()
    }
  }
  gptq_triinv_diag_kernel<<<C, 64, 0, st>>>(H, Ki, V);
  WUSH_GPTQ_CHECK()
  gptq_triinv_rows_kernel<<<C, 256, 0, st>>>(H, Ki, C, V);
  WUSH_GPTQ_CHECK()
  const int rows_per_split = (int)((N + kMomentSplits - 1) / kMomentSplits);
  for (int i = 0; i < C; ++i) {
    if (transform_given) {
      gptq_fixed_transform_kernel<<<1, 64, 0, st>>>(Tbits + (int64_t)i * 1024, Tb);
    } else {
      gptq_moment_kernel<<<kMomentSplits, 256, 0, st>>>(Wf, Ni, Ki, i, rows_per_split, partial);
      WUSH_GPTQ_CHECK()
      gptq_wush_kernel<<<1, 64, 0, st>>>(partial, kMomentSplits, Ni, MX + (int64_t)i * 1024, lambda,
                                         Tbits + (int64_t)i * 1024, Tb, status);
    }
    WUSH_GPTQ_CHECK()
    gptq_block_mats_kernel<<<1, 64, 0, st>>>(Tb, H, Ki, i, Tinv, R, status);
    WUSH_GPTQ_CHECK()
    gptq_quant_kernel<<<(unsigned)((N + 63) / 64), 64, 0, st>>>(Wf, Ni, Ki, i, Tb, Tinv, R, rule, tiled,
                                                                  (uint8_t*)Wq, (uint8_t*)Ws, E);
    WUSH_GPTQ_CHECK()
    if (i + 1 < C) {
      const int rest = Ki - 32 * (i + 1);
      gptq_pmat_kernel<<<(unsigned)((rest + 255) / 256), 256, 0, st>>>(H, V, Ki, i, P);
      WUSH_GPTQ_CHECK()
      gptq_propagate_kernel<<<dim3((unsigned)((rest + 63) / 64), (unsigned)((N + 63) / 64)), 256, 0, st>>>(Wf, Ni, Ki, i, E, P);
      WUSH_GPTQ_CHECK()
    }
  }
  return hipSuccess;
}
#undef WUSH_GPTQ_CHECK

}  // namespace wush
