// Offline weight path (Alg. 2, RTN case): T_xvsh = T_wush^{-T}, then
// q(T_xvsh W).  Also the quantizer-only test tap on FP32 values.
//
//   1. invert_blocks_kernel: one wavefront per 32x32 block, FP64 Gauss-Jordan
//      with partial pivoting on the augmented matrix [T | I] held in LDS.
//   2. weight_apply_quant_kernel: Wt = W_blk . inv(T_b) in FP64 (inv(T_b) in
//      LDS, one thread per (row, block) group), then the same RTN AbsMax MXFP4
//      rules as the activation kernel, evaluated on the FP64 values.
// This path runs once per layer, offline; it is written for exactness against
// an FP64 reference, not for speed.
#include "nvfp4_layout.hpp"
#include "wush_device.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

constexpr double kPivotFloor = 1e-290;

__global__ __launch_bounds__(64) void invert_blocks_kernel(const uint16_t* __restrict__ T,
                                                           double* __restrict__ Tinv,
                                                           int* __restrict__ status) {
  __shared__ double a[32][65];  // [T | I], padded row
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  for (int r = 0; r < 32; ++r) {
    double v;
    if (lane < 32) v = (double)bf16_bits_to_f32(T[((int64_t)b * 32 + r) * 32 + lane]);
    else v = (lane - 32 == r) ? 1.0 : 0.0;
    a[r][lane] = v;
  }
  __syncthreads();
  bool singular = false;
  for (int p = 0; p < 32; ++p) {
    // pivot search over rows p..31 in column p (first row of largest magnitude)
    double best = -1.0;
    int brow = p;
    {
      const int r = lane & 31;
      double mag = (r >= p) ? fabs(a[r][p]) : -1.0;
      int idx = r;
      for (int off = 16; off >= 1; off >>= 1) {
        const double omag = __shfl_xor(mag, off, 64);
        const int oidx = __shfl_xor(idx, off, 64);
        if (omag > mag || (omag == mag && oidx < idx)) { mag = omag; idx = oidx; }
      }
      best = mag;
      brow = idx;
    }
    if (!(best > kPivotFloor)) { singular = true; break; }  // uniform across the wave
    if (brow != p) {
      const double t0 = a[p][lane];
      a[p][lane] = a[brow][lane];
      a[brow][lane] = t0;
    }
    __syncthreads();
    const double inv_piv = 1.0 / a[p][p];
    __syncthreads();
    const double prow = a[p][lane] * inv_piv;
    a[p][lane] = prow;
    __syncthreads();
    for (int r = 0; r < 32; ++r) {
      if (r == p) continue;
      const double f = a[r][p];
      __syncthreads();
      a[r][lane] -= f * prow;
    }
    __syncthreads();
  }
  if (singular) {
    if (lane == 0) atomicExch(status, 1);
    for (int r = 0; r < 32; ++r)
      if (lane < 32) Tinv[((int64_t)b * 32 + r) * 32 + lane] = 0.0;
    return;
  }
  for (int r = 0; r < 32; ++r)
    if (lane >= 32) Tinv[((int64_t)b * 32 + r) * 32 + (lane - 32)] = a[r][lane];
}

__global__ void reset_status_kernel(int* status) {
  if (threadIdx.x < 4) status[threadIdx.x] = 0;
}

__global__ __launch_bounds__(256) void weight_apply_quant_kernel(
    const uint16_t* __restrict__ W, int64_t ldw, const double* __restrict__ Tinv,
    uint8_t* __restrict__ Wq, uint8_t* __restrict__ Ws, int N, int K, int C, int rule, int tiled) {
  __shared__ double ti[32][32];  // inv(T_b)[k][j]
  const int b = blockIdx.y;
  for (int i = threadIdx.x; i < 1024; i += 256) ti[i >> 5][i & 31] = Tinv[(int64_t)b * 1024 + i];
  __syncthreads();
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  double w[32];
  const uint16_t* wp = W + (int64_t)n * ldw + 32 * b;
#pragma unroll
  for (int k = 0; k < 32; k += 8) {
    const v4u raw = *reinterpret_cast<const v4u*>(wp + k);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      w[k + 2 * i] = (double)__uint_as_float(raw[i] << 16);
      w[k + 2 * i + 1] = (double)__uint_as_float(raw[i] & 0xFFFF0000u);
    }
  }
  double y[32];
  double amax = 0.0;
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    double acc = 0.0;
#pragma unroll
    for (int k = 0; k < 32; ++k) acc = fma(w[k], ti[k][j], acc);
    y[j] = acc;
    amax = fmax(amax, fabs(acc));
  }
  const int byte = scale_byte_f64(amax, rule);
  const double inv_scale = __longlong_as_double((int64_t)(uint64_t)(1023 + 127 - byte) << 52);  // 2^(127-byte)
  uint32_t words[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    uint32_t wd = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const double v = y[8 * g + i];
      const uint32_t sign = (uint32_t)(((uint64_t)__double_as_longlong(v)) >> 63);
      wd |= ((sign << 3) | e2m1_code_f64(fabs(v) * inv_scale)) << (4 * i);
    }
    words[g] = wd;
  }
  const v4u chunk = {words[0], words[1], words[2], words[3]};
  if (tiled) {
    *reinterpret_cast<v4u*>(Wq + tiled_chunk_offset(n, b, K >> 8)) = chunk;
    Ws[tiled_scale_offset(n, b, K >> 8)] = (uint8_t)byte;
  } else {
    *reinterpret_cast<v4u*>(Wq + (int64_t)n * (K / 2) + 16 * b) = chunk;
    Ws[(int64_t)n * C + b] = (uint8_t)byte;
  }
}

// INT4 variant (Table 1: 4-bit integers, BF16 scale per 32 = Gaussian-MSE-optimal step times the
// group's root mean square): the same FP64 product, then the quantizer decided in FP64 with one IEEE
// operation per step and no fused multiply-add in the sum of squares (channels 0..15 left to right,
// channels 16..31 left to right, the two sums added).  Tiled layout: nvfp4_layout.hpp.
__global__ __launch_bounds__(256) void weight_apply_quant_int4_kernel(
    const uint16_t* __restrict__ W, int64_t ldw, const double* __restrict__ Tinv, uint8_t* __restrict__ Wq,
    uint8_t* __restrict__ Ws, int N, int K, int C, int tiled) {
  __shared__ double ti[32][32];  // inv(T_b)[k][j]
  const int b = blockIdx.y;
  for (int i = threadIdx.x; i < 1024; i += 256) ti[i >> 5][i & 31] = Tinv[(int64_t)b * 1024 + i];
  __syncthreads();
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  double w[32];
  const uint16_t* wp = W + (int64_t)n * ldw + 32 * b;
#pragma unroll
  for (int k = 0; k < 32; k += 8) {
    const v4u raw = *reinterpret_cast<const v4u*>(wp + k);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      w[k + 2 * i] = (double)__uint_as_float(raw[i] << 16);
      w[k + 2 * i + 1] = (double)__uint_as_float(raw[i] & 0xFFFF0000u);
    }
  }
  double y[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    double acc = 0.0;
#pragma unroll
    for (int k = 0; k < 32; ++k) acc = fma(w[k], ti[k][j], acc);
    y[j] = acc;
  }
  uint32_t bits;
  double rcp;
  {
#pragma clang fp contract(off)
    double lo = y[0] * y[0], hi = y[16] * y[16];
#pragma unroll
    for (int j = 1; j < 16; ++j) {
      const double t0 = y[j] * y[j], t1 = y[16 + j] * y[16 + j];
      lo = lo + t0;
      hi = hi + t1;
    }
    const double ss = lo + hi;
    const double sigma = sqrt(ss * 0.03125);
    bits = f64_to_bf16_bits(0.33860793 * sigma);
    bits = bits < 0x80u ? 0u : bits;
    const double q = 1.0 / (double)__uint_as_float(bits << 16);
    rcp = bits == 0 ? 0.0 : q;
  }
  uint32_t words[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    uint32_t wd = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const double t = fmin(fmax(y[8 * g + i] * rcp, -8.0), 7.0);
      wd |= ((uint32_t)(int)rint(t) & 0xFu) << (4 * i);
    }
    words[g] = wd;
  }
  const v4u chunk = {words[0], words[1], words[2], words[3]};
  if (tiled) {
    const int KT = K >> 6;
    *reinterpret_cast<v4u*>(Wq + nv_tiled_chunk_offset(n, b >> 1, b & 1, KT)) = chunk;
    reinterpret_cast<uint16_t*>(Ws + nv_tiled_scale_offset(n, b >> 1, KT))[b & 1] = (uint16_t)bits;
  } else {
    *reinterpret_cast<v4u*>(Wq + (int64_t)n * (K / 2) + 16 * b) = chunk;
    reinterpret_cast<uint16_t*>(Ws)[(int64_t)n * C + b] = (uint16_t)bits;
  }
}

// Tiled -> canonical copy of packed codes and scales (inspection / tests).
__global__ __launch_bounds__(256) void unpack_tiled_kernel(const uint8_t* __restrict__ qt,
                                                           const uint8_t* __restrict__ st,
                                                           uint8_t* __restrict__ q, uint8_t* __restrict__ s,
                                                           int64_t rows, int C) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;   // one (row, group) per thread
  if (idx >= rows * C) return;
  const int row = (int)(idx / C), g = (int)(idx % C);
  *reinterpret_cast<v4u*>(q + (int64_t)row * C * 16 + 16 * g) =
      *reinterpret_cast<const v4u*>(qt + tiled_chunk_offset(row, g, C >> 3));
  s[(int64_t)row * C + g] = st[tiled_scale_offset(row, g, C >> 3)];
}

// Quantizer-only tap: one thread per group of 32 FP32 values.
__global__ __launch_bounds__(256) void quantize_f32_kernel(const float* __restrict__ Y,
                                                           uint8_t* __restrict__ q,
                                                           uint8_t* __restrict__ s,
                                                           int64_t groups, int C, int rule, int tiled) {
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= groups) return;
  float v[32];
  const v4f* src = reinterpret_cast<const v4f*>(Y + g * 32);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const v4f t = src[i];
    v[4 * i] = t[0]; v[4 * i + 1] = t[1]; v[4 * i + 2] = t[2]; v[4 * i + 3] = t[3];
  }
  float amax = 0.f;
#pragma unroll
  for (int i = 0; i < 32; ++i) amax = fmaxf(amax, fabsf(v[i]));
  const int byte = scale_byte_f32(amax, rule);
  const float sc = scale_as_f32(byte);
  v4u out;
#pragma unroll
  for (int i = 0; i < 4; ++i) out[i] = pack8_e2m1(v + 8 * i, sc);
  if (tiled) {
    const int row = (int)(g / C), grp = (int)(g % C);
    *reinterpret_cast<v4u*>(q + tiled_chunk_offset(row, grp, C >> 3)) = out;
    s[tiled_scale_offset(row, grp, C >> 3)] = (uint8_t)byte;
  } else {
    *reinterpret_cast<v4u*>(q + g * 16) = out;
    s[g] = (uint8_t)byte;
  }
}

}  // namespace

size_t weight_prep_status_offset(int64_t K) { return (size_t)(K / 32) * 1024 * sizeof(double); }

size_t weight_prep_workspace_bytes(int64_t /*N*/, int64_t K) { return weight_prep_status_offset(K) + 16; }

hipError_t launch_weight_prep(const void* W, int64_t N, int64_t K, int64_t ldw, const void* T, int rule,
                              int tiled, void* Wq, void* Ws, void* workspace, hipStream_t stream) {
  const int C = (int)(K / 32);
  double* tinv = reinterpret_cast<double*>(workspace);
  int* status = reinterpret_cast<int*>(reinterpret_cast<char*>(workspace) + weight_prep_status_offset(K));
  // cleared by a kernel, not a memset node, so the sequence stays capturable
  reset_status_kernel<<<dim3(1), dim3(64), 0, stream>>>(status);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  invert_blocks_kernel<<<dim3(C), dim3(64), 0, stream>>>((const uint16_t*)T, tinv, status);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 grid((unsigned)((N + 255) / 256), (unsigned)C);
  weight_apply_quant_kernel<<<grid, dim3(256), 0, stream>>>((const uint16_t*)W, ldw, tinv, (uint8_t*)Wq,
                                                           (uint8_t*)Ws, (int)N, (int)K, C, rule, tiled);
  return hipGetLastError();
}

hipError_t launch_int4_weight_prep(const void* W, int64_t N, int64_t K, int64_t ldw, const void* T, int tiled, void* Wq,
                                   void* Ws, void* workspace, hipStream_t stream) {
  const int C = (int)(K / 32);
  double* tinv = reinterpret_cast<double*>(workspace);
  int* status = reinterpret_cast<int*>(reinterpret_cast<char*>(workspace) + weight_prep_status_offset(K));
  reset_status_kernel<<<dim3(1), dim3(64), 0, stream>>>(status);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  invert_blocks_kernel<<<dim3(C), dim3(64), 0, stream>>>((const uint16_t*)T, tinv, status);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 grid((unsigned)((N + 255) / 256), (unsigned)C);
  weight_apply_quant_int4_kernel<<<grid, dim3(256), 0, stream>>>((const uint16_t*)W, ldw, tinv, (uint8_t*)Wq,
                                                                (uint8_t*)Ws, (int)N, (int)K, C, tiled);
  return hipGetLastError();
}

hipError_t launch_quantize_f32(const float* Y, int64_t M, int64_t K, int rule, int tiled, void* q, void* s,
                               hipStream_t stream) {
  const int64_t groups = M * (K / 32);
  quantize_f32_kernel<<<dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, stream>>>(
      Y, (uint8_t*)q, (uint8_t*)s, groups, (int)(K / 32), rule, tiled);
  return hipGetLastError();
}

hipError_t launch_unpack_tiled(const void* qt, const void* st, int64_t rows, int64_t K, void* q, void* s,
                               hipStream_t stream) {
  const int64_t n = rows * (K / 32);
  unpack_tiled_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(
      (const uint8_t*)qt, (const uint8_t*)st, (uint8_t*)q, (uint8_t*)s, rows, (int)(K / 32));
  return hipGetLastError();
}

}  // namespace wush
