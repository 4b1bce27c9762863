// NVFP4 variant of the two quantizers (paper: "Layerwise Quantization Loss" --
// NVFP4 uses group size 16 and the transform block size is matched to the group
// size; format: E2M1 elements, one E4M3 scale per 16 channels, one FP32 scale per
// tensor):
//   * fused activation transform (16 x 16 blocks) + quantizer, and the
//     quantizer-only test tap on FP32 values;
//   * offline weight side (Alg. 2, RTN case, with d = 16): FP64 inverse of every
//     16 x 16 block, W_blk . inv(T_b) in FP64, tensor scale from the AbsMax of the
//     transformed weights, quantization decided in FP64.
//
// Decision arithmetic (one IEEE operation per step, FP32 on the activation side,
// FP64 on the weight side):
//   c = 1 / (6 ts)   r = amax c   byte = E4M3(r)   d = value(byte) ts   rcp = 1 / d
//   code = E2M1(v rcp); byte 0 -> all magnitudes 0; the input's sign bit is kept;
//   ts = 0 (an all-zero tensor) -> c = 0, so every byte and magnitude is 0.
//
// Activation kernel: the MXFP4 kernel's dataflow (transform_quant_core.hpp) with
// two 16 x 16 blocks presented to the 32x32x16 BF16 MFMA as one block-diagonal
// 32 x 32 operand -- the zero half costs nothing (the kernel is bound by HBM
// traffic, and the accumulator layout then gives every lane exactly one group of 16).
#include "nvfp4_layout.hpp"
#include "transform_quant_core.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

using tq::kNB;
using tq::kTileM;
using tq::XFrag;
constexpr int kWaves = 4;

// ---------------------------------------------------------------------------
// E4M3 (finite-only FP8, bias 7): rounding and decoding
// ---------------------------------------------------------------------------
// r >= 0 rounded to the E4M3 grid (nearest, ties to even, saturating at 448), branch-free:
// adding and subtracting 2^(e-3+23), with e the exponent of r floored at -6 (below 2^-6 the
// grid is the multiples of 2^-9), leaves r rounded to 3 fraction bits.  Returns the value;
// `byte` gets its encoding (for a subnormal k * 2^-9 the fraction of k * 2^-9 + 2^-6 is k / 8).
__device__ __forceinline__ float round_e4m3_f32(float r, int& byte) {
  r = fminf(r, 448.0f);                                   // anything above rounds or saturates to 448
  const uint32_t eb = max(__float_as_uint(r) >> 23, 121u);
  const float magic = __uint_as_float((eb + 20u) << 23);
  const float t = (r + magic) - magic;
  const bool sub = t < 0.015625f;
  const float u = sub ? t + 0.015625f : t;
  byte = (int)(__float_as_uint(u) >> 20) - (sub ? (121 << 3) : (120 << 3));
  return t;
}

__device__ __forceinline__ double round_e4m3_f64(double r, int& byte) {
  r = fmin(r, 448.0);
  const uint64_t eb = max((uint64_t)__double_as_longlong(r) >> 52, (uint64_t)1017);
  const double magic = __longlong_as_double((long long)((eb + 49ull) << 52));
  const double t = (r + magic) - magic;
  const bool sub = t < 0.015625;
  const double u = sub ? t + 0.015625 : t;
  byte = (int)((uint64_t)__double_as_longlong(u) >> 49) - (sub ? (1017 << 3) : (1016 << 3));
  return t;
}

// Scale byte and element multiplier of one group (FP32 decision arithmetic).
__device__ __forceinline__ int group_scale_f32(float amax, float c, float ts, float& rcp) {
  int byte;
  const float d = round_e4m3_f32(amax * c, byte) * ts;
  const float q = 1.0f / d;             // IEEE division; d = 0 only with byte 0 (or ts = 0)
  rcp = byte == 0 ? 0.0f : q;
  return byte;
}

__device__ __forceinline__ uint32_t pack8_scaled(const float* v, float rcp) {
  float t[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) t[i] = v[i] * rcp;
  return pack8_e2m1(t, 1.0f);
}

// A operands: the two 16 x 16 blocks 2b, 2b+1 as one block-diagonal 32 x 32 T.
// Same row permutation as the MXFP4 kernel: accumulator r of lane half h is
// channel 16h + r of the pair, i.e. channel r of block 2b + h.
__device__ __forceinline__ void load_transforms16(v8bf (&ta)[kNB][2], const uint16_t* __restrict__ T16,
                                                  int bfirst, int C32, int tok, int h) {
  const int crow = 16 * ((tok >> 2) & 1) + 4 * (tok >> 3) + (tok & 3);
  const bool on = (crow >> 4) == h;  // this lane's 16 columns lie inside block 2b + h only for its rows
#pragma unroll
  for (int bb = 0; bb < kNB; ++bb) {
    const int b = min(bfirst + bb, C32 - 1);
    const uint16_t* p = T16 + ((int64_t)(2 * b + h) * 16 + (crow & 15)) * 16;
    const v8bf z = {0, 0, 0, 0, 0, 0, 0, 0};
    ta[bb][0] = on ? *reinterpret_cast<const v8bf*>(p) : z;
    ta[bb][1] = on ? *reinterpret_cast<const v8bf*>(p + 8) : z;
  }
}

// Transform + NVFP4 quantizer of one 32-token tile.  On return lanes 0..31 hold
// the 16 code bytes of 32-channel chunks 0 and 1 of their token, lanes 32..63
// those of chunks 2 and 3 (as in the MXFP4 kernel); scales = the token's 8
// scale bytes in channel order (valid in every lane).
template <bool DBG>
__device__ __forceinline__ void transform_quantize16(const v8bf (&ta)[kNB][2], const XFrag (&cur)[kNB], float c,
                                                     float ts, v4u (&out)[2], v2u& scales, float* dbg_row, int nb) {
  uint32_t w[kNB][2];
  uint32_t mine = 0;
#pragma unroll
  for (int bb = 0; bb < kNB; ++bb) {
    v16f acc = {0};
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ta[bb][0], cur[bb].lo, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ta[bb][1], cur[bb].hi, acc, 0, 0, 0);
    float v[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) v[r] = acc[r];
    if (DBG) {
      if (dbg_row && bb < nb) {
        float* d = dbg_row + 32 * bb;
#pragma unroll
        for (int r = 0; r < 16; r += 4)
          *reinterpret_cast<v4f*>(d + r) = (v4f){v[r], v[r + 1], v[r + 2], v[r + 3]};
      }
    }
    float amax = fabsf(v[0]);
#pragma unroll
    for (int r = 1; r < 16; ++r) amax = fmaxf(amax, fabsf(v[r]));
    float rcp;
    const int byte = group_scale_f32(amax, c, ts, rcp);
    w[bb][0] = pack8_scaled(v, rcp);
    w[bb][1] = pack8_scaled(v + 8, rcp);
    mine |= (uint32_t)byte << (8 * bb);
  }
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const auto s0 = __builtin_amdgcn_permlane32_swap(w[p][0], w[p + 2][0], false, false);
    const auto s1 = __builtin_amdgcn_permlane32_swap(w[p][1], w[p + 2][1], false, false);
    out[p] = (v4u){s0[0], s1[0], s0[1], s1[1]};
  }
  // scale bytes: this lane has group h of every chunk; interleave with the other half's
  const auto sw = __builtin_amdgcn_permlane32_swap(mine, mine, false, false);
  const uint32_t g0 = sw[0], g1 = sw[1];  // after the swap every lane sees (half 0's word, half 1's word)
  scales[0] = (g0 & 0xFFu) | (g1 & 0xFFu) << 8 | (g0 & 0xFF00u) << 8 | (g1 & 0xFF00u) << 16;
  scales[1] = (g0 >> 16 & 0xFFu) | (g1 >> 16 & 0xFFu) << 8 | (g0 >> 24) << 16 | (g1 >> 24) << 24;
}

// TG: groups of four waves per workgroup, each walking every TG-th of its tiles (transform_quant.hip).
// PF: tiles in flight ahead of the computed one: 1 with one wave group (three waves per SIMD), 2 with two (the
// workgroup is then its CU's only one: two waves per SIMD).
template <bool DBG, bool TILED, int TG, int PF>
__global__ __launch_bounds__(kWaves * TG * 64, (TG == 2 || DBG) ? 2 : 3) void nvfp4_transform_quant_kernel(
    const uint16_t* __restrict__ X, int64_t ldx, const uint16_t* __restrict__ T16, const float* __restrict__ tscale,
    uint8_t* __restrict__ Xq, uint8_t* __restrict__ Xs, float* __restrict__ dbg, int M, int K, int C32,
    int tiles_per_wg) {
  const int lane = threadIdx.x & 63;
  const int wave = (threadIdx.x >> 6) % kWaves;
  const int tg = (threadIdx.x >> 6) / kWaves;
  const int tok = lane & 31;
  const int h = lane >> 5;
  const int bfirst = (blockIdx.y * kWaves + wave) * kNB;
  if (bfirst >= C32) return;  // wave-uniform
  const int nb = min(kNB, C32 - bfirst);

  v8bf ta[kNB][2];
  load_transforms16(ta, T16, bfirst, C32, tok, h);
  const float ts = *tscale;
  const float c = ts == 0.0f ? 0.0f : 1.0f / (6.0f * ts);  // a zero tensor scale quantizes everything to zero

  // Walk step j of this workgroup is tile j gridDim.x + blockIdx.x, so that the grid as a whole moves
  // down the token rows front to back (transform_quant.hip: 10 % faster from HBM than a contiguous run of
  // tiles per workgroup).
  const int ntiles = (M + kTileM - 1) / kTileM;
  auto tile_of = [&](int j) { return j * (int)gridDim.x + (int)blockIdx.x; };
  auto valid = [&](int j) { return j < tiles_per_wg && tile_of(j) < ntiles; };
  if (!valid(tg)) return;

  // PF tiles in flight ahead of the one being computed, in PF + 1 register sets that take turns by unrolling
  // (no copies); every load is unconditional (a tile past the end of the walk becomes one row of the first tile, a
  // single resident cache line per instruction) and a finished wave leaves the kernel, so that the compiler's
  // wait counts are exact ones (transform_quant.hip).
  const int row_spare = min(tile_of(tg) * kTileM, M - 1);
  auto tile_row = [&](int j) { return valid(j) ? min(tile_of(j) * kTileM + tok, M - 1) : row_spare; };
  XFrag x[PF + 1][kNB];
#pragma unroll
  for (int s = 0; s < PF; ++s) {
    tq::load_tile(x[s], X, ldx, tile_row(tg + s * TG), bfirst, C32, h);
    __builtin_amdgcn_sched_barrier(0);
  }

  for (int base = tg; base < tiles_per_wg; base += (PF + 1) * TG) {
#pragma unroll
    for (int s = 0; s <= PF; ++s) {
      const int j = base + s * TG;
      if (!valid(j)) return;
      const XFrag (&cur)[kNB] = x[s];
      const int t = tile_of(j);
      const int m = t * kTileM + tok;
      const bool row_ok = m < M;
      tq::load_tile(x[(s + PF) % (PF + 1)], X, ldx, tile_row(j + PF * TG), bfirst, C32, h);

      v4u out[2];
      v2u scales;
      float* dbg_row = (DBG && row_ok) ? dbg + (int64_t)m * K + 32 * bfirst + 16 * h : nullptr;
      transform_quantize16<DBG>(ta, cur, c, ts, out, scales, dbg_row, nb);
      if (row_ok && TILED) {
        // K % 64 == 0: this lane's chunks 2h, 2h+1 are the two halves of K step bfirst/2 + h
        const int KT = K >> 6, kt = (bfirst >> 1) + h;
        if (2 * h < nb) {
          __builtin_nontemporal_store(out[0], reinterpret_cast<v4u*>(Xq + nv_tiled_chunk_offset(m, kt, 0, KT)));
          __builtin_nontemporal_store(out[1], reinterpret_cast<v4u*>(Xq + nv_tiled_chunk_offset(m, kt, 1, KT)));
          // every lane holds all 8 scale bytes of its token; each half writes its own step's four
          __builtin_nontemporal_store(scales[h], reinterpret_cast<uint32_t*>(Xs + nv_tiled_scale_offset(m, kt, KT)));
        }
      } else if (row_ok) {
        uint8_t* q = Xq + (int64_t)m * (K / 2) + 16 * bfirst + 32 * h;
        uint8_t* sp = Xs + (int64_t)m * (K / 16) + 2 * bfirst;
        if (nb == kNB && (C32 & 3) == 0) {
          __builtin_nontemporal_store(out[0], reinterpret_cast<v4u*>(q));
          __builtin_nontemporal_store(out[1], reinterpret_cast<v4u*>(q + 16));
          if (h == 0) __builtin_nontemporal_store(scales, reinterpret_cast<v2u*>(sp));
        } else {
          // ragged tail of the channel dimension: chunks 2h and 2h+1 of this lane
#pragma unroll
          for (int p = 0; p < 2; ++p)
            if (2 * h + p < nb) *reinterpret_cast<v4u*>(q + 16 * p) = out[p];
          if (h == 0)
            for (int g = 0; g < 2 * nb; ++g) sp[g] = (uint8_t)(scales[g >> 2] >> (8 * (g & 3)));
        }
      }
    }
  }
}

// Calibration of the activation tensor scale: AbsMax of T X over a batch (same transform, same
// FP32 accumulators as the quantizer), reduced with an atomic max on the bit pattern (non-negative
// floats order like their bits); a second tiny kernel turns it into AbsMax / (6 * 448).
__global__ __launch_bounds__(kWaves * 64, 3) void nvfp4_absmax_kernel(
    const uint16_t* __restrict__ X, int64_t ldx, const uint16_t* __restrict__ T16, unsigned int* __restrict__ amax_bits,
    int M, int C32, int tiles_per_wg) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int tok = lane & 31;
  const int h = lane >> 5;
  const int bfirst = (blockIdx.y * kWaves + wave) * kNB;
  if (bfirst >= C32) return;  // wave-uniform
  const int nb = min(kNB, C32 - bfirst);
  v8bf ta[kNB][2];
  load_transforms16(ta, T16, bfirst, C32, tok, h);
  const int ntiles = (M + kTileM - 1) / kTileM;
  const int tend = min((int)(blockIdx.x + 1) * tiles_per_wg, ntiles);
  float amax = 0.0f;
  for (int t = blockIdx.x * tiles_per_wg; t < tend; ++t) {
    XFrag cur[kNB];
    // rows past M re-read row M - 1 (its maximum is counted twice, which changes nothing)
    tq::load_tile(cur, X, ldx, min(t * kTileM + tok, M - 1), bfirst, C32, h);
#pragma unroll
    for (int bb = 0; bb < kNB; ++bb) {
      v16f acc = {0};
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ta[bb][0], cur[bb].lo, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ta[bb][1], cur[bb].hi, acc, 0, 0, 0);
      if (bb < nb) {  // blocks past the end were clamped to a valid one: harmless, but skip them
#pragma unroll
        for (int r = 0; r < 16; ++r) amax = fmaxf(amax, fabsf(acc[r]));
      }
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
  if (lane == 0) atomicMax(amax_bits, __float_as_uint(amax));
}

__global__ void nvfp4_reset_absmax_kernel(unsigned int* amax_bits) {
  if (threadIdx.x == 0) *amax_bits = 0u;
}

__global__ void nvfp4_finish_scale_kernel(float* ts) {
  if (threadIdx.x == 0) *ts = *ts / 2688.0f;  // the word holds the AbsMax (bit pattern of a float)
}

// Quantizer-only tap: one thread per group of 16 FP32 values.
__global__ __launch_bounds__(256) void nvfp4_quantize_f32_kernel(const float* __restrict__ Y,
                                                                 const float* __restrict__ tscale,
                                                                 uint8_t* __restrict__ q, uint8_t* __restrict__ s,
                                                                 int64_t groups, int C16, int tiled) {
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= groups) return;
  float v[16];
  const v4f* src = reinterpret_cast<const v4f*>(Y + g * 16);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const v4f t = src[i];
    v[4 * i] = t[0]; v[4 * i + 1] = t[1]; v[4 * i + 2] = t[2]; v[4 * i + 3] = t[3];
  }
  float amax = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(v[i]));
  const float ts = *tscale;
  const float c = ts == 0.0f ? 0.0f : 1.0f / (6.0f * ts);
  float rcp;
  const int byte = group_scale_f32(amax, c, ts, rcp);
  const v2u out = {pack8_scaled(v, rcp), pack8_scaled(v + 8, rcp)};
  if (tiled) {
    const int64_t row = g / C16;
    const int b = (int)(g % C16), kt = b >> 2, gi = b & 3;
    *reinterpret_cast<v2u*>(q + nv_tiled_chunk_offset(row, kt, gi >> 1, C16 >> 2) + 8 * (gi & 1)) = out;
    s[nv_tiled_scale_offset(row, kt, C16 >> 2) + gi] = (uint8_t)byte;
  } else {
    *reinterpret_cast<v2u*>(q + g * 8) = out;
    s[g] = (uint8_t)byte;
  }
}

// ---------------------------------------------------------------------------
// Weight side
// ---------------------------------------------------------------------------
constexpr double kPivotFloor = 1e-290;

// One wavefront per 16 x 16 block: FP64 Gauss-Jordan with partial pivoting on
// [T | I] (16 x 32) in LDS; lanes 0..31 each own one column.
__global__ __launch_bounds__(64) void invert16_kernel(const uint16_t* __restrict__ T16, double* __restrict__ Tinv,
                                                      int* __restrict__ status) {
  __shared__ double a[16][33];
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  const int col = lane & 31;
  for (int r = 0; r < 16; ++r) {
    double v;
    if (col < 16) v = (double)bf16_bits_to_f32(T16[((int64_t)b * 16 + r) * 16 + col]);
    else v = (col - 16 == r) ? 1.0 : 0.0;
    if (lane < 32) a[r][col] = v;
  }
  __syncthreads();
  bool singular = false;
  for (int p = 0; p < 16; ++p) {
    const int r = lane & 15;
    double mag = (r >= p) ? fabs(a[r][p]) : -1.0;
    int idx = r;
    for (int off = 8; off >= 1; off >>= 1) {
      const double omag = __shfl_xor(mag, off, 64);
      const int oidx = __shfl_xor(idx, off, 64);
      if (omag > mag || (omag == mag && oidx < idx)) { mag = omag; idx = oidx; }
    }
    if (!(mag > kPivotFloor)) { singular = true; break; }  // uniform across the wave
    if (idx != p && lane < 32) {
      const double t0 = a[p][col];
      a[p][col] = a[idx][col];
      a[idx][col] = t0;
    }
    __syncthreads();
    const double inv_piv = 1.0 / a[p][p];
    __syncthreads();
    const double prow = a[p][col] * inv_piv;
    if (lane < 32) a[p][col] = prow;
    __syncthreads();
    for (int rr = 0; rr < 16; ++rr) {
      if (rr == p) continue;
      const double f = a[rr][p];
      __syncthreads();
      if (lane < 32) a[rr][col] -= f * prow;
    }
    __syncthreads();
  }
  if (singular) {
    if (lane == 0) atomicExch(status, 1);
    for (int r = 0; r < 16; ++r)
      if (lane < 16) Tinv[((int64_t)b * 16 + r) * 16 + lane] = 0.0;
    return;
  }
  for (int r = 0; r < 16; ++r)
    if (lane >= 16 && lane < 32) Tinv[((int64_t)b * 16 + r) * 16 + (lane - 16)] = a[r][lane];
}

__global__ void reset_words_kernel(unsigned long long* amax_bits, int* status) {
  if (threadIdx.x == 0) { *amax_bits = 0ull; *status = 0; }
}

// y[j] = sum_k W[n, 16b+k] inv(T_b)[k][j] in FP64 (k ascending, fused multiply-add).
__device__ __forceinline__ void apply_block16(const uint16_t* __restrict__ wp, const double (*ti)[16], double (&y)[16]) {
  double w[16];
#pragma unroll
  for (int k = 0; k < 16; k += 8) {
    const v4u raw = *reinterpret_cast<const v4u*>(wp + k);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      w[k + 2 * i] = (double)__uint_as_float(raw[i] << 16);
      w[k + 2 * i + 1] = (double)__uint_as_float(raw[i] & 0xFFFF0000u);
    }
  }
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    double acc = 0.0;
#pragma unroll
    for (int k = 0; k < 16; ++k) acc = fma(w[k], ti[k][j], acc);
    y[j] = acc;
  }
}

// Pass 1 (QUANT = false): AbsMax of the transformed weights (positive doubles
// order like their bit patterns).  Pass 2 (QUANT = true): quantize with the
// tensor scale derived from it.  grid = (rows / 256, K / 16).
template <bool QUANT>
__global__ __launch_bounds__(256) void nvfp4_weight_kernel(const uint16_t* __restrict__ W, int64_t ldw,
                                                           const double* __restrict__ Tinv,
                                                           unsigned long long* __restrict__ amax_bits,
                                                           uint8_t* __restrict__ Wq, uint8_t* __restrict__ Ws,
                                                           float* __restrict__ ts_out, int N, int K, int tiled) {
  __shared__ double ti[16][16];
  __shared__ unsigned long long wg_max;
  const int b = blockIdx.y;
  if (threadIdx.x < 256) ti[threadIdx.x >> 4][threadIdx.x & 15] = Tinv[(int64_t)b * 256 + threadIdx.x];
  if (threadIdx.x == 0) wg_max = 0ull;
  __syncthreads();
  const int n = blockIdx.x * 256 + threadIdx.x;
  double y[16];
  double amax = 0.0;
  if (n < N) {
    apply_block16(W + (int64_t)n * ldw + 16 * b, ti, y);
#pragma unroll
    for (int j = 0; j < 16; ++j) amax = fmax(amax, fabs(y[j]));
  }
  if (!QUANT) {
    atomicMax(&wg_max, (unsigned long long)__double_as_longlong(amax));
    __syncthreads();
    if (threadIdx.x == 0) atomicMax(amax_bits, wg_max);
    return;
  }
  const float tsf = (float)(__longlong_as_double((long long)*amax_bits) / 2688.0);  // AbsMax / (6 * 448)
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *ts_out = tsf;
  if (n >= N) return;
  const double ts = (double)tsf;
  const double c = ts == 0.0 ? 0.0 : 1.0 / (6.0 * ts);
  int byte;
  const double d = round_e4m3_f64(amax * c, byte) * ts;
  const double rcp = byte == 0 ? 0.0 : 1.0 / d;
  uint32_t words[2];
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    uint32_t wd = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const double v = y[8 * g + i];
      const uint32_t sign = (uint32_t)(((uint64_t)__double_as_longlong(v)) >> 63);
      wd |= ((sign << 3) | e2m1_code_f64(fabs(v * rcp))) << (4 * i);
    }
    words[g] = wd;
  }
  if (tiled) {
    const int kt = b >> 2, gi = b & 3, KT = K >> 6;
    *reinterpret_cast<v2u*>(Wq + nv_tiled_chunk_offset(n, kt, gi >> 1, KT) + 8 * (gi & 1)) = (v2u){words[0], words[1]};
    Ws[nv_tiled_scale_offset(n, kt, KT) + gi] = (uint8_t)byte;
  } else {
    *reinterpret_cast<v2u*>(Wq + (int64_t)n * (K / 2) + 8 * b) = (v2u){words[0], words[1]};
    Ws[(int64_t)n * (K / 16) + b] = (uint8_t)byte;
  }
}

// Tiled -> canonical copy of packed codes and scales (inspection / tests): one thread per (row, K step).
__global__ __launch_bounds__(256) void nvfp4_unpack_tiled_kernel(const uint8_t* __restrict__ qt,
                                                                 const uint8_t* __restrict__ st,
                                                                 uint8_t* __restrict__ q, uint8_t* __restrict__ s,
                                                                 int64_t rows, int KT) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * KT) return;
  const int64_t row = idx / KT;
  const int kt = (int)(idx % KT);
  uint8_t* dst = q + row * KT * 32 + kt * 32;
  *reinterpret_cast<v4u*>(dst) = *reinterpret_cast<const v4u*>(qt + nv_tiled_chunk_offset(row, kt, 0, KT));
  *reinterpret_cast<v4u*>(dst + 16) = *reinterpret_cast<const v4u*>(qt + nv_tiled_chunk_offset(row, kt, 1, KT));
  *reinterpret_cast<uint32_t*>(s + row * KT * 4 + kt * 4) =
      *reinterpret_cast<const uint32_t*>(st + nv_tiled_scale_offset(row, kt, KT));
}

}  // namespace

hipError_t launch_nvfp4_transform_quant(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T16,
                                        const float* tscale, int tiled, void* Xq, void* Xs, float* dbg,
                                        hipStream_t stream) {
  const int C32 = (int)(K / 32);
  const int col_groups = (C32 + kWaves * kNB - 1) / (kWaves * kNB);
  const int ntiles = (int)((M + kTileM - 1) / kTileM);
  const Walk walk = token_walk_groups(ntiles, col_groups);
  const int tiles_per_wg = walk.tiles_per_wg;
  dim3 grid((ntiles + tiles_per_wg - 1) / tiles_per_wg, col_groups);
  dim3 block(kWaves * 64 * walk.groups);
#define WUSH_NVQ_LAUNCH(DBG, TILED, TG)                                                                          \
  nvfp4_transform_quant_kernel<DBG, TILED, TG, TG><<<grid, block, 0, stream>>>(                                  \
      (const uint16_t*)X, ldx, (const uint16_t*)T16, tscale, (uint8_t*)Xq, (uint8_t*)Xs, dbg, (int)M, (int)K, \
      C32, tiles_per_wg)
  if (walk.groups == 2) {
    if (dbg) {
      if (tiled) WUSH_NVQ_LAUNCH(true, true, 2); else WUSH_NVQ_LAUNCH(true, false, 2);
    } else {
      if (tiled) WUSH_NVQ_LAUNCH(false, true, 2); else WUSH_NVQ_LAUNCH(false, false, 2);
    }
  } else if (dbg) {
    if (tiled) WUSH_NVQ_LAUNCH(true, true, 1); else WUSH_NVQ_LAUNCH(true, false, 1);
  } else {
    if (tiled) WUSH_NVQ_LAUNCH(false, true, 1); else WUSH_NVQ_LAUNCH(false, false, 1);
  }
#undef WUSH_NVQ_LAUNCH
  return hipGetLastError();
}

// The output word doubles as the reduction target: zeroed, raised to the AbsMax, then scaled in place.
hipError_t launch_nvfp4_calibrate(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T16, float* ts_out,
                                  hipStream_t stream) {
  const int C32 = (int)(K / 32);
  const int col_groups = (C32 + kWaves * kNB - 1) / (kWaves * kNB);
  const int ntiles = (int)((M + kTileM - 1) / kTileM);
  const int tiles_per_wg = token_walk(ntiles, col_groups);
  unsigned int* word = reinterpret_cast<unsigned int*>(ts_out);
  nvfp4_reset_absmax_kernel<<<dim3(1), dim3(64), 0, stream>>>(word);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  nvfp4_absmax_kernel<<<dim3((ntiles + tiles_per_wg - 1) / tiles_per_wg, col_groups), dim3(kWaves * 64), 0, stream>>>(
      (const uint16_t*)X, ldx, (const uint16_t*)T16, word, (int)M, C32, tiles_per_wg);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  nvfp4_finish_scale_kernel<<<dim3(1), dim3(64), 0, stream>>>(ts_out);
  return hipGetLastError();
}

hipError_t launch_nvfp4_quantize_f32(const float* Y, int64_t M, int64_t K, const float* tscale, int tiled, void* q,
                                     void* s, hipStream_t stream) {
  const int64_t groups = M * (K / 16);
  nvfp4_quantize_f32_kernel<<<dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, stream>>>(
      Y, tscale, (uint8_t*)q, (uint8_t*)s, groups, (int)(K / 16), tiled);
  return hipGetLastError();
}

hipError_t launch_nvfp4_unpack_tiled(const void* qt, const void* st, int64_t rows, int64_t K, void* q, void* s,
                                     hipStream_t stream) {
  const int64_t n = rows * (K / 64);
  nvfp4_unpack_tiled_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(
      (const uint8_t*)qt, (const uint8_t*)st, (uint8_t*)q, (uint8_t*)s, rows, (int)(K / 64));
  return hipGetLastError();
}

// workspace: [K/16][16][16] FP64 inverses | u64 AbsMax bits | int32 status
size_t nvfp4_weight_prep_amax_offset(int64_t K) { return (size_t)(K / 16) * 256 * sizeof(double); }
size_t nvfp4_weight_prep_status_offset(int64_t K) { return nvfp4_weight_prep_amax_offset(K) + 8; }
size_t nvfp4_weight_prep_workspace_bytes(int64_t K) { return nvfp4_weight_prep_amax_offset(K) + 16; }

hipError_t launch_nvfp4_weight_prep(const void* W, int64_t N, int64_t K, int64_t ldw, const void* T16, int tiled,
                                    void* Wq, void* Ws, float* ts_out, void* workspace, hipStream_t stream) {
  double* tinv = reinterpret_cast<double*>(workspace);
  char* base = reinterpret_cast<char*>(workspace);
  unsigned long long* amax = reinterpret_cast<unsigned long long*>(base + nvfp4_weight_prep_amax_offset(K));
  int* status = reinterpret_cast<int*>(base + nvfp4_weight_prep_status_offset(K));
  reset_words_kernel<<<dim3(1), dim3(64), 0, stream>>>(amax, status);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  invert16_kernel<<<dim3((unsigned)(K / 16)), dim3(64), 0, stream>>>((const uint16_t*)T16, tinv, status);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 grid((unsigned)((N + 255) / 256), (unsigned)(K / 16));
  nvfp4_weight_kernel<false><<<grid, dim3(256), 0, stream>>>((const uint16_t*)W, ldw, tinv, amax, nullptr, nullptr,
                                                             nullptr, (int)N, (int)K, tiled);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  nvfp4_weight_kernel<true><<<grid, dim3(256), 0, stream>>>((const uint16_t*)W, ldw, tinv, amax, (uint8_t*)Wq,
                                                            (uint8_t*)Ws, ts_out, (int)N, (int)K, tiled);
  return hipGetLastError();
}

}  // namespace wush
