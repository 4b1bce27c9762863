// INT4 variant of the activation quantizer (paper: "Layerwise Quantization Loss",
// Table 1 -- "4-bit integers with Gaussian MSE clipping and BF16 scales of group
// size 32"; the transform block stays 32):
//   codes q in -8 .. 7 (two's-complement nibbles), one BF16 scale per group,
//   scale = BF16(STEP * sigma), sigma = root mean square of the group,
//   STEP = the step that minimizes the mean squared error of the 16-level grid on a
//   unit Gaussian, q = clip(round-half-even(v / scale), -8, 7).
// Decision arithmetic in FP32, one IEEE operation per step and in a fixed order
// (no fused multiply-add): t_i = v_i v_i; the 16 channels a lane holds summed left to
// right; the two halves added; sigma = sqrt(ss / 32); rcp = 1 / scale; v rcp rounded.
// Dataflow: the MXFP4 kernel's (transform_quant_core.hpp); only the quantizer differs.
#include "nvfp4_layout.hpp"
#include "transform_quant_core.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

using tq::kNB;
using tq::kTileM;
using tq::XFrag;
constexpr int kWaves = 4;
constexpr float kStepF32 = 0.33860793f;

// BF16 scale bits of a group from its sum of squares, and the element multiplier.
__device__ __forceinline__ uint32_t int4_scale(float ss, float& rcp) {
  const float sigma = sqrtf(ss * 0.03125f);
  uint32_t bits = f32_to_bf16_bits(kStepF32 * sigma);
  bits = bits < 0x80u ? 0u : bits;                      // below BF16's normal range: an empty group
  const float q = 1.0f / __uint_as_float(bits << 16);  // IEEE division
  rcp = bits == 0 ? 0.0f : q;
  return bits;
}

// Eight values times rcp -> eight two's-complement nibbles (element i in nibble i).
// v rcp is clamped to [-8, 7] and rounded to an integer by adding 1.5 * 2^23 (round to
// nearest even); the low four mantissa bits of the sum are the nibble.
__device__ __forceinline__ uint32_t pack8_int4(const float* v, float rcp) {
#pragma clang fp contract(off)
  uint32_t b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float t0 = fminf(fmaxf(v[2 * i] * rcp, -8.0f), 7.0f);
    const float t1 = fminf(fmaxf(v[2 * i + 1] * rcp, -8.0f), 7.0f);
    const uint32_t u0 = __float_as_uint(t0 + 12582912.0f), u1 = __float_as_uint(t1 + 12582912.0f);
    b[i] = ((u1 << 4) | (u0 & 0xFu)) & 0xFFu;
  }
  return b[0] | b[1] << 8 | b[2] << 16 | b[3] << 24;
}

__device__ __forceinline__ float sum_squares16(const float* v) {
#pragma clang fp contract(off)
  float ss = v[0] * v[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) {
    const float t = v[r] * v[r];
    ss = ss + t;
  }
  return ss;
}

// Transform + INT4 quantizer of one 32-token tile.  Codes come out as in the MXFP4
// kernel (lanes 0..31: the 16 bytes of blocks 0 and 1 of their token, lanes 32..63:
// blocks 2 and 3); sc[bb] = BF16 scale bits of block bb (valid in every lane).
template <bool DBG>
__device__ __forceinline__ void transform_quantize_int4(const v8bf (&ta)[kNB][2], const XFrag (&cur)[kNB],
                                                        v4u (&out)[2], uint32_t (&sc)[kNB], float* dbg_row, int nb) {
  uint32_t w[kNB][2];
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
    const uint32_t mine = __float_as_uint(sum_squares16(v));
    const auto sw = __builtin_amdgcn_permlane32_swap(mine, mine, false, false);
    const float ss = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);  // channels 0..15, then 16..31, in every lane
    float rcp;
    sc[bb] = int4_scale(ss, rcp);
    w[bb][0] = pack8_int4(v, rcp);
    w[bb][1] = pack8_int4(v + 8, rcp);
  }
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const auto s0 = __builtin_amdgcn_permlane32_swap(w[p][0], w[p + 2][0], false, false);
    const auto s1 = __builtin_amdgcn_permlane32_swap(w[p][1], w[p + 2][1], false, false);
    out[p] = (v4u){s0[0], s1[0], s0[1], s1[1]};
  }
}

// TG: groups of four waves per workgroup, each walking every TG-th of its tiles (transform_quant.hip).
// PF: tiles in flight ahead of the computed one: 1 with one wave group (three waves per SIMD), 2 with two (the
// workgroup is then its CU's only one: two waves per SIMD).
template <bool DBG, bool TILED, int TG, int PF>
__global__ __launch_bounds__(kWaves * TG * 64, (TG == 2 || DBG) ? 2 : 3) void int4_transform_quant_kernel(
    const uint16_t* __restrict__ X, int64_t ldx, const uint16_t* __restrict__ T, uint8_t* __restrict__ Xq,
    uint8_t* __restrict__ Xs, float* __restrict__ dbg, int M, int K, int C, int tiles_per_wg) {
  const int lane = threadIdx.x & 63;
  const int wave = (threadIdx.x >> 6) % kWaves;
  const int tg = (threadIdx.x >> 6) / kWaves;
  const int tok = lane & 31;
  const int h = lane >> 5;
  const int bfirst = (blockIdx.y * kWaves + wave) * kNB;
  if (bfirst >= C) return;  // wave-uniform
  const int nb = min(kNB, C - bfirst);

  v8bf ta[kNB][2];
  tq::load_transforms(ta, T, bfirst, C, tok, h);

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
    tq::load_tile(x[s], X, ldx, tile_row(tg + s * TG), bfirst, C, h);
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
      tq::load_tile(x[(s + PF) % (PF + 1)], X, ldx, tile_row(j + PF * TG), bfirst, C, h);

      v4u out[2];
      uint32_t sc[kNB];
      float* dbg_row = (DBG && row_ok) ? dbg + (int64_t)m * K + 32 * bfirst + 16 * h : nullptr;
      transform_quantize_int4<DBG>(ta, cur, out, sc, dbg_row, nb);
      if (row_ok && TILED) {
        // K % 64 == 0: this lane's blocks 2h, 2h+1 are the two groups of K step bfirst/2 + h
        const int KT = K >> 6, kt = (bfirst >> 1) + h;
        if (2 * h < nb) {
          __builtin_nontemporal_store(out[0], reinterpret_cast<v4u*>(Xq + nv_tiled_chunk_offset(m, kt, 0, KT)));
          __builtin_nontemporal_store(out[1], reinterpret_cast<v4u*>(Xq + nv_tiled_chunk_offset(m, kt, 1, KT)));
          const uint32_t pair = h ? (sc[2] | sc[3] << 16) : (sc[0] | sc[1] << 16);
          __builtin_nontemporal_store(pair, reinterpret_cast<uint32_t*>(Xs + nv_tiled_scale_offset(m, kt, KT)));
        }
      } else if (row_ok) {
        uint8_t* q = Xq + (int64_t)m * (K / 2) + 16 * bfirst + 32 * h;
        uint16_t* sp = reinterpret_cast<uint16_t*>(Xs) + (int64_t)m * C + bfirst;
        if (nb == kNB && (C & 3) == 0) {
          __builtin_nontemporal_store(out[0], reinterpret_cast<v4u*>(q));
          __builtin_nontemporal_store(out[1], reinterpret_cast<v4u*>(q + 16));
          if (h == 0)
            __builtin_nontemporal_store((v2u){sc[0] | sc[1] << 16, sc[2] | sc[3] << 16}, reinterpret_cast<v2u*>(sp));
        } else {
#pragma unroll
          for (int p = 0; p < 2; ++p)
            if (2 * h + p < nb) *reinterpret_cast<v4u*>(q + 16 * p) = out[p];
          if (h == 0) {
#pragma unroll
            for (int bb = 0; bb < kNB; ++bb)
              if (bb < nb) sp[bb] = (uint16_t)sc[bb];
          }
        }
      }
    }
  }
}

// Quantizer-only tap: one thread per group of 32 FP32 values (the two half sums as in the kernel).
__global__ __launch_bounds__(256) void int4_quantize_f32_kernel(const float* __restrict__ Y, uint8_t* __restrict__ q,
                                                                uint8_t* __restrict__ s, int64_t groups, int C,
                                                                int tiled) {
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= groups) return;
  float v[32];
  const v4f* src = reinterpret_cast<const v4f*>(Y + g * 32);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const v4f t = src[i];
    v[4 * i] = t[0]; v[4 * i + 1] = t[1]; v[4 * i + 2] = t[2]; v[4 * i + 3] = t[3];
  }
  const float ss = sum_squares16(v) + sum_squares16(v + 16);
  float rcp;
  const uint32_t bits = int4_scale(ss, rcp);
  const v4u out = {pack8_int4(v, rcp), pack8_int4(v + 8, rcp), pack8_int4(v + 16, rcp), pack8_int4(v + 24, rcp)};
  if (tiled) {
    const int64_t row = g / C;
    const int b = (int)(g % C), KT = C >> 1;
    *reinterpret_cast<v4u*>(q + nv_tiled_chunk_offset(row, b >> 1, b & 1, KT)) = out;
    reinterpret_cast<uint16_t*>(s + nv_tiled_scale_offset(row, b >> 1, KT))[b & 1] = (uint16_t)bits;
  } else {
    *reinterpret_cast<v4u*>(q + g * 16) = out;
    reinterpret_cast<uint16_t*>(s)[g] = (uint16_t)bits;
  }
}

}  // namespace

hipError_t launch_int4_transform_quant(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T, int tiled,
                                       void* Xq, void* Xs, float* dbg, hipStream_t stream) {
  const int C = (int)(K / 32);
  const int col_groups = (C + kWaves * kNB - 1) / (kWaves * kNB);
  const int ntiles = (int)((M + kTileM - 1) / kTileM);
  const Walk walk = token_walk_groups(ntiles, col_groups);
  const int tiles_per_wg = walk.tiles_per_wg;
  dim3 grid((ntiles + tiles_per_wg - 1) / tiles_per_wg, col_groups);
  dim3 block(kWaves * 64 * walk.groups);
#define WUSH_I4Q_LAUNCH(DBG, TILED, TG)                                                                       \
  int4_transform_quant_kernel<DBG, TILED, TG, TG><<<grid, block, 0, stream>>>(                                \
      (const uint16_t*)X, ldx, (const uint16_t*)T, (uint8_t*)Xq, (uint8_t*)Xs, dbg, (int)M, (int)K, C, tiles_per_wg)
  if (walk.groups == 2) {
    if (dbg) {
      if (tiled) WUSH_I4Q_LAUNCH(true, true, 2); else WUSH_I4Q_LAUNCH(true, false, 2);
    } else {
      if (tiled) WUSH_I4Q_LAUNCH(false, true, 2); else WUSH_I4Q_LAUNCH(false, false, 2);
    }
  } else if (dbg) {
    if (tiled) WUSH_I4Q_LAUNCH(true, true, 1); else WUSH_I4Q_LAUNCH(true, false, 1);
  } else {
    if (tiled) WUSH_I4Q_LAUNCH(false, true, 1); else WUSH_I4Q_LAUNCH(false, false, 1);
  }
#undef WUSH_I4Q_LAUNCH
  return hipGetLastError();
}

hipError_t launch_int4_quantize_f32(const float* Y, int64_t M, int64_t K, int tiled, void* q, void* s,
                                    hipStream_t stream) {
  const int64_t groups = M * (K / 32);
  int4_quantize_f32_kernel<<<dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, stream>>>(
      Y, (uint8_t*)q, (uint8_t*)s, groups, (int)(K / 32), tiled);
  return hipGetLastError();
}

}  // namespace wush
