// Wave-level pieces of the fused activation transform + MXFP4 quantizer
//   Xq, Xs = q(T_wush X)   (layer forward-pass equation; "Fused WUSH + Quant
//   kernel" in section "GPU Kernel Support"),
// shared by the stand-alone kernel and by the decode-sized fused layer kernel.
// One wave handles 32 tokens x 4 adjacent 32-channel blocks; see
// transform_quant.hip for the reasoning behind the operand orientation.
#pragma once
#include "wush_device.hpp"

namespace wush {
namespace tq {

constexpr int kNB = 4;       // blocks per wave
constexpr int kTileM = 32;   // tokens per MFMA tile

struct XFrag {
  v8bf lo, hi;  // channels 16h..16h+7 and 16h+8..16h+15 of one token, one block
};

// X-side operands of one tile: lane (tok, h) reads 16 consecutive BF16 of its
// token in each of the wave's blocks.  `row` is already clamped to a valid token.
__device__ __forceinline__ void load_tile(XFrag (&x)[kNB], const uint16_t* __restrict__ X,
                                          int64_t ldx, int row, int bfirst, int C, int h) {
#pragma unroll
  for (int bb = 0; bb < kNB; ++bb) {
    const int b = min(bfirst + bb, C - 1);  // clamped: out-of-range blocks reload a valid one
    const uint16_t* p = X + (int64_t)row * ldx + 32 * b + 16 * h;
    x[bb].lo = *reinterpret_cast<const v8bf*>(p);
    x[bb].hi = *reinterpret_cast<const v8bf*>(p + 8);
  }
}

// A operands (the wave's four T_b): MFMA row position i carries output channel
// c(i), chosen so that accumulator r of lane half h is channel 16h + r.
__device__ __forceinline__ void load_transforms(v8bf (&ta)[kNB][2], const uint16_t* __restrict__ T,
                                                int bfirst, int C, int tok, int h) {
  const int crow = 16 * ((tok >> 2) & 1) + 4 * (tok >> 3) + (tok & 3);
#pragma unroll
  for (int bb = 0; bb < kNB; ++bb) {
    const int b = min(bfirst + bb, C - 1);
    const uint16_t* p = T + ((int64_t)b * 32 + crow) * 32 + 16 * h;
    ta[bb][0] = *reinterpret_cast<const v8bf*>(p);
    ta[bb][1] = *reinterpret_cast<const v8bf*>(p + 8);
  }
}

// Transform, AbsMax, scale byte and E2M1 codes of one tile.  On return lanes
// 0..31 hold the 16 code bytes of blocks 0 and 1 of their token (out[0], out[1]),
// lanes 32..63 those of blocks 2 and 3; sbytes = the token's 4 scale bytes.
// dbg_row (DBG only): where this lane's 16 FP32 transformed values of block 0 go
// (null for rows past M); blocks >= nb are not written.
template <bool DBG>
__device__ __forceinline__ void transform_quantize(const v8bf (&ta)[kNB][2], const XFrag (&cur)[kNB], int rule,
                                                   v4u (&out)[2], uint32_t& sbytes, float* dbg_row, int nb) {
  uint32_t w[kNB][2];
  sbytes = 0;
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
    // other half of the group lives in lane ^ 32
    const uint32_t ab = __float_as_uint(amax);
    const auto sw = __builtin_amdgcn_permlane32_swap(ab, ab, false, false);
    amax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    const int byte = scale_byte_f32(amax, rule);
    const float sc = scale_as_f32(byte);
    w[bb][0] = pack8_e2m1(v, sc);
    w[bb][1] = pack8_e2m1(v + 8, sc);
    sbytes |= (uint32_t)byte << (8 * bb);
  }
  // Exchange halves: lanes 0..31 end up with the full 16 bytes of blocks 0
  // and 1 of their token, lanes 32..63 with blocks 2 and 3.
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const auto s0 = __builtin_amdgcn_permlane32_swap(w[p][0], w[p + 2][0], false, false);
    const auto s1 = __builtin_amdgcn_permlane32_swap(w[p][1], w[p + 2][1], false, false);
    out[p] = (v4u){s0[0], s1[0], s0[1], s1[1]};
  }
}

// Store one tile in the fragment-order layout (K % 256 == 0, so the wave's four
// blocks are whole and bfirst % 4 == 0).  Lanes 0..31 hold blocks bfirst,
// bfirst+1 of their token (kk = 0, 1), lanes 32..63 blocks bfirst+2, bfirst+3
// (kk = 2, 3); per instruction the 32 tokens of a half write 512 contiguous bytes.
// `t` = token tile = row block of the packed buffer.  STREAM: non-temporal stores
// (the output is not read again soon and must not displace X in the caches).
template <bool STREAM>
__device__ __forceinline__ void store_tile_tiled(const v4u (&out)[2], uint32_t sbytes, uint8_t* __restrict__ Xq,
                                                 uint8_t* __restrict__ Xs, int t, int KT, int bfirst, int tok, int h) {
  const int kt = bfirst >> 3, khg = (bfirst >> 2) & 1;
  const int64_t frag = ((int64_t)t * KT + kt) * 4;
  uint8_t* q = Xq + ((frag + 2 * h) * 64 + khg * 32 + tok) * 16;
  uint32_t* sp = reinterpret_cast<uint32_t*>(Xs + ((((int64_t)t * KT + kt) * 64) + khg * 32 + tok) * 4);
  if (STREAM) {
    __builtin_nontemporal_store(out[0], reinterpret_cast<v4u*>(q));
    __builtin_nontemporal_store(out[1], reinterpret_cast<v4u*>(q + 1024));
    if (h == 0) __builtin_nontemporal_store(sbytes, sp);
  } else {
    *reinterpret_cast<v4u*>(q) = out[0];
    *reinterpret_cast<v4u*>(q + 1024) = out[1];
    if (h == 0) *sp = sbytes;
  }
}

}  // namespace tq
}  // namespace wush
