// Weight-streaming GEMM of the NVFP4 and INT4 variants for at most 128 tokens (gfx950):
//   Y = tsx tsw * deq(Xq, Xs) . deq(Wq, Ws)^T
// (the sum over blocks of the layer forward-pass equation in the formats of the paper's
// experiments that have no block-scaled MFMA path: E2M1 x E4M3 per 16 x FP32 per tensor, and
// two's-complement codes x BF16 per 32).  At these sizes the layer is bound by reading the packed
// weights once (K/2 + K/16 bytes per output channel); the activations are a few hundred KiB that
// stay in the L2.
//
// Schedule: that of the MXFP4 kernel for few tokens.  A workgroup of four waves owns one block of 32
// output channels at a time; its waves split the K steps (64 channels each) into four contiguous
// ranges, so that a wave's weights are one contiguous run of the tiled layout, and the four partial
// tiles are summed through LDS in a fixed order.
// Arithmetic: that of the tiled kernels of these formats.  Element x group scale is exact in FP16, so
// both operands are dequantized in registers (hardware fp4 -> f16 convert or the magic-number INT4
// conversion, one packed multiply by the scale) and contracted on v_mfma_f32_32x32x16_f16 with FP32
// accumulators.  Which 16 channels an MFMA contracts is free as long as both operands agree: lane
// half h of a K step takes the step's 16-byte half h of its row (32 codes, ONE 128-bit load per lane
// and operand), and MFMA d = 0..3 of the step takes dword d of it.  The W fragment is the first
// operand, so a lane's accumulator quad is four consecutive output channels of one token.
// A wave loads its K steps in chunks of U and multiplies one chunk while the next is on its way; several
// workgroups share a CU.
// Every step costs a wave 32 vector operations per 32 x 64 block of codes it converts (W once, X once
// per 32 tokens) against 1152 bytes of weights: up to 64 tokens the conversion keeps pace with HBM.
#include "nvfp4_layout.hpp"
#include "skinny_reduce.hpp"
#include "w4_dequant.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

using skinny::kWaves;

struct RawStep {   // what a lane holds of one (32-row block, K step): its row's 16-byte half and scale dword
  v4u q;
  uint32_t s;
};

// K steps per chunk of loads; a wave keeps two chunks in flight (one being multiplied, one on its way).
template <int RB>
struct Depth { static constexpr int U = RB == 1 ? 4 : 2; };

// Block `blk` (32 rows) of a tiled operand with KT K steps: codes at
// (((blk KT + kt) 2 + h) 32 + r) 16, scale dword at ((blk KT + kt) 32 + r) 4.
__device__ __forceinline__ void load_step(RawStep& t, const uint8_t* __restrict__ q, const uint8_t* __restrict__ s,
                                          int64_t blk_kt, int r, int h) {
  t.q = *reinterpret_cast<const v4u*>(q + ((blk_kt * 2 + h) * 32 + r) * 16);
  t.s = *reinterpret_cast<const uint32_t*>(s + (blk_kt * 32 + r) * 4);
}

// The lane's 32 codes of a step as four MFMA operands (8 FP16 each).
template <int FMT>
__device__ __forceinline__ void dequant_step(const RawStep& t, int h, uint32_t sel, v8h (&f)[4]) {
  const v2h sc = w_step_scales<FMT>(t.s, h, sel);   // NVFP4: [0] groups 0, 1 of the half, [1] groups 2, 3; INT4: one scale
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const v2h s2 = {sc[d >> 1], sc[d >> 1]};
    const v4u u = FMT == kNvfp4 ? dequant8(t.q[d], s2) : dequant8_int4(t.q[d], s2);
    f[d] = __builtin_bit_cast(v8h, u);
  }
}

// CBW = blocks of 32 output channels a workgroup takes at a time: the X fragments of a K step are
// converted once and multiplied with CBW weight blocks (the conversion of X is the same work in every
// workgroup; with one block per pass it costs as much as that of the weights).
template <int RB, int CBW, int FMT, bool OUT_F32>
__global__ __launch_bounds__(kWaves * 64) void w4_skinny_kernel(
    const uint8_t* __restrict__ Xq, const uint8_t* __restrict__ Xs, const float* __restrict__ tsx,
    const uint8_t* __restrict__ Wq, const uint8_t* __restrict__ Ws, const float* __restrict__ tsw,
    int M, int N, int K, void* __restrict__ Y, int64_t ldy, int vec_store) {
  __shared__ float red[kWaves][RB][16][64];
  constexpr int U = Depth<RB>::U;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 31, h = lane >> 5;
  const int KT = K >> 6, NB = (N + 31) >> 5;
  const int groups = (NB + CBW - 1) / CBW;
  const uint32_t sel = 0x05040C0Cu + 0x02020000u * h;
  const float scale = FMT == kNvfp4 ? *tsx * *tsw : 1.0f;   // INT4 has no tensor scales (null pointers)
  int kt0, kt1;
  skinny::wave_k_range(KT, wave, kt0, kt1);

  struct Chunk {
    RawStep w[CBW][U], x[RB][U];
  };
  for (int g = blockIdx.x; g < groups; g += gridDim.x) {
    int64_t jb[CBW];   // weight blocks of this pass; one past the end repeats the last (never stored)
#pragma unroll
    for (int c = 0; c < CBW; ++c) jb[c] = min(g * CBW + c, NB - 1);
    v16f acc[CBW][RB];
#pragma unroll
    for (int c = 0; c < CBW; ++c)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) acc[c][rb] = (v16f){0};

    // Every load is unconditional (a step past the wave's range re-reads its last step), so the compiler
    // counts the loads in flight exactly and a chunk is multiplied while the next one is on its way.
    auto load_chunk = [&](Chunk& ch, int kt) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int k = min(kt + u, kt1 - 1);
#pragma unroll
        for (int c = 0; c < CBW; ++c) load_step(ch.w[c][u], Wq, Ws, jb[c] * KT + k, r, h);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int k = min(kt + u, kt1 - 1);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) load_step(ch.x[rb][u], Xq, Xs, (int64_t)rb * KT + k, r, h);
      }
    };
    auto multiply_chunk = [&](const Chunk& ch, int kt) {
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (kt + u < kt1) {
          v8h fx[RB][4];
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) dequant_step<FMT>(ch.x[rb][u], h, sel, fx[rb]);
#pragma unroll
          for (int c = 0; c < CBW; ++c) {
            v8h fw[4];
            dequant_step<FMT>(ch.w[c][u], h, sel, fw);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
              for (int d = 0; d < 4; ++d)
                acc[c][rb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw[d], fx[rb][d], acc[c][rb], 0, 0, 0);
          }
        }
    };
    if (kt0 < kt1) {
      Chunk a, b;
      load_chunk(a, kt0);
      for (int kt = kt0; kt < kt1; kt += 2 * U) {
        load_chunk(b, kt + U);
        multiply_chunk(a, kt);
        load_chunk(a, kt + 2 * U);
        multiply_chunk(b, kt + U);
      }
    }
#pragma unroll
    for (int c = 0; c < CBW; ++c)
      if (g * CBW + c < NB)
        skinny::reduce_store_block<RB, OUT_F32, FMT == kNvfp4>(acc[c], red, g * CBW + c, M, N, Y, ldy, vec_store, lane,
                                                               wave, scale);
  }
}

template <int FMT>
hipError_t launch(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws, const float* tsw,
                  int64_t M, int64_t N, int64_t K, int out_f32, void* Y, int64_t ldy, hipStream_t stream) {
  const int NB = (int)((N + 31) / 32);
  // Two weight blocks per pass once that still leaves every CU two workgroups or more (up to 64 tokens:
  // beyond, the accumulators of two blocks leave room for a single wave per SIMD).
  const int cbw = (M <= 64 && NB >= 4 * device_cu_count()) ? 2 : 1;
  const int groups = (NB + cbw - 1) / cbw;
  dim3 grid((unsigned)(groups < 4096 ? groups : 4096)), block(kWaves * 64);
  const int vec = skinny::decode_vec_store(Y, N, ldy, out_f32);
#define WUSH_W4S_LAUNCH(RB, CBW, F32)                                                                          \
  w4_skinny_kernel<RB, CBW, FMT, F32><<<grid, block, 0, stream>>>((const uint8_t*)Xq, (const uint8_t*)Xs, tsx, \
                                                                  (const uint8_t*)Wq, (const uint8_t*)Ws, tsw, \
                                                                  (int)M, (int)N, (int)K, Y, ldy, vec)
#define WUSH_W4S_BY_OUT(RB, CBW) \
  { if (out_f32) WUSH_W4S_LAUNCH(RB, CBW, true); else WUSH_W4S_LAUNCH(RB, CBW, false); }
  if (M <= 32) {
    if (cbw == 2) WUSH_W4S_BY_OUT(1, 2) else WUSH_W4S_BY_OUT(1, 1)
  } else if (M <= 64) {
    if (cbw == 2) WUSH_W4S_BY_OUT(2, 2) else WUSH_W4S_BY_OUT(2, 1)
  } else {
    WUSH_W4S_BY_OUT(4, 1)
  }
#undef WUSH_W4S_BY_OUT
#undef WUSH_W4S_LAUNCH
  return hipGetLastError();
}

}  // namespace

hipError_t launch_nvfp4_gemm_skinny(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws,
                                    const float* tsw, int64_t M, int64_t N, int64_t K, int out_f32, void* Y,
                                    int64_t ldy, hipStream_t stream) {
  return launch<kNvfp4>(Xq, Xs, tsx, Wq, Ws, tsw, M, N, K, out_f32, Y, ldy, stream);
}

hipError_t launch_int4_gemm_skinny(const void* Xq, const void* Xs, const void* Wq, const void* Ws, int64_t M, int64_t N,
                                   int64_t K, int out_f32, void* Y, int64_t ldy, hipStream_t stream) {
  return launch<kInt4>(Xq, Xs, nullptr, Wq, Ws, nullptr, M, N, K, out_f32, Y, ldy, stream);
}

}  // namespace wush
