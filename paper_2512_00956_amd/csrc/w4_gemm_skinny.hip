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
  const int nrb = (M + 31) >> 5;   // row blocks the X buffers hold (a multiple of 32 rows): a block past them re-reads the last, never stored
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
        for (int rb = 0; rb < RB; ++rb) load_step(ch.x[rb][u], Xq, Xs, (int64_t)min(rb, nrb - 1) * KT + k, r, h);
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

// Second schedule, for 65..128 tokens on layers with many output channels.  Above, every wave converts the
// X fragments it multiplies, RB row blocks per K step and workgroup of 32 output channels: with four row blocks the
// activations, read from the L2 and converted once per workgroup, outweigh the weight stream (four times its bytes
// and conversions).  Here the four waves of a workgroup take four different groups of CBW output-channel blocks
// and all walk the WHOLE K range in step, so that they multiply the same X fragments: each wave converts a quarter
// of them (two (row block, K step) pairs of a chunk of eight) to FP16 and leaves them in LDS in MFMA operand order
// (lane-linear 16-byte accesses, conflict free); a chunk is double buffered, one barrier per chunk; the barrier's
// fences name LDS only, so the weight loads of the chunks ahead stay in flight across it.  Per 32 x 64 block of
// weights a wave now spends its 32 conversion operations, RB x 4 LDS reads and RB x 4 MFMAs; the raw X traffic and
// its conversion drop by four.  No partial sums across waves: a wave's accumulators are final and go straight to
// Y (one FP32 chain over K per element).
// It needs a workgroup per 4 CBW blocks of output channels, so few channels leave CUs idle, and every MFMA reads
// its X fragment from LDS (with CBW = 1): the launcher takes it where it was measured faster (launch()).  The
// kernel is written for any RB and CBW; only RB = 4, CBW = 1 is instantiated.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Accumulator e of lane (r, h), row block rb: token 32 rb + r, output channel 32 j + 8 (e / 4) + 4 h + e % 4.
template <int RB, bool OUT_F32>
__device__ __forceinline__ void store_block(const v16f (&acc)[RB], int j, int M, int N, void* __restrict__ Y,
                                            int64_t ldy, int vec_store, int r, int h, float scale) {
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int row = 32 * rb + r;
    if (row >= M) continue;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int col = 32 * j + 8 * q + 4 * h;
      if (col >= N) continue;
      float v[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) v[t] = acc[rb][4 * q + t] * scale;
      if (OUT_F32) {
        float* y = reinterpret_cast<float*>(Y) + (int64_t)row * ldy + col;
        if (vec_store) {
          *reinterpret_cast<v4f*>(y) = (v4f){v[0], v[1], v[2], v[3]};
        } else {
#pragma unroll
          for (int t = 0; t < 4; ++t)
            if (col + t < N) y[t] = v[t];
        }
      } else {
        uint16_t* y = reinterpret_cast<uint16_t*>(Y) + (int64_t)row * ldy + col;
        if (vec_store) {
          v2u two;
          two[0] = (uint32_t)f32_to_bf16_bits(v[0]) | ((uint32_t)f32_to_bf16_bits(v[1]) << 16);
          two[1] = (uint32_t)f32_to_bf16_bits(v[2]) | ((uint32_t)f32_to_bf16_bits(v[3]) << 16);
          *reinterpret_cast<v2u*>(y) = two;
        } else {
#pragma unroll
          for (int t = 0; t < 4; ++t)
            if (col + t < N) y[t] = f32_to_bf16_bits(v[t]);
        }
      }
    }
  }
}

// (row block, K step) pairs of X per chunk, 4 KiB of FP16 fragments each: four K steps up to 64 tokens, two beyond
template <int RB>
struct Chunk {
  static constexpr int kPairs = RB == 1 ? 4 : 8;
};
// chunks of weights in flight ahead of the multiply: what the registers next to the accumulators allow
template <int RB, int CBW>
struct Ahead { static constexpr int kChunks = RB == 1 ? 2 : (CBW == 2 ? 1 : (RB == 4 ? 3 : 2)); };
static_assert(Chunk<4>::kPairs % kWaves == 0, "every wave converts the same number of pairs");

template <int RB, int CBW, int FMT, bool OUT_F32>
__global__ __launch_bounds__(kWaves * 64, 2) void w4_shared_x_kernel(
    const uint8_t* __restrict__ Xq, const uint8_t* __restrict__ Xs, const float* __restrict__ tsx,
    const uint8_t* __restrict__ Wq, const uint8_t* __restrict__ Ws, const float* __restrict__ tsw,
    int M, int N, int K, void* __restrict__ Y, int64_t ldy, int vec_store) {
  constexpr int kPairs = Chunk<RB>::kPairs;
  constexpr int U = kPairs / RB;            // K steps per chunk
  constexpr int kMine = kPairs / kWaves;    // pairs a wave converts per chunk
  __shared__ v4u xf[2][kPairs][4][64];      // [buffer][pair = step RB + row block][MFMA of the step][lane]: 32 or 64 KiB
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 31, h = lane >> 5;
  const int KT = K >> 6, NB = (N + 31) >> 5;
  const int nrb = (M + 31) >> 5;   // row blocks the X buffers hold: a block past them re-reads the last, never stored
  const int groups = (NB + kWaves * CBW - 1) / (kWaves * CBW);
  const int nch = (KT + U - 1) / U;
  const uint32_t sel = 0x05040C0Cu + 0x02020000u * h;
  const float scale = FMT == kNvfp4 ? *tsx * *tsw : 1.0f;

  for (int g = blockIdx.x; g < groups; g += gridDim.x) {
    int64_t jb[CBW];   // this wave's weight blocks; one past the end repeats the last (never stored)
#pragma unroll
    for (int c = 0; c < CBW; ++c) jb[c] = min((g * kWaves + wave) * CBW + c, NB - 1);
    v16f acc[CBW][RB];
#pragma unroll
    for (int c = 0; c < CBW; ++c)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) acc[c][rb] = (v16f){0};

    // All loads are unconditional (a step past the end re-reads the last one): exact wait counts.
    RawStep xr[kMine];
    auto load_x = [&](int ch) {
#pragma unroll
      for (int m = 0; m < kMine; ++m) {
        const int p = wave + kWaves * m, u = p / RB, rb = p % RB;
        load_step(xr[m], Xq, Xs, (int64_t)min(rb, nrb - 1) * KT + min(ch * U + u, KT - 1), r, h);
      }
    };
    auto convert_x = [&](int buf) {
#pragma unroll
      for (int m = 0; m < kMine; ++m) {
        v8h f[4];
        dequant_step<FMT>(xr[m], h, sel, f);
#pragma unroll
        for (int d = 0; d < 4; ++d) xf[buf][wave + kWaves * m][d][lane] = __builtin_bit_cast(v4u, f[d]);
      }
    };
    auto load_w = [&](RawStep (&w)[CBW][U], int ch) {
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int c = 0; c < CBW; ++c) load_step(w[c][u], Wq, Ws, jb[c] * KT + min(ch * U + u, KT - 1), r, h);
    };
    auto multiply = [&](const RawStep (&w)[CBW][U], int ch, int buf) {
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ch * U + u < KT) {
          v2h sc[CBW];
#pragma unroll
          for (int c = 0; c < CBW; ++c) sc[c] = w_step_scales<FMT>(w[c][u].s, h, sel);
          // one MFMA of the step (8 of the lane's 32 codes per operand) at a time: few registers in flight
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            v8h fw[CBW];
#pragma unroll
            for (int c = 0; c < CBW; ++c) {
              const v2h s2 = {sc[c][d >> 1], sc[c][d >> 1]};
              fw[c] = __builtin_bit_cast(v8h, FMT == kNvfp4 ? dequant8(w[c][u].q[d], s2) : dequant8_int4(w[c][u].q[d], s2));
            }
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
              const v8h fx = __builtin_bit_cast(v8h, xf[buf][u * RB + rb][d][lane]);
#pragma unroll
              for (int c = 0; c < CBW; ++c)
                acc[c][rb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw[c], fx, acc[c][rb], 0, 0, 0);
            }
          }
        }
    };
    // The weights of D chunks are in flight ahead of the one being multiplied (D + 1 register sets that take
    // turns by unrolling); the X fragments of the next chunk are converted while this one is multiplied.
    constexpr int D = Ahead<RB, CBW>::kChunks, NBUF = D + 1;
    RawStep w[NBUF][CBW][U];
#pragma unroll
    for (int s = 0; s < D; ++s) load_w(w[s], s);
    load_x(0);
    convert_x(0);
    load_x(1);
    lds_barrier();
    for (int base = 0; base < nch; base += NBUF) {
#pragma unroll
      for (int s = 0; s < NBUF; ++s) {
        const int ch = base + s;           // past the last chunk: loads repeat the last step, nothing is multiplied,
        load_w(w[(s + D) % NBUF], ch + D); // and every wave still meets the barrier
        convert_x((ch + 1) & 1);
        load_x(ch + 2);
        multiply(w[s], ch, ch & 1);
        lds_barrier();
      }
    }
#pragma unroll
    for (int c = 0; c < CBW; ++c) {
      const int j = (g * kWaves + wave) * CBW + c;
      if (j < NB) store_block<RB, OUT_F32>(acc[c], j, M, N, Y, ldy, vec_store, r, h, scale);
    }
  }
}

template <int FMT>
hipError_t launch_split_k(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws,
                          const float* tsw, int64_t M, int64_t N, int64_t K, int out_f32, void* Y, int64_t ldy,
                          hipStream_t stream) {
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

// The shared-X schedule is built for 65..128 tokens with one weight block per wave: the only shape in which it
// beats the K split (measured, us, K split | shared X, 8192 -> 57344 at 96 and 128 tokens: NVFP4 140 | 134 and
// 147 | 127, INT4 206 | 150 and 205 | 150; 8192 -> 28672: NVFP4 71 | 85 and 72 | 86, INT4 114 | 92 and 120 | 97;
// 4096 -> 24576: 32 | 46 and 51 | 50).  With fewer tokens the K split's conversions are already cheap, with two
// weight blocks per wave too few workgroups are left, and with fewer output channels the whole-K walk of a wave
// leaves CUs idle.
template <int FMT>
hipError_t launch_shared_x(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws,
                           const float* tsw, int64_t M, int64_t N, int64_t K, int out_f32, void* Y, int64_t ldy,
                           hipStream_t stream) {
  const int NB = (int)((N + 31) / 32);
  const int groups = (NB + kWaves - 1) / kWaves;
  dim3 grid((unsigned)(groups < 4096 ? groups : 4096)), block(kWaves * 64);
  const int vec = skinny::decode_vec_store(Y, N, ldy, out_f32);
  if (out_f32)
    w4_shared_x_kernel<4, 1, FMT, true><<<grid, block, 0, stream>>>((const uint8_t*)Xq, (const uint8_t*)Xs, tsx,
                                                                    (const uint8_t*)Wq, (const uint8_t*)Ws, tsw,
                                                                    (int)M, (int)N, (int)K, Y, ldy, vec);
  else
    w4_shared_x_kernel<4, 1, FMT, false><<<grid, block, 0, stream>>>((const uint8_t*)Xq, (const uint8_t*)Xs, tsx,
                                                                     (const uint8_t*)Wq, (const uint8_t*)Ws, tsw,
                                                                     (int)M, (int)N, (int)K, Y, ldy, vec);
  return hipGetLastError();
}

// Which schedule: shared X for 65..128 tokens once the layer has enough output channels for it (fitted on the
// cases above: from 3.5 workgroups of four blocks per CU for INT4, whose conversions cost more, from 7 for
// NVFP4); the switch kDbgW4Skinny forces one (1 = K split across the waves, 2 = shared X where it exists).
template <int FMT>
hipError_t launch(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws, const float* tsw,
                  int64_t M, int64_t N, int64_t K, int out_f32, void* Y, int64_t ldy, hipStream_t stream) {
  const int forced = debug_option(kDbgW4Skinny);
  const int64_t NB = (N + 31) / 32;
  const bool wide = 2 * NB >= (FMT == kInt4 ? 7 : 14) * (int64_t)device_cu_count();
  const bool shared_x = M > 64 && (forced == 2 || (forced != 1 && wide));
  if (shared_x) return launch_shared_x<FMT>(Xq, Xs, tsx, Wq, Ws, tsw, M, N, K, out_f32, Y, ldy, stream);
  return launch_split_k<FMT>(Xq, Xs, tsx, Wq, Ws, tsw, M, N, K, out_f32, Y, ldy, stream);
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
