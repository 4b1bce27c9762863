// MXFP4 x MXFP4 GEMM, FP32 accumulation, on CDNA4 block-scaled MFMA
// (v_mfma_scale_f32_32x32x64_f8f6f4 with both operands E2M1 and one E8M0 scale
// per 32 elements): Y = deq(Xq,Xs) . deq(Wq,Ws)^T, the sum over blocks of the
// layer forward-pass equation ("FP4-MatMul" in section "GPU Kernel Support").
//
// Operand mapping of the instruction (verified on hardware): for a 32x64
// operand tile, lane l holds row l%32 and the 32 consecutive K elements of
// half l/32 -- 16 bytes of the canonical packed layout -- plus the one scale
// byte of exactly that group.  Accumulator r of lane l is output row
// 8*(r/4) + 4*(l/32) + r%4, column l%32.
#include "wush_device.hpp"
#include <math.h>

#include "wush_kernels.hpp"

namespace wush {

namespace {

__device__ __forceinline__ void store_out(void* Y, int64_t ldy, int row, int col, float v, int out_f32) {
  if (out_f32) reinterpret_cast<float*>(Y)[(int64_t)row * ldy + col] = v;
  else reinterpret_cast<uint16_t*>(Y)[(int64_t)row * ldy + col] = f32_to_bf16_bits(v);
}

// Reference-grade kernel: one wavefront per 32x32 output tile, operands straight
// from global memory.  Handles every shape (ragged M, N, odd K/32).
__global__ __launch_bounds__(256) void gemm_simple_kernel(
    const uint8_t* __restrict__ Xq, const uint8_t* __restrict__ Xs,
    const uint8_t* __restrict__ Wq, const uint8_t* __restrict__ Ws,
    int M, int N, int K, int out_f32, void* __restrict__ Y, int64_t ldy) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int tiles_n = (N + 31) / 32;
  const int64_t tile = (int64_t)blockIdx.x * 4 + wave;
  const int tm = (int)(tile / tiles_n), tn = (int)(tile % tiles_n);
  if (tm * 32 >= M) return;  // wave-uniform
  const int r = lane & 31, kh = lane >> 5;
  const int C = K / 32;
  const int arow = min(tm * 32 + r, M - 1);
  const int brow = min(tn * 32 + r, N - 1);
  const uint8_t* ap = Xq + (int64_t)arow * (K / 2);
  const uint8_t* bp = Wq + (int64_t)brow * (K / 2);
  const uint8_t* as = Xs + (int64_t)arow * C;
  const uint8_t* bs = Ws + (int64_t)brow * C;
  v16f acc = {0};
  for (int g = 0; g < C; g += 2) {
    const int gg = g + kh;
    v4i a = {0, 0, 0, 0}, b = {0, 0, 0, 0};
    int sa = 127, sb = 127;
    if (gg < C) {
      a = *reinterpret_cast<const v4i*>(ap + 16 * gg);
      b = *reinterpret_cast<const v4i*>(bp + 16 * gg);
      sa = as[gg];
      sb = bs[gg];
    }
    const v8i A = {a[0], a[1], a[2], a[3], 0, 0, 0, 0};
    const v8i B = {b[0], b[1], b[2], b[3], 0, 0, 0, 0};
    acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, acc, 4, 4, 0, sa, 0, sb);
  }
  const int col = tn * 32 + r;
  if (col < N) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = tm * 32 + 8 * (i >> 2) + 4 * kh + (i & 3);
      if (row < M) store_out(Y, ldy, row, col, acc[i], out_f32);
    }
  }
}


// ---------------------------------------------------------------------------
// Tiled kernel: 256x256 output tile per workgroup, 4 wavefronts in a 2x2 grid,
// each owning a 128x128 sub-tile (4x4 MFMA tiles, 256 accumulator registers).
// K advances 256 elements (128 bytes per row) per iteration.
//
// Data path.  Both operand tiles go global -> LDS with global_load_lds_dwordx4
// (no VGPR staging; the destination of such a load is lane-linear, so one
// instruction fills 8 rows x 128 B).  The LDS tile is row-major with 128-byte
// rows; the 16-byte chunk at position p of row q holds source chunk
// p ^ ((q >> 1) & 7).  The swizzle is applied on the SOURCE side of the
// direct load (each lane picks which chunk of its row it fetches) and makes the
// fragment reads (32 consecutive rows, one chunk each, ds_read_b128) bank
// conflict free.  Two LDS stages (2 x 64 KiB), one barrier per iteration.
//
// K order inside a tile.  The MFMA contracts over 64 elements per issue; which
// 64 is free as long as both operands agree.  Issue kk (0..3) of lane half kh
// takes 32-element group 4*kh + kk of the 8 groups of the tile, so the four
// scale bytes a lane needs in one iteration are one aligned dword of the
// canonical scale row, consumed byte by byte through the op_sel field.  The
// scale dwords travel through LDS as well (global_load_lds_dword into a
// per-wave, lane-linear slot), so the main loop holds no VGPR-destination
// global load and the only vmcnt wait is the one in front of the barrier.
// ---------------------------------------------------------------------------
constexpr int kTM = 256, kTN = 256;
constexpr int kRowB = 128;                       // bytes of K per tile row (256 E2M1)
constexpr int kATileB = kTM * kRowB;             // 32 KiB
constexpr int kStageB = (kTM + kTN) * kRowB;     // 64 KiB
constexpr int kScaleStageB = 4 * 8 * 256;        // per stage: 4 waves x 8 sub-tiles x (64 lanes x 4 B)
constexpr int kScaleBase = 2 * kStageB;          // scale staging sits behind the two operand stages
constexpr int kGemmLds = 2 * kStageB + 2 * kScaleStageB;  // 144 KiB

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int KK>
__device__ __forceinline__ void mma_step(v16f (&acc)[4][4], const v4i (&af)[4], const v4i (&bf)[4],
                                         const int (&sa)[4], const int (&sb)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const v8i A = {af[i][0], af[i][1], af[i][2], af[i][3], 0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const v8i B = {bf[j][0], bf[j][1], bf[j][2], bf[j][3], 0, 0, 0, 0};
      acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, acc[i][j], 4, 4, KK, sa[i], KK, sb[j]);
    }
  }
}

template <bool OUT_F32>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(
    const uint8_t* __restrict__ Xq, const uint8_t* __restrict__ Xs,
    const uint8_t* __restrict__ Wq, const uint8_t* __restrict__ Ws,
    int M, int N, int K, void* __restrict__ Y, int64_t ldy, int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int r = lane & 31, kh = lane >> 5;

  // Workgroup -> tile.  Consecutive workgroup ids go round-robin over the 8
  // XCDs (each has its own L2), so every XCD is handed a contiguous range of
  // tile ids, and ids walk the grid in bands of 8 tile rows so that the tiles
  // an XCD runs concurrently share A and B panels.
  int id = blockIdx.x;
  const int total = tiles_m * tiles_n;
  id = xcd_contiguous_id(id, total);
  constexpr int kBand = 8;
  const int width = kBand * tiles_n;
  const int band = id / width;
  const int first_m = band * kBand;
  const int band_rows = min(tiles_m - first_m, kBand);
  const int tm = first_m + (id % width) % band_rows;
  const int tn = (id % width) / band_rows;
  const int m0 = tm * kTM, n0 = tn * kTN;

  const int C = K >> 5;
  const int64_t KB = K >> 1;
  const int KT = K >> 8;

  // ---- global -> LDS: this wave fills tile rows [64*wave, 64*wave + 64) of A and of B,
  // 8 rows per instruction.
  const int lrow = lane >> 3, lpos = lane & 7;
  const uint8_t* a_src[8];
  const uint8_t* b_src[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int q = 64 * wave + 8 * j + lrow;               // tile-local row
    const int chunk = lpos ^ ((q >> 1) & 7);
    a_src[j] = Xq + (int64_t)min(m0 + q, M - 1) * KB + 16 * chunk;
    b_src[j] = Wq + (int64_t)min(n0 + q, N - 1) * KB + 16 * chunk;
  }
  const int fill_off = (64 * wave) * kRowB;               // wave-uniform

  // ---- scale sources: one dword (groups 4kh..4kh+3 of the tile) per row sub-tile
  const uint8_t* sa_ptr[4];
  const uint8_t* sb_ptr[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    sa_ptr[s] = Xs + (int64_t)min(m0 + wm * 128 + s * 32 + r, M - 1) * C + 4 * kh;
    sb_ptr[s] = Ws + (int64_t)min(n0 + wn * 128 + s * 32 + r, N - 1) * C + 4 * kh;
  }
  const int scale_slot = kScaleBase + wave * (8 * 256);   // wave-uniform

  auto issue_tile = [&](int kt, int stage) {
    uint8_t* sa_ = smem + stage * kStageB + fill_off;
    uint8_t* sb_ = sa_ + kATileB;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      __builtin_amdgcn_global_load_lds((gptr_t)(a_src[j] + (int64_t)kt * kRowB), (lptr_t)(sa_ + j * 8 * kRowB), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((gptr_t)(b_src[j] + (int64_t)kt * kRowB), (lptr_t)(sb_ + j * 8 * kRowB), 16, 0, 0);
    }
    uint8_t* sc_ = smem + scale_slot + stage * kScaleStageB;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      __builtin_amdgcn_global_load_lds((gptr_t)(sa_ptr[s] + 8 * kt), (lptr_t)(sc_ + s * 256), 4, 0, 0);
      __builtin_amdgcn_global_load_lds((gptr_t)(sb_ptr[s] + 8 * kt), (lptr_t)(sc_ + (4 + s) * 256), 4, 0, 0);
    }
  };

  // ---- fragment read addresses
  const int swz = (r >> 1) & 7;
  int koff[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) koff[kk] = 16 * ((4 * kh + kk) ^ swz);
  const int a_rd = (wm * 128 + r) * kRowB;
  const int b_rd = kATileB + (wn * 128 + r) * kRowB;

  v16f acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = (v16f){0};

  issue_tile(0, 0);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int stage = kt & 1;
    if (kt + 1 < KT) issue_tile(kt + 1, stage ^ 1);
    const uint8_t* st = smem + stage * kStageB;
    const uint8_t* sc = smem + scale_slot + stage * kScaleStageB + 4 * lane;
    int sa[4], sb[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      sa[s] = *reinterpret_cast<const int*>(sc + s * 256);
      sb[s] = *reinterpret_cast<const int*>(sc + (4 + s) * 256);
    }
    v4i af[4], bf[4];
#define WUSH_LOAD_FRAGS(KK)                                                              \
    _Pragma("unroll") for (int s = 0; s < 4; ++s) {                                      \
      af[s] = *reinterpret_cast<const v4i*>(st + a_rd + s * 32 * kRowB + koff[KK]);      \
      bf[s] = *reinterpret_cast<const v4i*>(st + b_rd + s * 32 * kRowB + koff[KK]);      \
    }
    WUSH_LOAD_FRAGS(0) mma_step<0>(acc, af, bf, sa, sb);
    WUSH_LOAD_FRAGS(1) mma_step<1>(acc, af, bf, sa, sb);
    WUSH_LOAD_FRAGS(2) mma_step<2>(acc, af, bf, sa, sb);
    WUSH_LOAD_FRAGS(3) mma_step<3>(acc, af, bf, sa, sb);
#undef WUSH_LOAD_FRAGS
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's share of the next tile has landed
    __syncthreads();
  }

  // ---- epilogue: accumulator i of lane (r, kh) in MFMA tile (sm, sn) is output
  // row 32*sm + 8*(i/4) + 4*kh + i%4, column 32*sn + r of the wave's sub-tile.
#pragma unroll
  for (int sm = 0; sm < 4; ++sm) {
#pragma unroll
    for (int sn = 0; sn < 4; ++sn) {
      const int col = n0 + wn * 128 + sn * 32 + r;
      if (col < N) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int row = m0 + wm * 128 + sm * 32 + 8 * (i >> 2) + 4 * kh + (i & 3);
          if (row < M) {
            if (OUT_F32) reinterpret_cast<float*>(Y)[(int64_t)row * ldy + col] = acc[sm][sn][i];
            else reinterpret_cast<uint16_t*>(Y)[(int64_t)row * ldy + col] = f32_to_bf16_bits(acc[sm][sn][i]);
          }
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_mxfp4_gemm(const void* Xq, const void* Xs, const void* Wq, const void* Ws,
                             int64_t M, int64_t N, int64_t K, int out_f32, int tiled, void* Y, int64_t ldy,
                             hipStream_t stream) {
  if (tiled) {
    // Small batches: the streaming kernel (one workgroup per 32 output channels, the whole K) or
    // the tiled kernel with one row of 128-row tiles.  Up to 32 tokens the streaming kernel always
    // wins or ties.  Beyond, whichever the timing models below put first; they are fits to
    // measurements on ten layer shapes (4096 x 4096 .. 8192 x 57344 and 28672 x 8192), in us:
    //   streaming, 33..64 tokens : max(0.8 K/1024 + 2.5, MiB of weights / 5.5 + 3)
    //   streaming, 65..128 tokens: rounds of (N/32 workgroups over the CUs) x (1.05 K/1024 + 2.5)
    //   tiled                    : max(4.3 + 0.3 x K/256 x rounds of (N/128 tiles over the CUs),
    //                                  MiB of weights / 6.4 + 4)
    // (8192 x 57344, 64 tokens: 45.6 against 38.0; 128 tokens: 78.5 against 39.3;
    //  4096 x 24576, 128 tokens: 21.8 against 11.3; 28672 x 8192, 128 tokens: 31.1 against 41.4).
    bool skinny = M <= 32;
    if (!skinny && M <= 128) {
      const double cus = (double)device_cu_count();
      const double weight_mib = (double)N * (double)K * (17.0 / 32.0) / 1048576.0;
      const double kk = (double)K / 1024.0;
      const double skinny_us = M <= 64 ? fmax(0.8 * kk + 2.5, weight_mib / 5.5 + 3.0)
                                       : ceil((double)((N + 31) / 32) / cus) * (1.05 * kk + 2.5);
      const double tile_rounds = ceil((double)((N + 127) / 128) / cus);
      const double tiled_us = fmax(4.3 + 0.3 * (double)(K / 256) * tile_rounds, weight_mib / 6.4 + 4.0);
      skinny = skinny_us < tiled_us;
    }
    if (M <= 128 && debug_option(kDbgGemmSkinny) >= 0) skinny = debug_option(kDbgGemmSkinny) == 1;   // tests: force either kernel
    if (skinny) return launch_mxfp4_gemm_skinny(Xq, Xs, Wq, Ws, M, N, K, out_f32, Y, ldy, stream);
    return launch_mxfp4_gemm_frag(Xq, Xs, Wq, Ws, M, N, K, out_f32, Y, ldy, stream);
  }
  const bool force_simple = debug_option(kDbgGemmSimple) == 1;   // tests: the general kernel
  const bool tiled_ok = !force_simple && (K % 256 == 0) && (M * N >= 128 * 128);
  if (tiled_ok) {
    static DynamicLdsLimit lds_bf16, lds_f32;
    hipError_t attr = lds_bf16.ensure(reinterpret_cast<const void*>(gemm_tiled_kernel<false>), kGemmLds);
    if (attr == hipSuccess) attr = lds_f32.ensure(reinterpret_cast<const void*>(gemm_tiled_kernel<true>), kGemmLds);
    if (attr != hipSuccess) return attr;
    const int tiles_m = (int)((M + kTM - 1) / kTM), tiles_n = (int)((N + kTN - 1) / kTN);
    dim3 grid((unsigned)(tiles_m * tiles_n)), block(256);
    if (out_f32)
      gemm_tiled_kernel<true><<<grid, block, kGemmLds, stream>>>(
          (const uint8_t*)Xq, (const uint8_t*)Xs, (const uint8_t*)Wq, (const uint8_t*)Ws, (int)M, (int)N, (int)K,
          Y, ldy, tiles_m, tiles_n);
    else
      gemm_tiled_kernel<false><<<grid, block, kGemmLds, stream>>>(
          (const uint8_t*)Xq, (const uint8_t*)Xs, (const uint8_t*)Wq, (const uint8_t*)Ws, (int)M, (int)N, (int)K,
          Y, ldy, tiles_m, tiles_n);
    return hipGetLastError();
  }
  const int64_t tiles = ((M + 31) / 32) * ((N + 31) / 32);
  gemm_simple_kernel<<<dim3((unsigned)((tiles + 3) / 4)), dim3(256), 0, stream>>>(
      (const uint8_t*)Xq, (const uint8_t*)Xs, (const uint8_t*)Wq, (const uint8_t*)Ws,
      (int)M, (int)N, (int)K, out_f32, Y, ldy);
  return hipGetLastError();
}

}  // namespace wush
