// MXFP4 GEMM on operands stored in the fragment-order ("tiled") layout of
// wush_device.hpp: Y = deq(Xq,Xs) . deq(Wq,Ws)^T (the layer forward-pass
// equation summed over all blocks), v_mfma_scale_f32_32x32x64_f8f6f4.
//
// Workgroup tile 256 (M) x 256 (N), K advances 256 elements per iteration.
// The four wavefronts split N: each owns all 256 rows and 64 columns
// (8 x 2 MFMA tiles, 256 accumulator registers).
//   * W fragments (the wave's own 64 columns) go global -> VGPR directly: in
//     the tiled layout a fragment is 1 KiB contiguous in lane order, so every
//     load is a perfectly coalesced 128-bit access and no wave loads what
//     another one loads.  They are fetched one K iteration ahead.
//   * X fragments (shared by all four waves) go global -> VGPR -> LDS, also one
//     iteration ahead, into a double-buffered 2 x 32 KiB stage; the LDS image
//     is the same lane-linear fragment order, so ds_write_b128 / ds_read_b128
//     are bank-conflict free without any swizzle.
//   * Scales: one dword per lane per (row block, K tile) straight from the
//     tiled scale array (256 contiguous bytes per load); its 4 bytes are the
//     4 MFMA issues of the iteration, selected with op_sel.
// (Measured on MI355X: direct-to-LDS global loads sustain only ~16 B/clk/CU,
//  far below what this loop needs, hence the register-staged path.)
#include <type_traits>

#include "wush_device.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

constexpr int kTM = 256, kTN = 256;
constexpr int kFragB = 1024;                 // one 32-row x 64-element fragment
constexpr int kAStageB = 8 * 4 * kFragB;     // 8 row blocks x 4 issues = 32 KiB
constexpr int kLds = 2 * kAStageB;

struct BFrags { v4i f[2][4]; };              // [column block][issue]
struct Scales { int a[8]; int b[2]; };

template <int KK>
__device__ __forceinline__ void mma_issue(v16f (&acc)[8][2], const v4i (&af)[8], const BFrags& bf,
                                          const Scales& sc) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const v8i A = {af[i][0], af[i][1], af[i][2], af[i][3], 0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const v8i B = {bf.f[j][KK][0], bf.f[j][KK][1], bf.f[j][KK][2], bf.f[j][KK][3], 0, 0, 0, 0};
      acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, acc[i][j], 4, 4, KK, sc.a[i], KK, sc.b[j]);
    }
  }
}

template <bool OUT_F32>
__global__ __launch_bounds__(256) void gemm_frag_kernel(
    const uint8_t* __restrict__ Xq, const uint8_t* __restrict__ Xs,
    const uint8_t* __restrict__ Wq, const uint8_t* __restrict__ Ws,
    int M, int N, int K, void* __restrict__ Y, int64_t ldy, int tiles_m, int tiles_n) {
  __shared__ __attribute__((aligned(1024))) uint8_t smem[kLds];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: keeps bases in SGPRs
  const int r = lane & 31, kh = lane >> 5;

  // Workgroup -> tile: every XCD (workgroup id mod 8) gets a contiguous range of
  // tile ids; ids walk the grid in bands of 8 tile rows so that the tiles an XCD
  // runs concurrently share X and W panels in its L2.
  int id = blockIdx.x;
  const int total = tiles_m * tiles_n;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
  constexpr int kBand = 8;
  const int width = kBand * tiles_n;
  const int band = id / width;
  const int first_m = band * kBand;
  const int band_rows = min(tiles_m - first_m, kBand);
  const int tm = first_m + (id % width) % band_rows;
  const int tn = (id % width) / band_rows;
  const int m0 = tm * kTM, n0 = tn * kTN;

  const int KT = K >> 8;
  const int64_t tile_step = 4 * kFragB;                 // bytes of one (row block, K tile)

  // Operand buffers are padded to whole 256-row tiles, so every address below
  // is "uniform base + lane offset"; rows past M or N are read but never stored.
  // X tile: this wave stages row blocks 2*wave, 2*wave+1 (4 fragments each).
  const uint8_t* xsrc = Xq + (int64_t)(tm * 8 + 2 * wave) * KT * tile_step;
  // W fragments and scales of this wave's two column blocks.
  const uint8_t* wsrc = Wq + (int64_t)(tn * 8 + 2 * wave) * KT * tile_step;
  const uint8_t* wsc = Ws + (int64_t)(tn * 8 + 2 * wave) * KT * 256;
  const uint8_t* xsc = Xs + (int64_t)(tm * 8) * KT * 256;
  const int loff = 16 * lane, soff = 4 * lane;

  auto load_x = [&](v4i (&stg)[8], int kt) {
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        stg[u * 4 + kk] = *reinterpret_cast<const v4i*>(xsrc + ((int64_t)u * KT + kt) * tile_step + kk * kFragB + loff);
  };
  auto store_x = [&](const v4i (&stg)[8], int stage) {
    uint8_t* dst = smem + stage * kAStageB + (2 * wave) * (4 * kFragB) + loff;
#pragma unroll
    for (int f = 0; f < 8; ++f) *reinterpret_cast<v4i*>(dst + f * kFragB) = stg[f];
  };
  auto load_w_frag = [&](BFrags& bf, int kt, int kk) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
      bf.f[j][kk] = *reinterpret_cast<const v4i*>(wsrc + ((int64_t)j * KT + kt) * tile_step + kk * kFragB + loff);
  };
  auto load_scales = [&](Scales& sc, int kt) {
#pragma unroll
    for (int j = 0; j < 2; ++j) sc.b[j] = *reinterpret_cast<const int*>(wsc + ((int64_t)j * KT + kt) * 256 + soff);
#pragma unroll
    for (int i = 0; i < 8; ++i) sc.a[i] = *reinterpret_cast<const int*>(xsc + ((int64_t)i * KT + kt) * 256 + soff);
  };

  v16f acc[8][2];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = (v16f){0};

  // ---- prologue
  v4i stg[8];
  BFrags bf;
  Scales sc0, sc1;
  load_x(stg, 0);
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) load_w_frag(bf, 0, kk);
  load_scales(sc0, 0);
  store_x(stg, 0);
  __syncthreads();

  // One K iteration: fetch tile kt+1 (X into staging registers, scales into the
  // other scale set, each W fragment into its own registers as soon as the
  // issue that used it is done), run the 64 MFMAs of tile kt, then park the
  // staged X tile in the other LDS stage.
  auto iteration = [&](int kt, const Scales& scur, Scales& snxt, auto more_tag) {
    constexpr bool more = decltype(more_tag)::value;
    if (more) {
      load_x(stg, kt + 1);
      load_scales(snxt, kt + 1);
    }
    const uint8_t* st = smem + (kt & 1) * kAStageB + loff;
    v4i af0[8], af1[8];
#define WUSH_READ_A(dst, KK)                                                      \
    _Pragma("unroll") for (int i = 0; i < 8; ++i)                                 \
      dst[i] = *reinterpret_cast<const v4i*>(st + (i * 4 + KK) * kFragB);
    // sched_barrier(0) pins the order below: without it the compiler hoists all
    // fragment reads and next-tile loads to the top of the iteration and spills.
#define WUSH_FENCE __builtin_amdgcn_sched_barrier(0);
    WUSH_FENCE
    WUSH_READ_A(af0, 0)
    WUSH_READ_A(af1, 1)
    WUSH_FENCE
    mma_issue<0>(acc, af0, bf, scur);
    WUSH_FENCE
    if (more) load_w_frag(bf, kt + 1, 0);
    WUSH_READ_A(af0, 2)
    WUSH_FENCE
    mma_issue<1>(acc, af1, bf, scur);
    WUSH_FENCE
    if (more) load_w_frag(bf, kt + 1, 1);
    WUSH_READ_A(af1, 3)
    WUSH_FENCE
    mma_issue<2>(acc, af0, bf, scur);
    WUSH_FENCE
    if (more) load_w_frag(bf, kt + 1, 2);
    WUSH_FENCE
    mma_issue<3>(acc, af1, bf, scur);
    WUSH_FENCE
    if (more) load_w_frag(bf, kt + 1, 3);
#undef WUSH_FENCE
#undef WUSH_READ_A
    if (more) store_x(stg, (kt + 1) & 1);
    __syncthreads();
  };
  for (int kt = 0; kt + 1 < KT; ++kt) {
    iteration(kt, sc0, sc1, std::true_type{});
    sc0 = sc1;
  }
  iteration(KT - 1, sc0, sc1, std::false_type{});
  __builtin_amdgcn_sched_barrier(0);

  // ---- epilogue: accumulator e of lane (r, kh) in MFMA tile (i, j) is output
  // row 32*i + 8*(e/4) + 4*kh + e%4, column 64*wave + 32*j + r of the tile.
#pragma unroll
  for (int i = 0; i < 8; ++i) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      __builtin_amdgcn_sched_barrier(0);   // one MFMA tile at a time: keeps the epilogue out of scratch
      const int col = n0 + 64 * wave + 32 * j + r;
      if (col < N) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = m0 + 32 * i + 8 * (e >> 2) + 4 * kh + (e & 3);
          if (row < M) {
            if (OUT_F32) reinterpret_cast<float*>(Y)[(int64_t)row * ldy + col] = acc[i][j][e];
            else reinterpret_cast<uint16_t*>(Y)[(int64_t)row * ldy + col] = f32_to_bf16_bits(acc[i][j][e]);
          }
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_mxfp4_gemm_frag(const void* Xq, const void* Xs, const void* Wq, const void* Ws,
                                  int64_t M, int64_t N, int64_t K, int out_f32, void* Y, int64_t ldy,
                                  hipStream_t stream) {
  const int tiles_m = (int)((M + kTM - 1) / kTM), tiles_n = (int)((N + kTN - 1) / kTN);
  dim3 grid((unsigned)(tiles_m * tiles_n)), block(256);
  if (out_f32)
    gemm_frag_kernel<true><<<grid, block, 0, stream>>>((const uint8_t*)Xq, (const uint8_t*)Xs, (const uint8_t*)Wq,
                                                      (const uint8_t*)Ws, (int)M, (int)N, (int)K, Y, ldy, tiles_m, tiles_n);
  else
    gemm_frag_kernel<false><<<grid, block, 0, stream>>>((const uint8_t*)Xq, (const uint8_t*)Xs, (const uint8_t*)Wq,
                                                       (const uint8_t*)Ws, (int)M, (int)N, (int)K, Y, ldy, tiles_m, tiles_n);
  return hipGetLastError();
}

}  // namespace wush
