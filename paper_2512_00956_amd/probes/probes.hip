// Measurement aids for the benchmark, built into a library of their own
// (libwush_probes.so): nothing here is part of the layer path, and the
// product library neither contains nor calls any of it.
//
//   wushp_mfma_fp4 / wushp_mfma_f16   the GEMMs' MFMA instructions in a
//       register-only loop (the ceiling the GEMM kernels are compared against)
//   wushp_stream                       plain streaming kernels with the byte mix
//       of the fused transform + quantize kernel (4 bytes read per byte written,
//       non-temporal stores), linear or in that kernel's own access pattern.
//       Measured from HBM on 16384 x 4096 BF16: linear 5.5-5.6 TB/s; the quantizer's
//       tiles 5.3-5.4 when they are dealt round-robin over the workgroups (one window
//       moves down the rows) and 4.7 when every workgroup gets a contiguous run of them,
//       whatever the shape of a wave's tile (32 rows x 256 B, whole lines, 8 rows x 1 KiB)
//       and whatever the store pattern; the quantizer itself 5.2-5.4.
//
// C ABI (all pointers are device pointers, `stream` is a hipStream_t; return
// value: 0 = launched, 1 = bad argument, 2 = HIP launch error):
//   int wushp_mfma_fp4(const void* operand_bits, int iters, int blocks, void* cycles_ticks, void* stream);
//   int wushp_mfma_fp4_colmajor(...same...);   the same MFMAs issued column block by column block
//   int wushp_mfma_f16(const void* operand_f16, int iters, int blocks, void* cycles_ticks, void* stream);
//   int wushp_stream(const void* src, long long rows, long long row_bytes, void* dst, int mode, int blocks,
//                    void* stream);
//
// First probe: the block-scaled FP4 MFMA
// (v_mfma_scale_f32_32x32x64_f8f6f4) in a register-only loop, the ceiling the
// MXFP4 GEMM is compared against.  One wave per SIMD, 64 independent MFMAs per
// trip (the GEMM's 8 x 2 accumulator tiles x 4 issues), operands loaded once from
// a caller-provided buffer so that the caller decides the bit patterns: the
// sustained rate depends on them (the shader clock drops with switching
// activity), which is the point of the measurement.  Every workgroup reports its
// shader-clock cycles and 100 MHz real-time ticks.
#include "../csrc/transform_quant_core.hpp"

namespace wush {

namespace {

// ORDER 0: row block outer, column block inner (consecutive MFMAs share the X-side operand, the order of the
// GEMM's loop); ORDER 1: column block outer (eight consecutive MFMAs share the W-side operand).
template <int ORDER>
__global__ __launch_bounds__(256) void mfma_probe_kernel(const int* __restrict__ in, int iters,
                                                         unsigned long long* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  v16f acc[8][2];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = (v16f){0};
  v4i af[8], bf[2][4];
  int sa[8], sb[2];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    af[i] = *reinterpret_cast<const v4i*>(in + 4 * (64 * i + lane));           // 8 KiB of X-side fragments
    sa[i] = 0x7f7f7f7f;                                                         // scale 1.0
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) bf[j][kk] = *reinterpret_cast<const v4i*>(in + 2048 + 4 * (64 * (4 * j + kk) + lane));
    sb[j] = 0x7f7f7f7f;
  }
  __builtin_amdgcn_sched_barrier(0);
  const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  __builtin_amdgcn_sched_barrier(0);
  for (int it = 0; it < iters; ++it) {
#define WUSH_PROBE_MMA(KK, i, j)                                                                                      \
  {                                                                                                                   \
    const v8i A = {af[i][0], af[i][1], af[i][2], af[i][3], 0, 0, 0, 0};                                               \
    const v8i B = {bf[j][KK][0], bf[j][KK][1], bf[j][KK][2], bf[j][KK][3], 0, 0, 0, 0};                               \
    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(B, A, acc[i][j], 4, 4, KK, sb[j], KK, sa[i]);         \
  }
#define WUSH_PROBE_ISSUE(KK)                                                                                          \
  if (ORDER == 0) {                                                                                                   \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) _Pragma("unroll") for (int j = 0; j < 2; ++j) WUSH_PROBE_MMA(KK, i, j) \
  } else {                                                                                                            \
    _Pragma("unroll") for (int j = 0; j < 2; ++j) _Pragma("unroll") for (int i = 0; i < 8; ++i) WUSH_PROBE_MMA(KK, i, j) \
  }
    WUSH_PROBE_ISSUE(0)
    WUSH_PROBE_ISSUE(1)
    WUSH_PROBE_ISSUE(2)
    WUSH_PROBE_ISSUE(3)
#undef WUSH_PROBE_ISSUE
#undef WUSH_PROBE_MMA
  }
  __builtin_amdgcn_sched_barrier(0);
  const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  float r = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) r += acc[i][j][e];
  if (threadIdx.x == 0) {
    out[2 * blockIdx.x] = c1 - c0 + (r == 1.2345f ? 1 : 0);   // keeps the accumulators live
    out[2 * blockIdx.x + 1] = r1 - r0;
  }
}

// The same for the FP16 MFMA (v_mfma_f32_32x32x16_f16), the instruction of the NVFP4 GEMM:
// 4 x 4 accumulator tiles x 4 K steps = 64 independent MFMAs per trip.  `in` = 16 KiB of FP16:
// X-side fragments [4 steps][4 row blocks][64 lanes][8], then the W side likewise.
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(256) void mfma_f16_probe_kernel(const v8h* __restrict__ in, int iters,
                                                             unsigned long long* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  v16f acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = (v16f){0};
  // 8 KiB per side = 8 fragments of 1 KiB: two K steps x 4 row blocks, reused for steps 2 and 3
  v8h a[2][4], b[2][4];
#pragma unroll
  for (int g = 0; g < 2; ++g)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a[g][i] = in[(4 * g + i) * 64 + lane];
      b[g][i] = in[512 + (4 * g + i) * 64 + lane];
    }
  __builtin_amdgcn_sched_barrier(0);
  const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  __builtin_amdgcn_sched_barrier(0);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[g & 1][i], b[g & 1][j], acc[i][j], 0, 0, 0);
  }
  __builtin_amdgcn_sched_barrier(0);
  const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  float r = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) r += acc[i][j][e];
  if (threadIdx.x == 0) {
    out[2 * blockIdx.x] = c1 - c0 + (r == 1.2345f ? 1 : 0);   // keeps the accumulators live
    out[2 * blockIdx.x + 1] = r1 - r0;
  }
}


// Streaming kernels with the byte mix of the fused transform + quantize kernel: per 16 B
// read, 4 B of "codes" and 1/4 B of "scales" are written with non-temporal stores.
//   mode 0: linear.  A wave reads 4 KiB contiguous per step (four 128-bit loads per lane)
//           and writes 1 KiB; waves take steps round-robin.
//   mode 1: the quantizer's own pattern.  A wave reads 32 rows x 256 B (tile = 32 tokens x
//           4 transform blocks) with the same eight 128-bit loads per lane and writes the
//           tile's codes and scales at the offsets of the fragment-order layout; one tile
//           of lookahead in registers; tiles dealt round-robin over the workgroups of a column group.
//           What is left out is the arithmetic.
//   mode 2: as mode 1 with 8 blocks per wave (32 rows x 512 B).
//   mode 3: as mode 1 with a contiguous run of tiles per workgroup.
//   modes 4, 5, 6: as mode 1 with the same bytes stored at linear offsets / without the scale stores /
//           with cached instead of non-temporal stores.
//   modes 10, 11: read-pattern probes: a wave's tile is 32 or 8 rows x 256 B or 1 KiB of each,
//           linear stores of a quarter of the bytes.  mode 13: the tile of mode 10 (32 rows x 256 B) read
//           with whole 128-byte lines per load instruction (8 rows each) instead of 32 bytes of 32 rows.
//   mode 50: linear, read only (what a weight-streaming kernel could reach): the xor of all a wave read is stored
//           once, 1 KiB per wave, at the end.
//   modes 30, 40: as 0 and 20 with non-temporal loads.  From HBM the linear stream gains 3 % (5.75 TB/s) and
//           loses 13 % cache resident; the tile pattern, whose load instructions take a 128-byte line in
//           four parts, drops to 3.7 TB/s.
//   modes 20, 21, 23: as 10, 11, 13 with the tiles dealt round-robin over the workgroups of a column
//           group instead of in contiguous runs: at any time the chip reads one window of consecutive rows.
// rows x row_bytes is the source (row_bytes a multiple of 1024, rows of 32); dst holds
// rows * row_bytes / 4 bytes of "codes" followed by rows * row_bytes / 64 bytes of "scales".
template <bool NT>
__device__ __forceinline__ v4u load16(const v4u* p) {
  return NT ? __builtin_nontemporal_load(p) : *p;
}

template <bool NT, bool READ_ONLY = false>
__global__ __launch_bounds__(512) void stream_linear_kernel(const v4u* __restrict__ src, long long n_steps,
                                                            v4u* __restrict__ dst) {
  const int lane = threadIdx.x & 63;
  const long long wave = (long long)blockIdx.x * 8 + (threadIdx.x >> 6), nwaves = (long long)gridDim.x * 8;
  if (wave >= n_steps) return;
  // two steps in flight, two register sets that swap roles (no copies, no conditional loads: the
  // compiler's wait counts stay exact)
  v4u x[3][4];
  v4u sum = {0, 0, 0, 0};   // READ_ONLY: the xor of everything the wave read, stored once at the end
  auto step_of = [&](long long st) { return st < n_steps ? st : wave; };
#pragma unroll
  for (int s = 0; s < 2; ++s) {
#pragma unroll
    for (int i = 0; i < 4; ++i) x[s][i] = load16<NT>(src + step_of(wave + s * nwaves) * 256 + 64 * i + lane);
    __builtin_amdgcn_sched_barrier(0);
  }
  for (long long base = wave; base < n_steps; base += 3 * nwaves) {
#pragma unroll
    for (int s = 0; s < 3; ++s) {
      const long long st = base + s * nwaves;
      if (st >= n_steps) {
        if (READ_ONLY) dst[wave * 64 + lane] = sum;
        return;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) x[(s + 2) % 3][i] = load16<NT>(src + step_of(st + 2 * nwaves) * 256 + 64 * i + lane);
      const v4u o = x[s][0] ^ x[s][1] ^ x[s][2] ^ x[s][3];
      if (READ_ONLY) sum ^= o;
      else __builtin_nontemporal_store(o, dst + st * 64 + lane);
    }
  }
  if (READ_ONLY) dst[wave * 64 + lane] = sum;
}

template <int PF, int NBW>
__global__ __launch_bounds__(512) void stream_tiles_kernel(const uint16_t* __restrict__ X, int M, int K,
                                                           uint8_t* __restrict__ Xq, uint8_t* __restrict__ Xs,
                                                           int tiles_per_wg, int interleaved, int store_mode) {
  // NBW = blocks per wave (the quantizer: 4 = 256 B of every row; 8 = 512 B)
  // store_mode 0: the quantizer's stores; 1: the same bytes at linear offsets; 2: codes only; 3: cached stores
  using namespace tq;
  constexpr int TG = 2;
  const int lane = threadIdx.x & 63, wave = (threadIdx.x >> 6) & 3, tg = threadIdx.x >> 8;
  const int tok = lane & 31, h = lane >> 5, C = K / 32;
  const int bfirst = (blockIdx.y * 4 + wave) * NBW;
  if (bfirst >= C) return;
  const int ntiles = M / kTileM;
  // walk step j -> tile: dealt round-robin over the workgroups (the quantizer's walk) or in contiguous runs
  auto tile_of = [&](int j) {
    return interleaved ? j * (int)gridDim.x + (int)blockIdx.x : (int)blockIdx.x * tiles_per_wg + j;
  };
  auto valid = [&](int j) { return j < tiles_per_wg && tile_of(j) < ntiles; };
  if (!valid(tg)) return;
  const int row_spare = tile_of(tg) * kTileM;
  auto tile_row = [&](int j) { return valid(j) ? tile_of(j) * kTileM + tok : row_spare; };
  XFrag x[PF + 1][NBW];
  auto load = [&](XFrag (&d)[NBW], int row) {
#pragma unroll
    for (int g = 0; g < NBW / kNB; ++g)
      load_tile(reinterpret_cast<XFrag (&)[kNB]>(d[kNB * g]), X, K, row, bfirst + kNB * g, C, h);
  };
#pragma unroll
  for (int s = 0; s < PF; ++s) {
    load(x[s], tile_row(tg + s * TG));
    __builtin_amdgcn_sched_barrier(0);
  }
  for (int base = tg; base < tiles_per_wg; base += (PF + 1) * TG) {
#pragma unroll
    for (int s = 0; s <= PF; ++s) {
      const int j = base + s * TG;
      if (!valid(j)) return;
      const int t = tile_of(j);
      load(x[(s + PF) % (PF + 1)], tile_row(j + PF * TG));
      typedef unsigned int u4 __attribute__((ext_vector_type(4)));
#pragma unroll
      for (int g = 0; g < NBW / kNB; ++g) {
        v4u out[2];
#pragma unroll
        for (int p = 0; p < 2; ++p)
          out[p] = __builtin_bit_cast(u4, x[s][4 * g + 2 * p].lo) ^ __builtin_bit_cast(u4, x[s][4 * g + 2 * p].hi) ^
                   __builtin_bit_cast(u4, x[s][4 * g + 2 * p + 1].lo) ^ __builtin_bit_cast(u4, x[s][4 * g + 2 * p + 1].hi);
        const uint32_t sb = out[0][0] ^ out[1][0];
        if (store_mode == 0) {
          store_tile_tiled<true>(out, sb, Xq, Xs, t, K >> 8, bfirst + kNB * g, tok, h);
        } else if (store_mode == 1) {
          const int64_t unit = ((int64_t)t * gridDim.y * 4 + blockIdx.y * 4 + wave) * (NBW / kNB) + g;
          v4u* q = reinterpret_cast<v4u*>(Xq) + unit * 128 + lane;
          __builtin_nontemporal_store(out[0], q);
          __builtin_nontemporal_store(out[1], q + 64);
          if (h == 0) __builtin_nontemporal_store(sb, reinterpret_cast<uint32_t*>(Xs) + unit * 32 + tok);
        } else if (store_mode == 2) {
          const int bf = bfirst + kNB * g, kt = bf >> 3, khg = (bf >> 2) & 1;
          uint8_t* q = Xq + ((((int64_t)t * (K >> 8) + kt) * 4 + 2 * h) * 64 + khg * 32 + tok) * 16;
          __builtin_nontemporal_store(out[0], reinterpret_cast<v4u*>(q));
          __builtin_nontemporal_store(out[1], reinterpret_cast<v4u*>(q + 1024));
        } else {
          store_tile_tiled<false>(out, sb, Xq, Xs, t, K >> 8, bfirst + kNB * g, tok, h);
        }
      }
    }
  }
}

// Read-pattern probe: a wave's tile is ROWS rows x (8 KiB / ROWS) contiguous bytes of each (eight 128-bit
// loads per lane, one tile of lookahead), the four column waves of a workgroup sit side by side, two wave
// groups take alternate tiles; stores are linear (a quarter of the bytes read).  ROWS = 32 is the
// quantizer's footprint, smaller ROWS make it more linear.
// FULL_LINES (ROWS = 32 only): the same tile, but every load instruction covers 8 rows x one whole 128-byte line
// instead of 32 rows x 32 bytes.
template <int ROWS, bool FULL_LINES = false, bool NT = false>
__global__ __launch_bounds__(512) void stream_rows_kernel(const uint8_t* __restrict__ X, int rows, int row_bytes,
                                                          v4u* __restrict__ dst, int tiles_per_wg, int interleaved) {
  constexpr int kSeg = 8192 / ROWS;          // bytes of a row per wave tile
  constexpr int kLanesPerRow = 64 / ROWS;    // lanes side by side on one row within a load instruction
  const int lane = threadIdx.x & 63, wave = (threadIdx.x >> 6) & 3, tg = threadIdx.x >> 8;
  const int r = lane / kLanesPerRow, c = lane % kLanesPerRow;
  const int64_t col0 = ((int64_t)blockIdx.y * 4 + wave) * kSeg;
  if (col0 >= row_bytes) return;
  const int ntiles = rows / ROWS;
  // Walk step j of this workgroup -> tile.  Contiguous: the workgroup owns tiles_per_wg consecutive tiles
  // (the quantizer's walk).  Interleaved: at step j all workgroups of a column group read gridDim.x
  // consecutive tiles, so the chip as a whole moves one window down the rows.
  auto tile_of = [&](int j) {
    return interleaved ? j * (int)gridDim.x + (int)blockIdx.x : (int)blockIdx.x * tiles_per_wg + j;
  };
  auto valid = [&](int j) { return j < tiles_per_wg && tile_of(j) < ntiles; };
  if (!valid(tg)) return;
  const int t_spare = tile_of(tg);
  auto load = [&](v4u (&d)[8], int j) {
    const int tt = valid(j) ? tile_of(j) : t_spare;
    if (FULL_LINES) {
      const uint8_t* p = X + ((int64_t)tt * ROWS + (lane >> 3)) * row_bytes + col0 + (lane & 7) * 16;
#pragma unroll
      for (int i = 0; i < 8; ++i) d[i] = load16<NT>(reinterpret_cast<const v4u*>(p + (int64_t)(8 * (i & 3)) * row_bytes + 128 * (i >> 2)));
    } else {
      const uint8_t* p = X + ((int64_t)tt * ROWS + r) * row_bytes + col0 + c * 16;
#pragma unroll
      for (int i = 0; i < 8; ++i) d[i] = load16<NT>(reinterpret_cast<const v4u*>(p + i * (kSeg / 8)));
    }
  };
  v4u x[2][8];
  load(x[0], tg);
  __builtin_amdgcn_sched_barrier(0);
  const int64_t units_per_tile = (int64_t)gridDim.y * 4;   // (tile, column wave) units
  for (int base = tg; base < tiles_per_wg; base += 4) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int j = base + 2 * s;
      if (!valid(j)) return;
      load(x[s ^ 1], j + 2);
      v4u o0 = x[s][0] ^ x[s][1] ^ x[s][2] ^ x[s][3], o1 = x[s][4] ^ x[s][5] ^ x[s][6] ^ x[s][7];
      const int64_t unit = (int64_t)tile_of(j) * units_per_tile + blockIdx.y * 4 + wave;
      __builtin_nontemporal_store(o0, dst + unit * 128 + lane);
      __builtin_nontemporal_store(o1, dst + unit * 128 + 64 + lane);
    }
  }
}

}  // namespace

}  // namespace wush

extern "C" {

int wushp_mfma_f16(const void* operand_f16, int iters, int blocks, void* cycles_ticks, void* stream) {
  if (!operand_f16 || !cycles_ticks || iters <= 0 || iters > (1 << 20) || blocks <= 0 || blocks > 4096) return 1;
  wush::mfma_f16_probe_kernel<<<dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const wush::v8h*>(operand_f16), iters, static_cast<unsigned long long*>(cycles_ticks));
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

int wushp_mfma_fp4(const void* operand_bits, int iters, int blocks, void* cycles_ticks, void* stream) {
  if (!operand_bits || !cycles_ticks || iters <= 0 || iters > (1 << 20) || blocks <= 0 || blocks > 4096) return 1;
  wush::mfma_probe_kernel<0><<<dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const int*>(operand_bits), iters, static_cast<unsigned long long*>(cycles_ticks));
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

int wushp_mfma_fp4_colmajor(const void* operand_bits, int iters, int blocks, void* cycles_ticks, void* stream) {
  if (!operand_bits || !cycles_ticks || iters <= 0 || iters > (1 << 20) || blocks <= 0 || blocks > 4096) return 1;
  wush::mfma_probe_kernel<1><<<dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const int*>(operand_bits), iters, static_cast<unsigned long long*>(cycles_ticks));
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

int wushp_stream(const void* src, long long rows, long long row_bytes, void* dst, int mode, int blocks, void* stream) {
  if (!src || !dst || rows <= 0 || rows % 32 != 0 || row_bytes <= 0 || row_bytes % 1024 != 0 || blocks <= 0 ||
      blocks > 65536 || rows > (1 << 30) || row_bytes > (1 << 23))
    return 1;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (mode == 0) {
    wush::stream_linear_kernel<false><<<dim3((unsigned)blocks), dim3(512), 0, st>>>(
        static_cast<const wush::v4u*>(src), rows * row_bytes / 4096, static_cast<wush::v4u*>(dst));
  } else if (mode == 50) {   // read only: every wave stores 1 KiB once (dst: at least blocks * 8 KiB)
    wush::stream_linear_kernel<false, true><<<dim3((unsigned)blocks), dim3(512), 0, st>>>(
        static_cast<const wush::v4u*>(src), rows * row_bytes / 4096, static_cast<wush::v4u*>(dst));
  } else if (mode == 30) {
    wush::stream_linear_kernel<true><<<dim3((unsigned)blocks), dim3(512), 0, st>>>(
        static_cast<const wush::v4u*>(src), rows * row_bytes / 4096, static_cast<wush::v4u*>(dst));
  } else if (mode >= 1 && mode <= 6) {
    const int nbw = mode == 2 ? 8 : 4;
    const int interleaved = mode != 3;
    const int store_mode = mode >= 4 ? mode - 3 : 0;   // modes 4, 5, 6: mode 1 with other stores
    const int K = (int)(row_bytes / 2), ntiles = (int)(rows / 32);
    if (K % (128 * nbw) != 0) return 1;
    const int col_groups = K / (128 * nbw);
    const int wg_rows = blocks / col_groups > 0 ? blocks / col_groups : 1;
    int walk = (ntiles + wg_rows - 1) / wg_rows;
    if (walk < 2) walk = 2;
    dim3 grid((unsigned)((ntiles + walk - 1) / walk), (unsigned)col_groups);
    uint8_t* q = static_cast<uint8_t*>(dst);
    uint8_t* s = q + rows * row_bytes / 4;
    const uint16_t* x = static_cast<const uint16_t*>(src);
    if (nbw == 4) wush::stream_tiles_kernel<1, 4><<<grid, dim3(512), 0, st>>>(x, (int)rows, K, q, s, walk, interleaved, store_mode);
    else wush::stream_tiles_kernel<1, 8><<<grid, dim3(512), 0, st>>>(x, (int)rows, K, q, s, walk, interleaved, store_mode);
  } else if (mode == 40) {   // mode 20 with non-temporal loads
    if (row_bytes % 1024 != 0) return 1;
    const int col_groups = (int)(row_bytes / 1024), ntiles = (int)(rows / 32);
    const int wg_rows = blocks / col_groups > 0 ? blocks / col_groups : 1;
    int walk = (ntiles + wg_rows - 1) / wg_rows;
    if (walk < 2) walk = 2;
    dim3 grid((unsigned)((ntiles + walk - 1) / walk), (unsigned)col_groups);
    wush::stream_rows_kernel<32, false, true><<<grid, dim3(512), 0, st>>>(
        static_cast<const uint8_t*>(src), (int)rows, (int)row_bytes, static_cast<wush::v4u*>(dst), walk, 1);
  } else if (mode == 10 || mode == 11 || mode == 13 || mode == 20 || mode == 21 || mode == 23) {
    const int interleaved = mode >= 20;   // modes 20, 21, 23: the walks of 10, 11, 13 interleaved across workgroups
    mode -= interleaved ? 10 : 0;
    const int ROWS = mode == 11 ? 8 : 32;
    const int seg = 8192 / ROWS;
    if (row_bytes % (4 * seg) != 0 || rows % ROWS != 0) return 1;
    const int col_groups = (int)(row_bytes / (4 * seg)), ntiles = (int)(rows / ROWS);
    const int wg_rows = blocks / col_groups > 0 ? blocks / col_groups : 1;
    int walk = (ntiles + wg_rows - 1) / wg_rows;
    if (walk < 2) walk = 2;
    dim3 grid((unsigned)((ntiles + walk - 1) / walk), (unsigned)col_groups);
    const uint8_t* x = static_cast<const uint8_t*>(src);
    wush::v4u* d = static_cast<wush::v4u*>(dst);
    if (mode == 10) wush::stream_rows_kernel<32><<<grid, dim3(512), 0, st>>>(x, (int)rows, (int)row_bytes, d, walk, interleaved);
    else if (mode == 11) wush::stream_rows_kernel<8><<<grid, dim3(512), 0, st>>>(x, (int)rows, (int)row_bytes, d, walk, interleaved);
    else wush::stream_rows_kernel<32, true><<<grid, dim3(512), 0, st>>>(x, (int)rows, (int)row_bytes, d, walk, interleaved);
  } else {
    return 1;
  }
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

}  // extern "C"
