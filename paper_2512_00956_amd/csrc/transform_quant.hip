// Fused activation transform + MXFP4 quantization for gfx950:
//   Xq, Xs = q(T_wush X)   (layer forward-pass equation; "Fused WUSH + Quant
//   kernel" in section "GPU Kernel Support" states the operation: C independent
//   dense GxG transforms fused with the quantizer, memory bound at G = 32).
//
// Design (ours, for CDNA4).  The product is computed transposed,
// Yt_b^T = T_b . X_b^T, on v_mfma_f32_32x32x16_bf16 (two issues per 32x32x32
// block product).  With that orientation
//   * the X-side operand of a lane is 16 consecutive BF16 of one token: two
//     128-bit global loads straight into VGPRs, no LDS round trip;
//   * T_b is the A operand and stays in registers while the wave walks down
//     the token dimension (each wave owns 4 adjacent blocks = 256 B of every
//     token row, the 4 waves of a workgroup cover 1 KiB of the row);
//   * after the MFMA a lane holds 16 output channels of ONE token, so the
//     per-32 AbsMax is 15 in-register max + one v_permlane32_swap;
//   * rows of T_b are fed in a permuted order so that those 16 channels are
//     a contiguous half of the group; the hardware fp4 convert then emits the
//     codes in canonical nibble order.
// Codes of two blocks are exchanged between the wave halves so every lane
// stores 32 contiguous bytes; the 4 scale bytes of a token go out as one dword.
#include "transform_quant_core.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

using tq::kNB;
using tq::kTileM;
using tq::XFrag;
constexpr int kWaves = 4;    // waves per workgroup

// TG = token tiles a workgroup handles at a time: its 4 TG waves are TG groups of four, group g
// taking steps g, g + TG, ... of the workgroup's walk.  A wave's tile is one long dependent chain (MFMA,
// accumulator reads, max tree, lane swap, scale, converts: about 2600 cycles for 280 instructions), so
// a CU with one wave per SIMD idles most of the time; a second group per workgroup fills the gaps
// without leaving the placement of more, smaller workgroups to the dispatcher.
// PF = tiles a wave keeps in flight ahead of the one it computes on (PF + 1 operand register sets of
// 32 VGPRs, rotated by unrolling, never copied).  PF = 1 with one wave group (three waves per SIMD fit),
// PF = 2 with two (one workgroup per CU, two waves per SIMD, so 190 registers cost nothing): 2-3 % faster from
// HBM on 16384 x 4096 and 8192 x 8192 activations (5.2 -> 5.3 TB/s); a third tile ahead adds nothing.
template <bool DBG, bool TILED, int TG, int PF>
__global__ __launch_bounds__(kWaves * TG * 64) void transform_quant_kernel(
    const uint16_t* __restrict__ X, int64_t ldx, const uint16_t* __restrict__ T,
    uint8_t* __restrict__ Xq, uint8_t* __restrict__ Xs, float* __restrict__ dbg,
    int M, int K, int C, int tiles_per_wg, int rule) {
  const int lane = threadIdx.x & 63;
  const int wave = (threadIdx.x >> 6) % kWaves;   // which four blocks
  const int tg = (threadIdx.x >> 6) / kWaves;     // which tile group
  const int tok = lane & 31;
  const int h = lane >> 5;
  const int bfirst = (blockIdx.y * kWaves + wave) * kNB;
  if (bfirst >= C) return;  // wave-uniform
  const int nb = min(kNB, C - bfirst);

  v8bf ta[kNB][2];
  tq::load_transforms(ta, T, bfirst, C, tok, h);

  // Walk step j of this workgroup is tile j gridDim.x + blockIdx.x: at any time the workgroups of the grid
  // are within one window of consecutive token tiles, so the chip as a whole reads (and writes) HBM
  // front to back.  With contiguous runs of tiles per workgroup instead, the same loads reach 4.7 TB/s
  // from HBM where this order reaches 5.4 (16384 x 4096, measured with the arithmetic left out).
  const int ntiles = (M + kTileM - 1) / kTileM;
  auto tile_of = [&](int j) { return j * (int)gridDim.x + (int)blockIdx.x; };
  auto valid = [&](int j) { return j < tiles_per_wg && tile_of(j) < ntiles; };
  if (!valid(tg)) return;

  // Every load of the walk is issued unconditionally: a tile past the end of the walk is replaced by
  // one row of the first tile for all lanes (a single cache line per instruction, already resident).
  // With a branch around the prefetch the compiler cannot know how many loads are outstanding where
  // it waits for the current tile and drains them all, which ends the lookahead.
  const int row_spare = min(tile_of(tg) * kTileM, M - 1);
  auto tile_row = [&](int j) { return valid(j) ? min(tile_of(j) * kTileM + tok, M - 1) : row_spare; };
  XFrag x[PF + 1][kNB];
#pragma unroll
  for (int s = 0; s < PF; ++s) {
    tq::load_tile(x[s], X, ldx, tile_row(tg + s * TG), bfirst, C, h);
    // keeps the tiles' loads in walk order: the first wait of the loop counts the loads behind tile 0
    __builtin_amdgcn_sched_barrier(0);
  }

  for (int base = tg; base < tiles_per_wg; base += (PF + 1) * TG) {
#pragma unroll
    for (int s = 0; s <= PF; ++s) {
      const int j = base + s * TG;
      if (!valid(j)) return;  // wave-uniform; leaves the kernel so that no path with fewer loads in flight rejoins the loop
      const int t = tile_of(j);
      const int m = t * kTileM + tok;
      const bool row_ok = m < M;
      tq::load_tile(x[(s + PF) % (PF + 1)], X, ldx, tile_row(j + PF * TG), bfirst, C, h);

      v4u out[2];
      uint32_t sbytes;
      float* dbg_row = (DBG && row_ok) ? dbg + (int64_t)m * K + 32 * bfirst + 16 * h : nullptr;
      tq::transform_quantize<DBG>(ta, x[s], rule, out, sbytes, dbg_row, nb);
      if (TILED) {
        if (row_ok) tq::store_tile_tiled<true>(out, sbytes, Xq, Xs, t, K >> 8, bfirst, tok, h);
      } else if (row_ok) {
        uint8_t* q = Xq + (int64_t)m * (K / 2) + 16 * bfirst + 32 * h;
        if (nb == kNB && (C & 3) == 0) {
          __builtin_nontemporal_store(out[0], reinterpret_cast<v4u*>(q));
          __builtin_nontemporal_store(out[1], reinterpret_cast<v4u*>(q + 16));
          if (h == 0) __builtin_nontemporal_store(sbytes, reinterpret_cast<uint32_t*>(Xs + (int64_t)m * C + bfirst));
        } else {
          // ragged tail of the channel dimension: blocks 2h and 2h+1 of this lane
#pragma unroll
          for (int p = 0; p < 2; ++p)
            if (2 * h + p < nb) *reinterpret_cast<v4u*>(q + 16 * p) = out[p];
          if (h == 0)
            for (int bb = 0; bb < nb; ++bb) Xs[(int64_t)m * C + bfirst + bb] = (uint8_t)(sbytes >> (8 * bb));
        }
      }
    }
  }
}

}  // namespace

int device_cu_count() {
  static std::atomic<int> cus[64];   // zero-initialized; per device
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  const bool tracked = dev >= 0 && dev < 64;
  if (tracked && (n = cus[dev].load(std::memory_order_relaxed)) > 0) return n;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) return 256;
  if (tracked) cus[dev].store(n, std::memory_order_relaxed);
  return n;
}

// Token tiles each workgroup walks down (the register-resident transforms are loaded once per
// wave).  Chosen from the number of (tile, channel group) units T against the CU count, after
// sweeps of the walk on 512..32768 tokens x 4096..28672 channels (graph replay for the small ones):
//   T <= 1.5 CUs : 1   (latency bound: 1024 x 4096 takes 3.7 us with a walk of 1, 4.6 with 2)
//   T <= 6 CUs   : 2   (2048 x 4096: 4.9 us against 5.2; 2048 x 8192: 8.8 against 9.7)
//   T < 16 CUs   : 4   (4096 x 8192: 15.8 us against 21.2 with 1 and 16.4 with 8)
//   larger       : a grid of at most one workgroup per CU, all busy from start to end: 6.0-7.2 TB/s
//                  cache resident, where grids of 2-4 workgroups per CU lose up to a third to an
//                  uneven last round (8192 x 8192: 42 -> 28 us).
int token_walk(int ntiles, int col_groups) {
  const int cus = device_cu_count();
  const int64_t units = (int64_t)ntiles * col_groups;
  if (2 * units <= 3 * cus) return 1;
  if (units <= 6 * cus) return 2;
  if (units < 16 * cus) return 4;
  const int wg_rows = cus / col_groups > 0 ? cus / col_groups : 1;
  return (ntiles + wg_rows - 1) / wg_rows;
}

// The same for a kernel whose workgroups can take two tiles at a time (tile groups, above):
// tiles per workgroup and groups.  Up to 3 CUs' worth of units the single group wins or ties
// (2048 x 4096: 5.0 us against 5.2).  Beyond, two groups and a grid of at most one workgroup per CU
// (a CU holds one eight-wave workgroup of this kernel at a time): 2048 x 8192: 8.2 us against 8.7,
// 4096 x 8192: 15.0 against 15.9, 16384 x 4096: 26.2 against 28.3, 8192 x 8192: 26.7 against 28.4
// (three and four groups: 26.7-27.6).
Walk token_walk_groups(int ntiles, int col_groups) {
  const int cus = device_cu_count();
  const int64_t units = (int64_t)ntiles * col_groups;
  if (units <= 3 * cus) return {token_walk(ntiles, col_groups), 1};
  const int wg_rows = cus / col_groups > 0 ? cus / col_groups : 1;
  const int walk = (ntiles + wg_rows - 1) / wg_rows;
  return {walk < 2 ? 2 : walk, 2};
}

hipError_t launch_transform_quant(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T,
                                  int rule, int tiled, void* Xq, void* Xs, float* dbg, hipStream_t stream) {
  const int C = (int)(K / 32);
  const int col_groups = (C + kWaves * kNB - 1) / (kWaves * kNB);
  const int ntiles = (int)((M + kTileM - 1) / kTileM);
  const Walk walk = token_walk_groups(ntiles, col_groups);
  const int tiles_per_wg = walk.tiles_per_wg;
  dim3 grid((ntiles + tiles_per_wg - 1) / tiles_per_wg, col_groups);
  dim3 block(kWaves * 64 * walk.groups);
  // two tiles of lookahead where the workgroup is the CU's only one (two waves per SIMD, 256 registers each)
#define WUSH_TQ_LAUNCH(DBG, TILED, TG)                                                                 \
  transform_quant_kernel<DBG, TILED, TG, TG><<<grid, block, 0, stream>>>(                              \
      (const uint16_t*)X, ldx, (const uint16_t*)T, (uint8_t*)Xq, (uint8_t*)Xs, dbg, (int)M, (int)K, C, \
      tiles_per_wg, rule)
  if (walk.groups == 2) {
    if (dbg) {
      if (tiled) WUSH_TQ_LAUNCH(true, true, 2); else WUSH_TQ_LAUNCH(true, false, 2);
    } else {
      if (tiled) WUSH_TQ_LAUNCH(false, true, 2); else WUSH_TQ_LAUNCH(false, false, 2);
    }
  } else if (dbg) {
    if (tiled) WUSH_TQ_LAUNCH(true, true, 1); else WUSH_TQ_LAUNCH(true, false, 1);
  } else {
    if (tiled) WUSH_TQ_LAUNCH(false, true, 1); else WUSH_TQ_LAUNCH(false, false, 1);
  }
#undef WUSH_TQ_LAUNCH
  return hipGetLastError();
}

}  // namespace wush
