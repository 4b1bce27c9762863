// MXFP4 GEMM on operands stored in the fragment-order ("tiled") layout of
// wush_device.hpp: Y = deq(Xq,Xs) . deq(Wq,Ws)^T (the layer forward-pass
// equation summed over all blocks), v_mfma_scale_f32_32x32x64_f8f6f4.
//
// Workgroup tile 256 (M) x 256 (N), 128 x 384, 128 x 256 or 128 x 128, K advances 256
// elements per iteration.  The four wavefronts split N: each owns all rows of the tile and 64
// (96) columns -- 8 x 2 (4 x 3) MFMA tiles, 256 (192) accumulator registers -- so
// one wave per SIMD.  The second shape has 3/4 of the area; the launcher takes it
// when it needs fewer rounds of the 256 CUs (2048 x 6144: 256 tiles instead of 192
// on 256 CUs).  RB = row blocks of the tile, CB = column blocks per wave.
// With a single wave per SIMD nothing hides memory or LDS latency but the
// software pipeline.  Every stream runs two K iterations ahead, and the loads
// of an iteration are spread one by one between its 64 MFMAs so that no burst
// of memory instructions ever blocks the (in-order) MFMA issue:
//   * W fragments (the wave's own 64 columns) go global -> VGPR directly: in
//     the tiled layout a fragment is 1 KiB contiguous in lane order, so every
//     load is a perfectly coalesced 128-bit access and no two waves load the
//     same bytes.  Two register sets; a fragment register is refilled with
//     tile kt+2 right after the MFMA issue of tile kt that consumed it.  The
//     last issue runs column by column (and its last column out of register
//     copies), so that the fragments and scale dwords it consumes are refilled
//     one per MFMA slot as well instead of in a block behind the last MFMA
//     (a block of 2 CB loads there cost 70 to 160 cycles per iteration).
//   * X fragments and X scales (shared by all four waves) go global -> LDS with
//     direct-to-LDS loads (no VGPRs in flight) into a 4-stage ring; the LDS
//     image is the same lane-linear fragment order, so the ds_read_b128 of the
//     MFMA operands are bank-conflict free without any swizzle.  A ring stage
//     is made visible one full iteration before its tile is computed, so the
//     first operand reads of tile kt+1 are issued during the last MFMAs of
//     tile kt and the per-iteration barrier never exposes LDS latency.
//   * W scales: one dword per lane per (column block, K tile); its 4 bytes are
//     the 4 MFMA issues of the iteration, selected with op_sel.
// vmcnt completes in order, so the wait in front of the per-iteration barrier
// is a fixed count: everything issued after the ring stage about to be read.
// The W fragment is the MFMA's first operand: a lane then holds four consecutive
// output columns of one token per accumulator quad, which the BF16 epilogue packs
// with two converts and writes to its LDS transpose buffer as one 8-byte store.
//
// The main-loop loads are issued from inline asm (see below), so their
// destination registers are invisible to the compiler's dependency tracking.
// The build is only valid while every W register set keeps one physical
// register assignment over the whole kernel (no copy of a register whose load
// is still in flight) and nothing spills; tests/test_build_invariants.py
// checks both on the generated code.
#include <type_traits>

#include "wush_device.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

constexpr int kFragB = 1024;                 // one 32-row x 64-element fragment
constexpr int kStages = 4;
// ring: per stage RB row blocks x 4 issues of 1 KiB, plus RB x 64 lanes x 4 B of scales
constexpr int lds_bytes(int RB) { return kStages * (RB * 4 * kFragB + RB * 256); }   // 136 KiB for RB = 8

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int CB>
struct WSet { v4i f[CB][4]; int s[CB]; };    // W fragments [column block][issue] and scale dwords

// s_waitcnt immediate (gfx9 encoding) waiting only on vmcnt <= n.
constexpr int vmcnt_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0F70; }

template <bool OUT_F32, int RB, int CB>
__global__ __launch_bounds__(256) void gemm_frag_kernel(
    const uint8_t* __restrict__ Xq, const uint8_t* __restrict__ Xs,
    const uint8_t* __restrict__ Wq, const uint8_t* __restrict__ Ws,
    int M, int N, int K, void* __restrict__ Y, int64_t ldy, int tiles_m, int tiles_n, int vec_store, int w_blocks) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
  constexpr int kTM = 32 * RB, kTN = 4 * 32 * CB;
  constexpr int kUB = RB / 4;                          // row blocks of the ring each wave fills
  constexpr int kXStageB = RB * 4 * kFragB, kXsStageB = RB * 256, kXsBase = kStages * kXStageB;
  // VMEM instructions one wave issues per pipelined iteration: its share of the X
  // fragments and X scales (direct to LDS), then CB x 4 W fragments and CB W scales.
  constexpr int kDmaPerIter = 5 * kUB, kWPerIter = 5 * CB, kVmemPerIter = kDmaPerIter + kWPerIter;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: keeps bases in SGPRs
  const int r = lane & 31, kh = lane >> 5;

  // Workgroup -> tile: every XCD (workgroup id mod 8) gets a contiguous range of
  // tile ids; ids walk the grid in bands of 8 tile rows so that the tiles an XCD
  // runs concurrently share X and W panels in its L2.
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

  const int KT = K >> 8;
  const int64_t tile_step = 4 * kFragB;                 // bytes of one (row block, K tile)

  // Operand buffers are padded to whole 256-row tiles, so every address below
  // is "uniform base + lane offset"; rows past M or N are read but never stored.
  // Every global address is "wave-uniform 64-bit base (SGPR pair) + per-lane 32-bit
  // offset (one constant VGPR) + immediate": no vector ALU work per load.
  const int loff = 16 * lane, soff = 4 * lane;
  // X: this wave fills row blocks kUB*wave .. of every ring stage.
  const uint8_t* xsrc = Xq + (int64_t)(tm * RB + kUB * wave) * KT * tile_step;
  const uint8_t* xssrc = Xs + (int64_t)(tm * RB + kUB * wave) * KT * 256;
  // W fragments and scales of this wave's CB column blocks.  The packed buffers are
  // padded to 256 rows (w_blocks blocks of 32); a 384-wide tile can reach past that,
  // so every block index is clamped to the last block of the buffer: the load stays
  // in bounds and the columns it feeds lie past N, which are never stored.
  int64_t wblk[CB];
#pragma unroll
  for (int j = 0; j < CB; ++j) wblk[j] = min(tn * 4 * CB + CB * wave + j, w_blocks - 1);

  // direct-to-LDS loads of tile kt: fragment f (0..7) of this wave's two row
  // blocks, and their two scale dwords
  // The direct-to-LDS loads are issued from inline asm on purpose.  The compiler
  // classifies global_load_lds as a load AND a store; with such an operation
  // pending it assumes vmcnt may retire out of order and turns every wait for a
  // W register load into vmcnt(0), which drains the whole two-iteration
  // pipeline once per iteration.  Issued from asm they are invisible to its
  // bookkeeping; its own vmcnt(n) waits then undercount the younger operations
  // (they wait for more than needed, never for less) and the explicit wait in
  // front of the barrier covers the LDS data.  m0 has no other user in this kernel, and the
  // compiler never keeps a value of its own in it across statements: it is a reserved register of
  // this target (naming it in the clobber list is rejected with "clobber list contains reserved
  // registers"), written immediately before each instruction the compiler itself emits that reads it.
  const uint32_t lds_base = (uint32_t)(uintptr_t)smem;   // LDS byte address of the ring
  // The four fragments (kk) of one (row block, K tile) are 4 KiB contiguous both in
  // memory and in the ring stage; the instruction's immediate offset is added to
  // the global AND to the LDS address, so they share one base and one m0 value.
  auto dma16 = [&](const uint8_t* src, uint32_t lds_addr, int kk) {
    switch (kk) {
      case 0: asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(loff), "s"(src), "s"(lds_addr)); break;
      case 1: asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024" ::"v"(loff), "s"(src), "s"(lds_addr)); break;
      case 2: asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 offset:2048" ::"v"(loff), "s"(src), "s"(lds_addr)); break;
      default: asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 offset:3072" ::"v"(loff), "s"(src), "s"(lds_addr)); break;
    }
  };
  auto dma4 = [&](const uint8_t* src, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dword %0, %1" ::"v"(soff), "s"(src), "s"(lds_addr));
  };
  auto dma_x_frag = [&](int kt, int f) {
    const int u = f >> 2, kk = f & 3;
    dma16(xsrc + ((int64_t)u * KT + kt) * tile_step, lds_base + (kt % kStages) * kXStageB + (kUB * wave + u) * 4 * kFragB, kk);
  };
  auto dma_x_scale = [&](int kt, int u) {
    dma4(xssrc + ((int64_t)u * KT + kt) * 256, lds_base + kXsBase + (kt % kStages) * kXsStageB + (kUB * wave + u) * 256);
  };
  auto dma_x = [&](int kt) {
#pragma unroll
    for (int f = 0; f < 4 * kUB; ++f) dma_x_frag(kt, f);
#pragma unroll
    for (int u = 0; u < kUB; ++u) dma_x_scale(kt, u);
  };
  // W register loads are issued from asm as well, so that NO global load of the
  // main loop is visible to the compiler's vmcnt bookkeeping and every vmcnt wait
  // below is an explicit, exact count.  Their destination registers are written
  // asynchronously; nothing may read them before the explicit wait at the start
  // of the iteration that consumes them (the generated code is checked for that:
  // no spill and no register copy in the loop).
  auto load_w_scale = [&](WSet<CB>& w, int kt, int j) {
    const uint8_t* p = Ws + (wblk[j] * KT + kt) * 256;
    asm volatile("global_load_dword %0, %1, %2" : "+v"(w.s[j]) : "v"(soff), "s"(p));
  };
  auto load_w_scales = [&](WSet<CB>& w, int kt) {
#pragma unroll
    for (int j = 0; j < CB; ++j) load_w_scale(w, kt, j);
  };
  auto load_w_frag = [&](WSet<CB>& w, int kt, int kk, int j) {
    const uint8_t* p = Wq + (wblk[j] * KT + kt) * tile_step;
    switch (kk) {
      case 0: asm volatile("global_load_dwordx4 %0, %1, %2" : "+v"(w.f[j][kk]) : "v"(loff), "s"(p)); break;
      case 1: asm volatile("global_load_dwordx4 %0, %1, %2 offset:1024" : "+v"(w.f[j][kk]) : "v"(loff), "s"(p)); break;
      case 2: asm volatile("global_load_dwordx4 %0, %1, %2 offset:2048" : "+v"(w.f[j][kk]) : "v"(loff), "s"(p)); break;
      default: asm volatile("global_load_dwordx4 %0, %1, %2 offset:3072" : "+v"(w.f[j][kk]) : "v"(loff), "s"(p)); break;
    }
  };
  auto read_x_frag = [&](int kt, int kk, int i) {
    return *reinterpret_cast<const v4i*>(smem + (kt % kStages) * kXStageB + (i * 4 + kk) * kFragB + loff);
  };
  auto read_x_scale = [&](int kt, int i) {
    return *reinterpret_cast<const int*>(smem + kXsBase + (kt % kStages) * kXsStageB + i * 256 + soff);
  };

  v16f acc[RB][CB];
#pragma unroll
  for (int i = 0; i < RB; ++i)
#pragma unroll
    for (int j = 0; j < CB; ++j) acc[i][j] = (v16f){0};

  // ---- prologue.  The two W register sets (and X scale sets) alternate by
  // iteration, chosen so that the LAST iteration always runs on set 0: the
  // drain code then exists in a single version.
  WSet<CB> wset[2];
  // The load asm takes its destination as a read-write operand, which ties every load of a W
  // register to the register its predecessor used; the chain starts here.
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int j = 0; j < CB; ++j) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) wset[t].f[j][kk] = (v4i){0, 0, 0, 0};
      wset[t].s[j] = 0;
    }
  int xsc[2][RB];
  v4i af0[RB], af1[RB];
  const int p0 = (KT - 1) & 1;                 // set of iteration 0
  // Issue order X0, X1, W(tile 0), X2, W(tile 1) -- the steady-state order (the
  // ring loads, then the W loads of an iteration) -- so that the first barrier has to wait
  // for ring stages 0 and 1 only and the first MFMA for W(tile 0) only, with the
  // same in-order counts as in the loop; the rest of the lookahead lands during
  // iteration 0.  K < 768 takes no shortcut.
  auto load_w = [&](WSet<CB>& w, int kt) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int j = 0; j < CB; ++j) load_w_frag(w, kt, kk, j);
    load_w_scales(w, kt);
  };
  dma_x(0);
  if (KT > 1) dma_x(1);
  if (p0 == 0) {
    load_w(wset[0], 0);
    if (KT > 2) dma_x(2);
    if (KT > 1) load_w(wset[1], 1);
  } else {
    load_w(wset[1], 0);
    if (KT > 2) dma_x(2);
    load_w(wset[0], 1);
  }
  if (KT > 2) __builtin_amdgcn_s_waitcnt(vmcnt_imm(kWPerIter + kVmemPerIter));
  else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_barrier");
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < RB; ++i) {
    af0[i] = read_x_frag(0, 0, i);
    af1[i] = read_x_frag(0, 1, i);
  }
  if (p0 == 0) {
#pragma unroll
    for (int i = 0; i < RB; ++i) xsc[0][i] = read_x_scale(0, i);
  } else {
#pragma unroll
    for (int i = 0; i < RB; ++i) xsc[1][i] = read_x_scale(0, i);
  }

  // One K iteration on tile kt with W set w and X scales xs (af0, af1 already
  // hold its issue-0 and issue-1 operands).  Flags say which streams still have
  // work: PFX = tile kt+3 exists (X ring), PFW = tile kt+2 exists (W registers),
  // NEXT = tile kt+1 exists (its first operands and scales are read here).
  // Each slot = MFMA, one LDS read, MFMA, at most one global load (, MFMA): the read
  // sits in the shadow of the first MFMA and the load in the shadow of the second.
#define WUSH_MMA(KK, AF, i, j)                                                                                 \
  {                                                                                                            \
    const v8i A_ = {AF[i][0], AF[i][1], AF[i][2], AF[i][3], 0, 0, 0, 0};                                       \
    const v8i B_ = {w.f[j][KK][0], w.f[j][KK][1], w.f[j][KK][2], w.f[j][KK][3], 0, 0, 0, 0};                   \
    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(B_, A_, acc[i][j], 4, 4, KK, w.s[j], KK, xs[i]); \
  }
#define WUSH_MMA_REST(KK, AF, i)                   \
  if constexpr (CB > 2) {                          \
    WUSH_FENCE                                     \
    WUSH_MMA(KK, AF, i, CB - 1)                    \
  }
#define WUSH_FENCE __builtin_amdgcn_sched_barrier(0);
  auto iteration = [&](int kt, WSet<CB>& w, const int (&xs)[RB], int (&xs_next)[RB], auto pfx_tag, auto pfw_tag,
                       auto next_tag) {
    constexpr bool PFX = decltype(pfx_tag)::value, PFW = decltype(pfw_tag)::value, NEXT = decltype(next_tag)::value;
    // W fragments and scales of tile kt were issued two iterations ago; the last of
    // them (the scales) is followed by exactly the operations of the previous
    // iteration: its ring loads if tile kt+2 exists, its W loads if tile kt+1 exists.
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(PFW ? kVmemPerIter : (NEXT ? kWPerIter : 0)));
    WUSH_FENCE
#pragma unroll
    for (int i = 0; i < RB; ++i) {           // issue 0: X ring refill, operands of issue 2
      WUSH_MMA(0, af0, i, 0)
      const v4i nx_ = read_x_frag(kt, 2, i);
      WUSH_FENCE
      if constexpr (CB > 1) WUSH_MMA(0, af0, i, 1)
      if (PFX && i < 4 * kUB) dma_x_frag(kt + 3, i);
      WUSH_MMA_REST(0, af0, i)
      af0[i] = nx_;
      WUSH_FENCE
    }
#pragma unroll
    for (int i = 0; i < RB; ++i) {           // issue 1: X scales, W fragments of issue 0, operands of issue 3
      WUSH_MMA(1, af1, i, 0)
      const v4i nx_ = read_x_frag(kt, 3, i);
      WUSH_FENCE
      if constexpr (CB > 1) WUSH_MMA(1, af1, i, 1)
      if (PFX && i < kUB) dma_x_scale(kt + 3, i);
      if (PFW && i >= kUB && i < kUB + CB) load_w_frag(w, kt + 2, 0, i - kUB);
      WUSH_MMA_REST(1, af1, i)
      af1[i] = nx_;
      WUSH_FENCE
    }
    // Copies of the last column's issue-3 fragment and scale dword (one register move per slot, by
    // asm so that they are values of their own: the W registers keep their assignment): issue 3
    // multiplies the last column out of these, and its registers can be refilled a pass earlier.
    v4i last_f;
    int last_s;
#pragma unroll
    for (int i = 0; i < RB; ++i) {           // issue 2: W fragments of issue 1, next tile's issue-0 operands
      if (i >= RB - 4) asm volatile("v_mov_b32 %0, %1" : "=v"(last_f[i - (RB - 4)]) : "v"(w.f[CB - 1][3][i - (RB - 4)]));
      if (i == RB - 1) asm volatile("v_mov_b32 %0, %1" : "=v"(last_s) : "v"(w.s[CB - 1]));
      WUSH_MMA(2, af0, i, 0)
      v4i nx_ = af0[i];
      if (NEXT) nx_ = read_x_frag(kt + 1, 0, i);
      WUSH_FENCE
      if constexpr (CB > 1) WUSH_MMA(2, af0, i, 1)
      if (PFW && i < CB) load_w_frag(w, kt + 2, 1, i);
      WUSH_MMA_REST(2, af0, i)
      af0[i] = nx_;
      WUSH_FENCE
    }
    // issue 3, column by column: a column's last fragment and its scale dword are free as soon as its
    // pass is through and are refilled (tile kt+2) in the first slots of the next pass; the last column
    // multiplies out of copies, so that its registers are free from the start of its pass.  Every
    // global load has a slot of its own: a block of loads behind the last MFMA would stall the MFMA
    // pipe for its whole length (some 30 cycles per load).  The last pass also fetches the next tile's
    // issue-1 operands and scales.
#pragma unroll
    for (int j = 0; j < CB; ++j) {
#pragma unroll
      for (int i = 0; i < RB; ++i) {
        {
          const v4i f_ = j == CB - 1 ? last_f : w.f[j][3];
          const int s_ = j == CB - 1 ? last_s : w.s[j];
          const v8i A_ = {af1[i][0], af1[i][1], af1[i][2], af1[i][3], 0, 0, 0, 0};
          const v8i B_ = {f_[0], f_[1], f_[2], f_[3], 0, 0, 0, 0};
          acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(B_, A_, acc[i][j], 4, 4, 3, s_, 3, xs[i]);
        }
        if (NEXT && j == CB - 1) {
          af1[i] = read_x_frag(kt + 1, 1, i);
          xs_next[i] = read_x_scale(kt + 1, i);
        }
        if (PFW) {
          if (j * RB + i < CB) load_w_frag(w, kt + 2, 2, j * RB + i);
          if (j >= 1 && i == 0) load_w_frag(w, kt + 2, 3, j - 1);
          if (j >= 1 && i == 1) load_w_scale(w, kt + 2, j - 1);
          if (j == CB - 1 && i == 2) load_w_frag(w, kt + 2, 3, CB - 1);
          if (j == CB - 1 && i == 3) load_w_scale(w, kt + 2, CB - 1);
        }
        WUSH_FENCE
      }
    }
    // Ring stage kt+2 (this wave's share, issued during iteration kt-1) must have
    // landed before the barrier publishes it; vmcnt retires in order, and since
    // that share the wave issued the W loads of iteration kt-1 and all the
    // memory instructions of this one.
    if (PFX) __builtin_amdgcn_s_waitcnt(vmcnt_imm(kWPerIter + kVmemPerIter));
    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    WUSH_FENCE
    // A bare s_barrier: __syncthreads() carries a workgroup fence for which the
    // compiler drains vmcnt to 0, i.e. it would wait for the loads issued two
    // iterations ahead on every iteration.  The only cross-wave data here are the
    // direct-to-LDS writes, whose arrival the explicit vmcnt above already
    // guarantees.  No "memory" clobber either: the compiler models such an asm as
    // an unknown (flat) access and answers with vmcnt(0) lgkmcnt(0) at the next
    // wait.  The sched_barrier fences keep the LDS reads on their side.
    asm volatile("s_barrier");
  };
  using T = std::true_type;
  using F = std::false_type;
  // Pull the epilogue's kernel arguments into SGPRs now.  A scalar load still
  // pending at the loop entry shares its counter with the LDS reads and can
  // return out of order, for which the compiler answers with lgkmcnt(0) at the
  // loop top, i.e. a full LDS drain on every trip.
  asm volatile("" ::"s"(Y), "s"(ldy), "s"(M), "s"(N), "s"(vec_store));
  int kt = 0;
  const int n_main = KT - 3;                   // iterations with every stream active
  if (n_main > 0 && (n_main & 1)) {            // odd count: one iteration on set 1 first
    iteration(0, wset[1], xsc[1], xsc[0], T{}, T{}, T{});
    kt = 1;
  }
  for (; kt + 3 < KT; kt += 2) {
    iteration(kt, wset[0], xsc[0], xsc[1], T{}, T{}, T{});
    iteration(kt + 1, wset[1], xsc[1], xsc[0], T{}, T{}, T{});
  }
  // drain: KT-3 on set 0, KT-2 on set 1, KT-1 on set 0
  if (KT >= 3) iteration(KT - 3, wset[0], xsc[0], xsc[1], F{}, T{}, T{});
  if (KT >= 2) iteration(KT - 2, wset[1], xsc[1], xsc[0], F{}, F{}, T{});
  iteration(KT - 1, wset[0], xsc[0], xsc[1], F{}, F{}, F{});
#undef WUSH_MMA
#undef WUSH_MMA_REST
#undef WUSH_FENCE
  __builtin_amdgcn_sched_barrier(0);

  // ---- epilogue.  The W fragment is the MFMA's first operand, so a tile of D is
  // (32 output columns) x (32 tokens): lane (r, kh) of MFMA tile (i, j) holds token
  // row 32*i + r, and its accumulator e is output column
  // 32*CB*wave + 32*j + 8*(e/4) + 4*kh + e%4 -- four consecutive columns per e/4.
  if (!OUT_F32 && vec_store) {
    // BF16, 16-byte-aligned rows.  Four consecutive columns = two packed converts =
    // one 8-byte LDS write; a wave-private LDS image of 32 rows x 32*CB columns is
    // read back as 16 bytes per lane so that the stores cover whole row segments
    // (128 or 192 bytes).  Row pitch = segment + 16 B (144 / 208): the 8-byte writes
    // of a wave (pitch 36 / 52 dwords, +2 dwords for the upper lane half) hit every
    // bank 4 times, the minimum.  The ring is free after the last barrier; each wave
    // uses a private double buffer, so no barrier.
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    typedef float v2f __attribute__((ext_vector_type(2)));
    constexpr int kChunks = 4 * CB;                       // 16-byte chunks per row segment
    constexpr int kPitch = 16 * kChunks + 16, kBuf = 32 * kPitch;
    static_assert(4 * 2 * kBuf <= lds_bytes(RB), "transpose buffers must fit in the ring");
    uint8_t* area = smem + wave * (2 * kBuf);
    uint16_t* Yb = reinterpret_cast<uint16_t*>(Y);
#pragma unroll
    for (int i = 0; i < RB; ++i) {
      __builtin_amdgcn_sched_barrier(0);
      uint8_t* buf = area + (i & 1) * kBuf;
#pragma unroll
      for (int j = 0; j < CB; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const v2bf lo = __builtin_convertvector((v2f){acc[i][j][4 * q], acc[i][j][4 * q + 1]}, v2bf);
          const v2bf hi = __builtin_convertvector((v2f){acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]}, v2bf);
          v2u two;
          two[0] = __builtin_bit_cast(uint32_t, lo);
          two[1] = __builtin_bit_cast(uint32_t, hi);
          *reinterpret_cast<v2u*>(buf + r * kPitch + 2 * (32 * j + 8 * q + 4 * kh)) = two;
        }
      }
#pragma unroll
      for (int p = 0; p < 2 * CB; ++p) {                  // 32 rows x kChunks chunks, 64 per round
        const int idx = 64 * p + lane;
        const int row_l = idx / kChunks;
        const int chunk = idx % kChunks;
        const v4i v = *reinterpret_cast<const v4i*>(buf + row_l * kPitch + 16 * chunk);
        const int row = m0 + 32 * i + row_l;
        const int col = n0 + 32 * CB * wave + 8 * chunk;
        // streaming store: the output is not read again by this kernel, and lines that
        // leave the L2 as they are written shorten the write-back at the kernel's end
        if (row < M && col < N) __builtin_nontemporal_store(v, reinterpret_cast<v4i*>(Yb + (int64_t)row * ldy + col));
      }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < RB; ++i) {
#pragma unroll
    for (int j = 0; j < CB; ++j) {
      __builtin_amdgcn_sched_barrier(0);   // one MFMA tile at a time: keeps the epilogue out of scratch
      const int row = m0 + 32 * i + r;
      if (row < M) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int col = n0 + 32 * CB * wave + 32 * j + 8 * (e >> 2) + 4 * kh + (e & 3);
          if (col < N) {
            if (OUT_F32) reinterpret_cast<float*>(Y)[(int64_t)row * ldy + col] = acc[i][j][e];
            else reinterpret_cast<uint16_t*>(Y)[(int64_t)row * ldy + col] = f32_to_bf16_bits(acc[i][j][e]);
          }
        }
      }
    }
  }
}

template <bool OUT_F32, int RB, int CB>
hipError_t launch_shape(const void* Xq, const void* Xs, const void* Wq, const void* Ws, int64_t M, int64_t N, int64_t K,
                        void* Y, int64_t ldy, hipStream_t stream) {
  constexpr int kLds = lds_bytes(RB);
  static DynamicLdsLimit lds_limit;   // per instantiation
  const hipError_t attr = lds_limit.ensure(reinterpret_cast<const void*>(gemm_frag_kernel<OUT_F32, RB, CB>), kLds);
  if (attr != hipSuccess) return attr;
  constexpr int kTM = 32 * RB, kTN = 4 * 32 * CB;
  const int tiles_m = (int)((M + kTM - 1) / kTM), tiles_n = (int)((N + kTN - 1) / kTN);
  dim3 grid((unsigned)(tiles_m * tiles_n)), block(256);
  // 128-bit stores need whole 8-column chunks at 16-byte aligned addresses
  const int vec_store = (N % 8 == 0) && (ldy % 8 == 0) && ((reinterpret_cast<uintptr_t>(Y) & 15) == 0);
  const int w_blocks = (int)((N + 255) / 256 * 8);   // 32-row blocks the packed W buffers hold
  gemm_frag_kernel<OUT_F32, RB, CB><<<grid, block, kLds, stream>>>(
      (const uint8_t*)Xq, (const uint8_t*)Xs, (const uint8_t*)Wq, (const uint8_t*)Ws, (int)M, (int)N, (int)K, Y, ldy,
      tiles_m, tiles_n, vec_store, w_blocks);
  return hipGetLastError();
}

// Estimated duration of the GEMM with tiles of tm x tn, in us: rounds of the CUs times the time one
// tile takes, t_iter per K iteration of 256 plus a fixed part (prologue, epilogue, dispatch).  A partly
// filled last round costs a whole one (workgroups are dispatched as CUs fall free).  The pairs
// (t_iter, fixed) are fits to launches of 8192 tokens on 4096 -> 14336 and 8192 -> 28672 with each
// shape forced: 256 x 256: (1.51, 7.4), 128 x 384: (1.175, 5.1), 128 x 256: (0.8125, 4.1),
// 128 x 128: (0.5125, 0.6; several of its workgroups share a CU and cover each other's fixed part).
// Against the earlier weight "rounds x MFMAs per iteration" this accounts for what small tiles lose
// to their operand traffic (8192 -> 28672, 5120 tokens: 490 us with 256 x 256 tiles, 598 us with
// 128 x 128, which the MFMA count alone put first).
double shape_cost_us(int64_t M, int64_t N, int64_t K, int tm, int tn, double t_iter, double fixed, int cus) {
  const int64_t tiles = ((M + tm - 1) / tm) * ((N + tn - 1) / tn);
  return (double)((tiles + cus - 1) / cus) * (t_iter * (double)(K / 256) + fixed);
}

}  // namespace

hipError_t launch_mxfp4_gemm_frag(const void* Xq, const void* Xs, const void* Wq, const void* Ws,
                                  int64_t M, int64_t N, int64_t K, int out_f32, void* Y, int64_t ldy,
                                  hipStream_t stream) {
  const int cus = device_cu_count();
  // Four instantiations: 256 x 256 (8 x 2 MFMA tiles per wave), 128 x 384 (4 x 3), 128 x 256 (4 x 2)
  // and 128 x 128 (4 x 1).  The cheapest by the estimate above wins, ties go to the larger tile
  // (less operand traffic).  wush_debug_set(WUSH_DEBUG_GEMM_TILE, 0..3) forces one of them.
  const double cost[4] = {shape_cost_us(M, N, K, 256, 256, 1.51, 7.4, cus), shape_cost_us(M, N, K, 128, 384, 1.175, 5.1, cus),
                          shape_cost_us(M, N, K, 128, 256, 0.8125, 4.1, cus), shape_cost_us(M, N, K, 128, 128, 0.5125, 0.6, cus)};
  int shape = 0;
  for (int c = 1; c < 4; ++c)
    if (cost[c] < cost[shape]) shape = c;
  if (const int forced = debug_option(kDbgGemmTile); forced >= 0 && forced <= 3) shape = forced;
  if (shape == 1) {
    if (out_f32) return launch_shape<true, 4, 3>(Xq, Xs, Wq, Ws, M, N, K, Y, ldy, stream);
    return launch_shape<false, 4, 3>(Xq, Xs, Wq, Ws, M, N, K, Y, ldy, stream);
  }
  if (shape == 2) {
    if (out_f32) return launch_shape<true, 4, 2>(Xq, Xs, Wq, Ws, M, N, K, Y, ldy, stream);
    return launch_shape<false, 4, 2>(Xq, Xs, Wq, Ws, M, N, K, Y, ldy, stream);
  }
  if (shape == 3) {
    if (out_f32) return launch_shape<true, 4, 1>(Xq, Xs, Wq, Ws, M, N, K, Y, ldy, stream);
    return launch_shape<false, 4, 1>(Xq, Xs, Wq, Ws, M, N, K, Y, ldy, stream);
  }
  if (out_f32) return launch_shape<true, 8, 2>(Xq, Xs, Wq, Ws, M, N, K, Y, ldy, stream);
  return launch_shape<false, 8, 2>(Xq, Xs, Wq, Ws, M, N, K, Y, ldy, stream);
}

}  // namespace wush
