// GEMMs of the two 4-bit formats without a block-scaled MFMA path, NVFP4 and INT4 (BF16 scale per
// 32; element * scale has at most 3 + 8 significant bits: exact in FP16 as long as the scale lies in
// FP16's normal range), with FP32 accumulation for gfx950.  Written for NVFP4:
//   Y = tsx tsw * deq(Xq, Xs) . deq(Wq, Ws)^T
// (the sum over blocks of the layer forward-pass equation, in the NVFP4 variant
// of the paper's experiments: E2M1 elements, E4M3 scale per 16, FP32 tensor scale).
//
// CDNA4's block-scaled MFMA takes power-of-two (E8M0) scales per 32 elements; an
// E4M3 scale per 16 has no hardware path.  The product element * group-scale,
// however, has at most 2 + 4 significant bits and lies in [2^-10, 2688], so it is
// EXACT in FP16.  The kernel therefore dequantizes while staging: packed codes and
// scale bytes (row-major, or tiled so that a tile's K step is a few contiguous runs:
// a 256-row tile otherwise pulls 16 bytes out of 256 different cache lines per load)
// travel HBM -> registers, become FP16 (hardware fp4 -> f16 convert,
// one packed multiply by the group scale), land in LDS in MFMA operand order, and
// the contraction runs on v_mfma_f32_32x32x16_f16.  Nothing but the FP32
// accumulation order separates the result from the exact one.
//
// Tiling: one workgroup (4 waves, 2 x 2) per 256 x 64*CB output tile (CB = 4, 3 or 2:
// 256, 192 or 128 output channels, chosen per problem so that the last round of tiles
// leaves few CUs idle), K in steps of 64 (= 4 scale groups), two LDS stages.  Two kernels:
//   * w4_f16_gemm_kernel stages both operands in LDS (each thread converts one X row and one
//     W row of the next step); it serves any K;
//   * w4_wreg_gemm_kernel (K a multiple of 128) keeps W out of LDS: every wave converts the W
//     fragments it multiplies in its own registers.
// In both the conversion of the next step is cut into single instructions and dealt out over
// the MFMAs of the current one: with one wave per SIMD the MFMA pipe is busy 32 cycles per
// instruction and a handful of independent vector instructions issue in that shadow for free,
// while anything issued as a block (conversions, register moves, global loads, address
// arithmetic) stalls the pipe for its length.
#include <type_traits>
#include <utility>

#include "nvfp4_layout.hpp"
#include "w4_dequant.hpp"
#include "wush_device.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

constexpr int kBM = 256, kBK = 64;
constexpr int kXBytes = 8 * 256 * 16;            // X part of a stage: [k chunk of 8][256 rows][16 B]
// The W part has the same geometry whatever the tile width (rows past 64*CB are written by the
// threads that have no W row of their own -- a duplicate, never read -- so that the conversion
// stream has no branch in it).
constexpr int kStage = 2 * kXBytes;
constexpr int kLdsBytes = 2 * kStage;            // 128 KiB

struct Raw {
  v4u q[2];    // 64 codes of one row
  uint32_t s;  // their 4 scale bytes
};

// Where a lane finds its row of a tile's packed operand: a uniform 64-bit base (the tile's
// first row, K step 0: scalar registers) plus a 32-bit lane offset, for the codes and for the
// scale dwords; a K step adds a uniform stride.  Covers the canonical row-major layout and the
// tiled one (nvfp4_layout.hpp).  A load then takes its base from scalar registers and no vector
// instruction computes an address.
struct Strides {
  int q_step, q_half, s_step;   // bytes per K step (codes), between a step's two 16-byte halves, per K step (scales)
};
__device__ __forceinline__ Strides layout_strides(int tiled) {
  Strides st = {tiled ? 1024 : 32, tiled ? 512 : 16, tiled ? 128 : 4};
  asm volatile("" : "+s"(st.q_step), "+s"(st.q_half), "+s"(st.s_step));   // plain numbers from here on: one loop, not one per layout
  return st;
}
struct OperandAddr {
  const uint8_t* q0;
  const uint8_t* s0;
  uint32_t oq, os;
};
// row0 = the tile's first row (a multiple of 32), row >= row0 the lane's row, hh = which 16-byte half
// of a K step the code offset points at.
__device__ __forceinline__ OperandAddr operand_addr(const uint8_t* __restrict__ q, const uint8_t* __restrict__ s,
                                                    int64_t row0, int64_t row, int hh, int K, int tiled) {
  OperandAddr a;
  const int KT = K >> 6;
  if (tiled) {
    const int64_t bq = nv_tiled_chunk_offset(row0, 0, 0, KT), bs = nv_tiled_scale_offset(row0, 0, KT);
    a.q0 = q + bq;
    a.s0 = s + bs;
    a.oq = (uint32_t)(nv_tiled_chunk_offset(row, 0, hh, KT) - bq);
    a.os = (uint32_t)(nv_tiled_scale_offset(row, 0, KT) - bs);
  } else {
    a.q0 = q + row0 * (K / 2);
    a.s0 = s + row0 * (K / 16);
    a.oq = (uint32_t)((row - row0) * (K / 2) + hh * 16);
    a.os = (uint32_t)((row - row0) * (K / 16));
  }
  return a;
}
// One load of K step kt.  The empty asm keeps the lane offset apart from the scalar base (otherwise
// the compiler folds both into a 64-bit vector address that it then has to advance per step).
__device__ __forceinline__ v4u load_codes(OperandAddr& a, const Strides& st, int kt, int half) {
  asm volatile("" : "+v"(a.oq));
  return *reinterpret_cast<const v4u*>(a.q0 + ((int64_t)kt * st.q_step + half * st.q_half) + a.oq);
}
__device__ __forceinline__ uint32_t load_scales(OperandAddr& a, const Strides& st, int kt) {
  asm volatile("" : "+v"(a.os));
  return *reinterpret_cast<const uint32_t*>(a.s0 + (int64_t)kt * st.s_step + a.os);
}
// which = 0, 1: the two halves of the row's codes, 2: its scale dword
__device__ __forceinline__ void load_raw_piece(Raw& r, OperandAddr& a, const Strides& st, int kt, int which) {
  if (which < 2) r.q[which] = load_codes(a, st, kt, which);
  else r.s = load_scales(a, st, kt);
}
__device__ __forceinline__ void load_raw(Raw& r, OperandAddr& a, const Strides& st, int kt) {
  r.q[0] = load_codes(a, st, kt, 0);
  r.q[1] = load_codes(a, st, kt, 1);
  r.s = load_scales(a, st, kt);
}


// Group g (16 elements) of a row's K step: two 16-byte LDS chunks, k = 16g + 8hh + 0..7.
// `operand` = the X or W part of a stage, `rows` = its row count.  The row's scale dword holds
// four E4M3 bytes (NVFP4: one per 16 elements) or two BF16 numbers (INT4: one per 32).
template <int FMT>
__device__ __forceinline__ void convert_group(const Raw& r, int g, char* operand, int rows, int row) {
  _Float16 sc;
  if (FMT == kNvfp4) {
    const v2h pair = g < 2 ? e4m3x2_to_f16<false>(r.s) : e4m3x2_to_f16<true>(r.s);
    sc = pair[g & 1];
  } else {
    sc = (_Float16)__uint_as_float(g < 2 ? r.s << 16 : r.s & 0xFFFF0000u);
  }
  const v2h s = {sc, sc};
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {
    const uint32_t w = r.q[g >> 1][(g & 1) * 2 + hh];
    *reinterpret_cast<v4u*>(operand + ((2 * g + hh) * rows + row) * 16) =
        FMT == kNvfp4 ? dequant8(w, s) : dequant8_int4(w, s);
  }
}

// ---------------------------------------------------------------------------
// The K step as a hand-ordered instruction stream.  Measured on this GPU (FP16 MFMA 32x32x16,
// one wave per SIMD): up to about four independent VALU operations issue in the shadow of each
// 32-cycle MFMA for free (8 cost 10-14 cycles more, 16 double the time), while a block of 130
// conversion operations with no MFMA between them simply adds its 500-1000 cycles to the step.
// So the conversion of step kt+1 is cut into micro-operations (per 8 codes: 4 converts, 4
// multiplies, one 16-byte LDS write; more for INT4) and dealt out over the MFMAs of step kt, a
// few per MFMA, converts well ahead of the multiplies that use them; the LDS reads of the next
// group of fragments and the global loads of step kt+2 go into the same slots.  A scheduling
// barrier after every slot keeps the compiler from regrouping them.
// ---------------------------------------------------------------------------
template <int FMT>
struct Conv {
  static constexpr int kOpsPerTask = FMT == kNvfp4 ? 9 : 15;   // micro-operations per 8 codes
  v2h h[4];
  uint32_t x, y;
};

// Micro-operation U of the dword task (8 codes -> one 16-byte LDS chunk).  w = the 8 codes,
// s = the group scale in both halves, dst = where the chunk goes.
template <int FMT, int U>
__device__ __forceinline__ void micro_op(Conv<FMT>& c, uint32_t w, v2h s, char* dst) {
  if constexpr (FMT == kNvfp4) {
    if constexpr (U < 4) c.h[U] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, U);
    else if constexpr (U < 8) c.h[U - 4] = c.h[U - 4] * s;
    else {
      union { v2h h[4]; v4u u; } o;
      o.h[0] = c.h[0]; o.h[1] = c.h[1]; o.h[2] = c.h[2]; o.h[3] = c.h[3];
      *reinterpret_cast<v4u*>(dst) = o.u;
    }
  } else {
    if constexpr (U == 0) c.x = w ^ 0x88888888u;
    else if constexpr (U == 1) c.y = c.x >> 8;
    else if constexpr (U < 6) c.h[U - 2] = int4_pair(U < 4 ? c.x : c.y, (U - 2) & 1);
    else if constexpr (U < 10) c.h[U - 6] = c.h[U - 6] - int4_bias((U - 6) & 1);
    else if constexpr (U < 14) c.h[U - 10] = c.h[U - 10] * s;
    else {
      union { v2h h[4]; v4u u; } o;
      o.h[0] = c.h[0]; o.h[1] = c.h[1]; o.h[2] = c.h[2]; o.h[3] = c.h[3];
      *reinterpret_cast<v4u*>(dst) = o.u;
    }
  }
}

// The four group scales of a row's K step as FP16 (NVFP4: four E4M3 bytes; INT4: two BF16
// numbers, each serving two groups of 16).
template <int FMT>
__device__ __forceinline__ void step_scales(uint32_t sdw, v2h (&sc)[2]) {
  if constexpr (FMT == kNvfp4) {
    sc[0] = e4m3x2_to_f16<false>(sdw);
    sc[1] = e4m3x2_to_f16<true>(sdw);
  } else {
    const _Float16 s0 = (_Float16)__uint_as_float(sdw << 16), s1 = (_Float16)__uint_as_float(sdw & 0xFFFF0000u);
    sc[0] = (v2h){s0, s0};
    sc[1] = (v2h){s1, s1};
  }
}

template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), unrolled at compile time.
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

template <bool OUT_F32, int CB, int FMT>
__global__ __launch_bounds__(256) void w4_f16_gemm_kernel(
    const uint8_t* __restrict__ Xq, const uint8_t* __restrict__ Xs, const float* __restrict__ tsx,
    const uint8_t* __restrict__ Wq, const uint8_t* __restrict__ Ws, const float* __restrict__ tsw,
    void* __restrict__ Yv, int64_t ldy, int M, int N, int K, int tiles_m, int tiles_n, int tiled) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  constexpr int kBN = 64 * CB;         // output channels per tile
  constexpr int kSlots = 16 * CB;      // MFMAs per K step and wave
  constexpr int kGroup = 4 * CB;       // MFMAs per 16-element K group
  // slots that carry conversion work; the workgroup barrier follows, then the first fragments of the next step
  constexpr int kConvSlots = FMT == kNvfp4 ? 12 * CB : 16 * CB - 4;
  constexpr int kOps = Conv<FMT>::kOpsPerTask;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, h = lane >> 5;

  // Tile order: workgroups that run on one XCD (ids congruent mod 8) get a contiguous
  // run of tiles, M fastest, so that they share W tiles in that XCD's L2.
  const int ntiles = tiles_m * tiles_n;
  int id = blockIdx.x;
  id = xcd_contiguous_id(id, ntiles);
  const int tm = id % tiles_m, tn = id / tiles_m;
  const int m0 = tm * kBM, n0 = tn * kBN;

  const int64_t rowX = min(m0 + tid, M - 1);  // rows past the end re-read the last valid row
  const int64_t rowW = min(n0 + min(tid, kBN - 1), N - 1);   // threads past the tile's W rows repeat its last row
  const int KT = K / kBK;

  auto convert = [&](const Raw& x, const Raw& w, char* stage) {
#pragma unroll
    for (int g = 0; g < 4; ++g) convert_group<FMT>(x, g, stage, 256, tid);
#pragma unroll
    for (int g = 0; g < 4; ++g) convert_group<FMT>(w, g, stage + kXBytes, 256, tid);
  };

  // Packed operands in flight: (ax_, aw_) = step kt+1, converted during step kt; (bx_, bw_) = step
  // kt+2, loaded at the start of step kt.  Step numbers are clamped (surplus loads re-read the last step).
  const Strides st = layout_strides(tiled);
  OperandAddr ax = operand_addr(Xq, Xs, m0, rowX, 0, K, tiled), aw = operand_addr(Wq, Ws, n0, rowW, 0, K, tiled);
  Raw ax_, aw_, bx_, bw_;
  load_raw(ax_, ax, st, 0);
  load_raw(aw_, aw, st, 0);
  convert(ax_, aw_, lds);
  load_raw(ax_, ax, st, min(1, KT - 1));
  load_raw(aw_, aw, st, min(1, KT - 1));
  __syncthreads();

  v16f acc[4][CB];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < CB; ++j) acc[i][j] = (v16f){0};

  // Fragment registers of two K groups: group g of a step uses set g & 1.
  v8h fa[2][4], fb[2][CB];
  const int a_off = (h * 256 + wm * 128 + l32) * 16;                          // + 2g chunks, + 32 i rows
  const int b_off = kXBytes + (h * 256 + wn * (32 * CB) + l32) * 16;
  auto read_frag = [&](const char* stage, int g, int r, int set) {            // r: 0..3 = A rows, 4.. = B rows
    if (r < 4) fa[set][r] = *reinterpret_cast<const v8h*>(stage + a_off + (2 * g * 256 + 32 * r) * 16);
    else fb[set][r - 4] = *reinterpret_cast<const v8h*>(stage + b_off + (2 * g * 256 + 32 * (r - 4)) * 16);
  };
#pragma unroll
  for (int r = 0; r < 4 + CB; ++r) read_frag(lds, 0, r, 0);

  // One K step.  NEXT: another step follows (convert it, synchronize, fetch its first fragments).
  auto step = [&](int kt, auto next_tag) {
    constexpr bool NEXT = decltype(next_tag)::value;
    const char* cur = lds + (kt & 1) * kStage;
    char* nxt = lds + ((kt + 1) & 1) * kStage;
    char* xdst = nxt + tid * 16;                 // + chunk * 256 rows * 16
    char* wdst = nxt + kXBytes + tid * 16;
    Conv<FMT> cv;
    v2h sx[2], sw[2];
    if (NEXT) {
      step_scales<FMT>(ax_.s, sx);
      step_scales<FMT>(aw_.s, sw);
    }
    const int kl = min(kt + 2, KT - 1);
    __builtin_amdgcn_sched_barrier(0);
    static_for<kSlots>([&](auto slot) {
      constexpr int S = decltype(slot)::value;
      constexpr int g = S / kGroup, idx = S % kGroup, i = idx / CB, j = idx % CB;
      if (NEXT && S == kConvSlots) __syncthreads();   // every conversion write of this step is behind us
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[g & 1][i], fb[g & 1][j], acc[i][j], 0, 0, 0);
      // fragments of the next group: one LDS read per slot from the second slot of the group on
      if constexpr (g < 3) {
        if constexpr (idx >= 1 && idx - 1 < 4 + CB) read_frag(cur, g + 1, idx - 1, (g + 1) & 1);
      }
      if constexpr (NEXT && S >= kConvSlots) {
        // behind the barrier: the first fragments of the next step, spread over the remaining slots
        constexpr int left = kSlots - kConvSlots, r0 = (S - kConvSlots) * (4 + CB) / left,
                      r1 = (S - kConvSlots + 1) * (4 + CB) / left;
        static_for<r1 - r0>([&](auto q) { read_frag(nxt, 0, r0 + decltype(q)::value, 0); });
      }
      // the six loads of step kt+2, one per slot (a load costs its slot about 30 cycles; six in a row
      // stall the MFMA pipe for all of them): the last two slots of the groups 0 to 2
      if constexpr (NEXT && g < 3 && idx >= kGroup - 2) {
        constexpr int piece = 2 * g + (idx - (kGroup - 2));
        if constexpr (piece < 3) load_raw_piece(bx_, ax, st, kl, piece);
        else load_raw_piece(bw_, aw, st, kl, piece - 3);
      }
      // conversion micro-operations of this slot: 8 X tasks, then 8 W tasks
      if constexpr (NEXT && S < kConvSlots) {
        constexpr int total = 16 * kOps, u0 = S * total / kConvSlots, u1 = (S + 1) * total / kConvSlots;
        static_for<u1 - u0>([&](auto q) {
          constexpr int u = u0 + decltype(q)::value, task = u / kOps, op = u % kOps, d = task & 7;
          if constexpr (task < 8) {
            micro_op<FMT, op>(cv, ax_.q[d >> 2][d & 3], (v2h){sx[d >> 2][(d >> 1) & 1], sx[d >> 2][(d >> 1) & 1]},
                              xdst + d * 256 * 16);
          } else {
            micro_op<FMT, op>(cv, aw_.q[d >> 2][d & 3], (v2h){sw[d >> 2][(d >> 1) & 1], sw[d >> 2][(d >> 1) & 1]},
                              wdst + d * 256 * 16);
          }
        });
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    if (NEXT) {
      ax_ = bx_;
      aw_ = bw_;
    }
  };

  for (int kt = 0; kt + 1 < KT; ++kt) step(kt, std::true_type{});
  step(KT - 1, std::false_type{});

  const float scale = FMT == kNvfp4 ? *tsx * *tsw : 1.0f;   // INT4 has no tensor scales (null pointers)
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int j = 0; j < CB; ++j) {
      const int n = n0 + wn * (32 * CB) + 32 * j + l32;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 128 + 32 * i + 8 * (r >> 2) + 4 * h + (r & 3);
        if (m < M && n < N) {
          const float v = acc[i][j][r] * scale;
          if (OUT_F32) reinterpret_cast<float*>(Yv)[(int64_t)m * ldy + n] = v;
          else reinterpret_cast<uint16_t*>(Yv)[(int64_t)m * ldy + n] = f32_to_bf16_bits(v);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// K a multiple of 128: the W operand goes straight into registers.  Every wave loads the
// packed W fragments it multiplies by itself and converts them in registers (the two waves that
// share the columns each do it); only X passes through LDS.  The order of the 16 k of an MFMA is
// free as long as both operands agree: MFMA group g of a K step takes, in lane half h, the eight
// codes of dword 4h+g of the row's 32 bytes, so the four groups of a lane are ONE 16-byte load
// and its scales are bytes 2h, 2h+1 of the row's scale dword (NVFP4: two E4M3 bytes, one per two
// groups; INT4: the one BF16 number of its 32 codes).  Against the staged kernel: half the LDS
// traffic and half the barriers' work for 40 % more conversion arithmetic, which costs nothing as
// long as it sits in the shadow of the MFMAs.
//
// What the slots of a K step carry besides their MFMA (measured: arithmetic dealt out like this is
// free, a global load costs its slot about 30 cycles, so there is one per slot at most, with a
// scalar base and a 32-bit lane offset; a block of loads or register moves stalls the MFMA pipe
// for its whole length, hence two K steps per loop trip with the register sets swapping roles
// instead of being copied):
//   every slot        two (INT4: three or four) conversion operations of the W fragments of the next group
//   group 0           the three loads of X for step kt+2        (its register set is free)
//   group 1           the W scale dwords for step kt+2          (consumed in group 3 of step kt-1)
//   group 2           the W codes for step kt+2, fragment by fragment as its last group is through
//   slots < 16 CB - 4 the conversion of X for step kt+1 into the other LDS stage
//   then the workgroup barrier and the first four A fragments of step kt+1
// ---------------------------------------------------------------------------

// Room a slot of the register-W kernel has for X conversion work, in instructions: about six issue
// in the shadow of one MFMA; the slot's own fragment read, W conversion pair, scale conversion and
// global load (which costs several) come off that.
template <int CB, int FMT>
constexpr int wreg_slot_room(int S) {
  constexpr int kRoom = FMT == kNvfp4 ? 6 : 7, kLoadCost = 3;
  const int kGroup = 4 * CB, g = S / kGroup, idx = S % kGroup;
  int used = FMT == kNvfp4 ? 2 : 4;                          // the W conversion operations
  if (g < 3 && idx >= 1 && idx <= 4) used += 1;              // A fragment read
  if (g == 3 && idx < CB) used += 2;                         // W scale pair: shift and convert
  if (g == 0 && idx >= kGroup - 3) used += kLoadCost;                // global loads
  if (g == 1 && idx >= kGroup - CB) used += kLoadCost;
  if (g == 2 && (idx & 3) == 3) used += kLoadCost;
  return used >= kRoom ? 0 : kRoom - used;
}
// Conversion operations of X dealt to the slots before `S`, out of `total`, in proportion to the room.
template <int CB, int FMT>
constexpr int wreg_x_ops_before(int S, int total, int conv_slots) {
  int all = 0, before = 0;
  for (int t = 0; t < conv_slots; ++t) {
    all += wreg_slot_room<CB, FMT>(t);
    if (t < S) before += wreg_slot_room<CB, FMT>(t);
  }
  return (int)((long long)total * before / all);
}
struct RawW {
  v4u q;       // the lane's 32 codes of one row's K step (dwords 4h .. 4h+3)
  uint32_t s;  // the row's 4 scale bytes
};
union Frag {
  v2h h[4];
  v4u u;
  v8h v;
};

// Conversion of a W fragment (8 codes of one lane -> 8 FP16 in registers) as micro-operations.
template <int FMT>
struct ConvW {
  static constexpr int kOps = FMT == kNvfp4 ? 8 : 14;
  uint32_t x, y;
};
template <int FMT, int U>
__device__ __forceinline__ void w_micro_op(ConvW<FMT>& c, uint32_t w, v2h s, Frag& f) {
  if constexpr (FMT == kNvfp4) {
    if constexpr (U < 4) f.h[U] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, U);
    else f.h[U - 4] = f.h[U - 4] * s;
  } else {
    if constexpr (U == 0) c.x = w ^ 0x88888888u;
    else if constexpr (U == 1) c.y = c.x >> 8;
    else if constexpr (U < 6) f.h[U - 2] = int4_pair(U < 4 ? c.x : c.y, (U - 2) & 1);
    else if constexpr (U < 10) f.h[U - 6] = f.h[U - 6] - int4_bias((U - 6) & 1);
    else f.h[U - 10] = f.h[U - 10] * s;
  }
}
template <bool OUT_F32, int CB, int FMT>
__global__ __launch_bounds__(256) void w4_wreg_gemm_kernel(
    const uint8_t* __restrict__ Xq, const uint8_t* __restrict__ Xs, const float* __restrict__ tsx,
    const uint8_t* __restrict__ Wq, const uint8_t* __restrict__ Ws, const float* __restrict__ tsw,
    void* __restrict__ Yv, int64_t ldy, int M, int N, int K, int tiles_m, int tiles_n, int tiled) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  constexpr int kBN = 64 * CB;
  constexpr int kSlots = 16 * CB, kGroup = 4 * CB;
  constexpr int kConvSlots = 16 * CB - 4;
  constexpr int kXSlots = (FMT == kNvfp4 && CB == 4) ? 48 : 16 * CB - 4;   // slots that carry X conversion work (measured)
  constexpr int kOps = Conv<FMT>::kOpsPerTask, kWOps = ConvW<FMT>::kOps;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, h = lane >> 5;

  const int ntiles = tiles_m * tiles_n;
  int id = blockIdx.x;
  id = xcd_contiguous_id(id, ntiles);
  const int tm = id % tiles_m, tn = id / tiles_m;
  const int m0 = tm * kBM, n0 = tn * kBN;
  const int KT = K / kBK;   // even

  const Strides st = layout_strides(tiled);
  OperandAddr ax = operand_addr(Xq, Xs, m0, min(m0 + tid, M - 1), 0, K, tiled);   // rows past the end re-read the last valid row
  // W fragment j of this wave: rows n0 + 32 CB wn + 32 j + l32; lane half h takes the 16-byte half h of the K step
  OperandAddr aw[CB];
#pragma unroll
  for (int j = 0; j < CB; ++j) aw[j] = operand_addr(Wq, Ws, n0, min(n0 + wn * (32 * CB) + 32 * j + l32, N - 1), h, K, tiled);
  const uint32_t ssel = 0x05040C0Cu + 0x02020000u * h;
  auto load_x = [&](Raw& r, int kt, int which) { load_raw_piece(r, ax, st, kt, which); };
  auto load_wq = [&](RawW& r, int kt, int j) { r.q = load_codes(aw[j], st, kt, 0); };
  auto load_ws = [&](RawW& r, int kt, int j) { r.s = load_scales(aw[j], st, kt); };

  Raw xr[2];                  // X of step kt+1 lives in xr[(kt+1) & 1] during step kt; the other set receives step kt+2
  RawW wr[2][CB];             // W of step kt in wr[kt & 1]; refilled with step kt+2 as its groups are converted
  v2h wsc[2][CB];             // their scales as FP16 pairs: [group >> 1]
  ConvW<FMT> cw;
  Frag fb[2][CB];
  v8h fa[2][4];

#pragma unroll
  for (int w = 0; w < 3; ++w) load_x(xr[0], 0, w);
#pragma unroll
  for (int j = 0; j < CB; ++j) {
    load_wq(wr[0][j], 0, j);
    load_ws(wr[0][j], 0, j);
  }
#pragma unroll
  for (int j = 0; j < CB; ++j) {
    load_wq(wr[1][j], 1, j);
    load_ws(wr[1][j], 1, j);
  }
#pragma unroll
  for (int g = 0; g < 4; ++g) convert_group<FMT>(xr[0], g, lds, 256, tid);
#pragma unroll
  for (int w = 0; w < 3; ++w) load_x(xr[1], 1, w);
#pragma unroll
  for (int j = 0; j < CB; ++j) {
    wsc[0][j] = w_step_scales<FMT>(wr[0][j].s, h, ssel);
    const v2h s = {wsc[0][j][0], wsc[0][j][0]};
    fb[0][j].u = FMT == kNvfp4 ? dequant8(wr[0][j].q[0], s) : dequant8_int4(wr[0][j].q[0], s);
  }
  __syncthreads();

  v16f acc[4][CB];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < CB; ++j) {
      acc[i][j] = (v16f){0};
      asm volatile("" : "+a"(acc[i][j]));   // pins the accumulators to their registers from here to the epilogue
    }

  // A fragment of MFMA group g, lane half h: LDS chunk 4h + g (the dword order W is loaded in)
  const int a_off = (4 * h * 256 + wm * 128 + l32) * 16;
  auto read_frag = [&](const char* stage, int g, int r, int set) {
    fa[set][r] = *reinterpret_cast<const v8h*>(stage + a_off + (g * 256 + 32 * r) * 16);
  };
#pragma unroll
  for (int r = 0; r < 4; ++r) read_frag(lds, 0, r, 0);

  // One K step of parity P = kt & 1 (LDS stage and register sets are compile-time choices).  Every
  // step prepares a successor; behind the last one that is the last step again (clamped loads),
  // converted into a stage and a fragment set nobody reads.
  auto step = [&](int kt, auto parity) {
    constexpr int P = decltype(parity)::value, Q = P ^ 1;
    const char* cur = lds + P * kXBytes;
    char* nxt = lds + Q * kXBytes;
    char* xdst = nxt + tid * 16;
    Conv<FMT> cv;
    v2h sx[2];
    step_scales<FMT>(xr[Q].s, sx);
    const int kl = min(kt + 2, KT - 1);   // the step the free register sets are refilled with
    __builtin_amdgcn_sched_barrier(0);
    static_for<kSlots>([&](auto slot) {
      constexpr int S = decltype(slot)::value;
      constexpr int g = S / kGroup, idx = S % kGroup, i = idx / CB, j = idx % CB;
      if (S == kConvSlots) __syncthreads();
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[g & 1][i], fb[g & 1][j].v, acc[i][j], 0, 0, 0);
      if constexpr (g < 3) {
        if constexpr (idx >= 1 && idx <= 4) read_frag(cur, g + 1, idx - 1, (g + 1) & 1);
      }
      if constexpr (S >= kConvSlots) read_frag(nxt, 0, S - kConvSlots, 0);
      // W fragments of the next group (group 0 of the next step behind group 3): a fragment's
      // operations spread over four slots
      {
        constexpr int tg = (g + 1) & 3, set = (g + 1) & 1, R = g == 3 ? Q : P;
        if constexpr (g == 3 && idx < CB) wsc[Q][idx] = w_step_scales<FMT>(wr[Q][idx].s, h, ssel);
        constexpr int u0 = idx * kWOps / 4, u1 = (idx + 1) * kWOps / 4;
        static_for<u1 - u0>([&](auto q) {
          constexpr int u = u0 + decltype(q)::value, task = u / kWOps, op = u % kWOps;
          const v2h& sp = wsc[R][task];
          w_micro_op<FMT, op>(cw, wr[R][task].q[tg], (v2h){sp[tg >> 1], sp[tg >> 1]}, fb[set][task]);
        });
      }
      // refills, one load per slot, each once its registers are free
      if constexpr (g == 0 && idx >= kGroup - 3) load_x(xr[P], kl, idx - (kGroup - 3));
      if constexpr (g == 1 && idx >= kGroup - CB) load_ws(wr[P][idx - (kGroup - CB)], kl, idx - (kGroup - CB));
      if constexpr (g == 2 && (idx & 3) == 3) load_wq(wr[P][idx >> 2], kl, idx >> 2);
      if constexpr (S < kXSlots) {
        constexpr int total = 8 * kOps, u0 = wreg_x_ops_before<CB, FMT>(S, total, kXSlots),
                      u1 = wreg_x_ops_before<CB, FMT>(S + 1, total, kXSlots);
        static_for<u1 - u0>([&](auto q) {
          constexpr int u = u0 + decltype(q)::value, d = u / kOps, op = u % kOps;
          micro_op<FMT, op>(cv, xr[Q].q[d >> 2][d & 3], (v2h){sx[d >> 2][(d >> 1) & 1], sx[d >> 2][(d >> 1) & 1]},
                            xdst + d * 256 * 16);
        });
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };

#pragma clang loop unroll(disable)
  for (int kt = 0; kt < KT; kt += 2) {
    step(kt, std::integral_constant<int, 0>{});
    step(kt + 1, std::integral_constant<int, 1>{});
  }

  const float scale = FMT == kNvfp4 ? *tsx * *tsw : 1.0f;   // INT4 has no tensor scales (null pointers)
  // Output coordinates from a fresh copy of the thread index: nothing of the prologue's index
  // arithmetic has to stay in registers across the loop.
  int te = threadIdx.x;
  asm volatile("" : "+v"(te));
  const int e_row = m0 + (te >> 7) * 128 + 4 * ((te >> 5) & 1), e_col = n0 + ((te >> 6) & 1) * (32 * CB) + (te & 31);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int j = 0; j < CB; ++j) {
      const int n = e_col + 32 * j;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = e_row + 32 * i + 8 * (r >> 2) + (r & 3);
        if (m < M && n < N) {
          const float v = acc[i][j][r] * scale;
          if (OUT_F32) reinterpret_cast<float*>(Yv)[(int64_t)m * ldy + n] = v;
          else reinterpret_cast<uint16_t*>(Yv)[(int64_t)m * ldy + n] = f32_to_bf16_bits(v);
        }
      }
      __builtin_amdgcn_sched_barrier(0);   // one 32 x 32 block at a time: the accumulators leave their registers block by block
    }
  }
}

template <bool OUT_F32, int CB, int FMT>
hipError_t launch_wreg(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws,
                       const float* tsw, int64_t M, int64_t N, int64_t K, int tiled, void* Y, int64_t ldy,
                       hipStream_t stream) {
  static DynamicLdsLimit lds_limit;   // per instantiation
  const hipError_t e = lds_limit.ensure(reinterpret_cast<const void*>(w4_wreg_gemm_kernel<OUT_F32, CB, FMT>), 2 * kXBytes);
  if (e != hipSuccess) return e;
  const int tiles_m = (int)((M + kBM - 1) / kBM), tiles_n = (int)((N + 64 * CB - 1) / (64 * CB));
  w4_wreg_gemm_kernel<OUT_F32, CB, FMT><<<dim3((unsigned)(tiles_m * tiles_n)), dim3(256), 2 * kXBytes, stream>>>(
      (const uint8_t*)Xq, (const uint8_t*)Xs, tsx, (const uint8_t*)Wq, (const uint8_t*)Ws, tsw, Y, ldy, (int)M, (int)N,
      (int)K, tiles_m, tiles_n, tiled);
  return hipGetLastError();
}

template <bool OUT_F32, int CB, int FMT>
hipError_t launch_shape(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws,
                        const float* tsw, int64_t M, int64_t N, int64_t K, int tiled, void* Y, int64_t ldy,
                        hipStream_t stream) {
  static DynamicLdsLimit lds_limit;   // per instantiation
  const hipError_t e = lds_limit.ensure(reinterpret_cast<const void*>(w4_f16_gemm_kernel<OUT_F32, CB, FMT>), kLdsBytes);
  if (e != hipSuccess) return e;
  const int tiles_m = (int)((M + kBM - 1) / kBM), tiles_n = (int)((N + 64 * CB - 1) / (64 * CB));
  w4_f16_gemm_kernel<OUT_F32, CB, FMT><<<dim3((unsigned)(tiles_m * tiles_n)), dim3(256), kLdsBytes, stream>>>(
      (const uint8_t*)Xq, (const uint8_t*)Xs, tsx, (const uint8_t*)Wq, (const uint8_t*)Ws, tsw, Y, ldy, (int)M, (int)N,
      (int)K, tiles_m, tiles_n, tiled);
  return hipGetLastError();
}

// Cost of a tile width in issue cycles per K step and SIMD, times the number of rounds the
// tiles take on `cus` CUs: 16*CB MFMAs of 32 cycles plus about 150 conversion / LDS slots of 4.
int64_t width_cost(int64_t M, int64_t N, int CB, int cus) {
  const int64_t tiles = ((M + kBM - 1) / kBM) * ((N + 64 * CB - 1) / (64 * CB));
  return ((tiles + cus - 1) / cus) * (512 * CB + 600);
}

}  // namespace

namespace {

template <int FMT>
hipError_t launch_w4_f16_gemm(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws,
                              const float* tsw, int64_t M, int64_t N, int64_t K, int out_f32, int tiled, void* Y,
                              int64_t ldy, hipStream_t stream) {
  const int cus = device_cu_count();
  int best = 4;
  for (int cb = 3; cb >= 2; --cb)
    if (width_cost(M, N, cb, cus) < width_cost(M, N, best, cus)) best = cb;   // ties keep the wider tile
  if (const int forced = debug_option(kDbgW4Width); forced >= 2 && forced <= 4) best = forced;   // tests: force a tile width
  if (K % 128 == 0) {   // an even number of K steps: W in registers
#define WUSH_WR_LAUNCH(F32, CB) launch_wreg<F32, CB, FMT>(Xq, Xs, tsx, Wq, Ws, tsw, M, N, K, tiled, Y, ldy, stream)
    if (out_f32) return best == 4 ? WUSH_WR_LAUNCH(true, 4) : best == 3 ? WUSH_WR_LAUNCH(true, 3) : WUSH_WR_LAUNCH(true, 2);
    return best == 4 ? WUSH_WR_LAUNCH(false, 4) : best == 3 ? WUSH_WR_LAUNCH(false, 3) : WUSH_WR_LAUNCH(false, 2);
#undef WUSH_WR_LAUNCH
  }
#define WUSH_NV_LAUNCH(F32, CB) launch_shape<F32, CB, FMT>(Xq, Xs, tsx, Wq, Ws, tsw, M, N, K, tiled, Y, ldy, stream)
  if (out_f32) return best == 4 ? WUSH_NV_LAUNCH(true, 4) : best == 3 ? WUSH_NV_LAUNCH(true, 3) : WUSH_NV_LAUNCH(true, 2);
  return best == 4 ? WUSH_NV_LAUNCH(false, 4) : best == 3 ? WUSH_NV_LAUNCH(false, 3) : WUSH_NV_LAUNCH(false, 2);
#undef WUSH_NV_LAUNCH
}

}  // namespace

// Up to 128 tokens the layer is bound by reading the weights once: the weight-streaming kernel of
// w4_gemm_skinny.hip takes over (tiled layout only; the switch kDbgW4Skinny forces either kernel).
static bool w4_streaming(int64_t M, int tiled) {
  if (!tiled || M > 128) return false;
  const int forced = debug_option(kDbgW4Skinny);
  return forced >= 0 ? forced >= 1 : true;   // 1, 2: either schedule of the streaming kernel
}

hipError_t launch_nvfp4_gemm(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws,
                             const float* tsw, int64_t M, int64_t N, int64_t K, int out_f32, int tiled, void* Y,
                             int64_t ldy, hipStream_t stream) {
  if (w4_streaming(M, tiled)) return launch_nvfp4_gemm_skinny(Xq, Xs, tsx, Wq, Ws, tsw, M, N, K, out_f32, Y, ldy, stream);
  return launch_w4_f16_gemm<kNvfp4>(Xq, Xs, tsx, Wq, Ws, tsw, M, N, K, out_f32, tiled, Y, ldy, stream);
}

hipError_t launch_int4_gemm(const void* Xq, const void* Xs, const void* Wq, const void* Ws, int64_t M, int64_t N,
                            int64_t K, int out_f32, int tiled, void* Y, int64_t ldy, hipStream_t stream) {
  if (w4_streaming(M, tiled)) return launch_int4_gemm_skinny(Xq, Xs, Wq, Ws, M, N, K, out_f32, Y, ldy, stream);
  return launch_w4_f16_gemm<kInt4>(Xq, Xs, nullptr, Wq, Ws, nullptr, M, N, K, out_f32, tiled, Y, ldy, stream);
}

}  // namespace wush
