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
// leaves few CUs idle), K in steps of 64 (= 4 scale groups); each thread converts one X
// row (and one W row) of the next step after the MFMAs of the current one; two LDS
// stages.  On this GPU a SIMD does not overlap VALU issue with MFMA execution (measured:
// n VALU operations between two 32-cycle MFMAs cost 4n cycles more, for one wave per
// SIMD and for two), so the conversion is priced in issue slots and nothing is gained by
// interleaving it; it runs as one block per K step.
#include <stdlib.h>

#include <type_traits>
#include <utility>

#include "nvfp4_layout.hpp"
#include "wush_device.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

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

// Where a row's K steps live: byte offset of step 0 plus a stride per step, for the
// codes (two 16-byte halves, `half` bytes apart) and for the scale dword.  Covers
// the canonical row-major layout and the tiled one (nvfp4_layout.hpp).
struct RowAddr {
  const uint8_t* q;
  const uint8_t* s;
  int q_step, q_half, s_step;
};

__device__ __forceinline__ RowAddr row_addr(const uint8_t* __restrict__ q, const uint8_t* __restrict__ s, int64_t row,
                                            int K, int tiled) {
  RowAddr a;
  if (tiled) {
    const int KT = K >> 6;
    a.q = q + nv_tiled_chunk_offset(row, 0, 0, KT);
    a.s = s + nv_tiled_scale_offset(row, 0, KT);
    a.q_step = 1024; a.q_half = 512; a.s_step = 128;
  } else {
    a.q = q + row * (K / 2);
    a.s = s + row * (K / 16);
    a.q_step = 32; a.q_half = 16; a.s_step = 4;
  }
  return a;
}

__device__ __forceinline__ void load_raw(Raw& r, const RowAddr& a, int kt) {
  const uint8_t* p = a.q + (int64_t)kt * a.q_step;
  r.q[0] = *reinterpret_cast<const v4u*>(p);
  r.q[1] = *reinterpret_cast<const v4u*>(p + a.q_half);
  r.s = *reinterpret_cast<const uint32_t*>(a.s + (int64_t)kt * a.s_step);
}

// Two E4M3 scale bytes (word `HI` of the row's scale dword) -> two FP16 values, by the
// hardware FP8 convert (gfx950 reads FP8 as OCP E4M3); every finite E4M3 value is an
// FP16 normal, so the conversion is exact.
template <bool HI>
__device__ __forceinline__ v2h e4m3x2_to_f16(uint32_t scales) {
  return __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(scales, 1.0f, HI);
}

// Eight codes (one dword, element i in nibble i) times the group scale -> 8 FP16.
__device__ __forceinline__ v4u dequant8(uint32_t w, v2h s) {
  const float one = 1.0f;
  union { v2h h[4]; v4u u; } c;
  c.h[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, one, 0) * s;
  c.h[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, one, 1) * s;
  c.h[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, one, 2) * s;
  c.h[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, one, 3) * s;
  return c.u;
}

// Eight two's-complement INT4 codes times the group scale -> 8 FP16.  A nibble n becomes the
// FP16 number 1024 + (n ^ 8) by OR-ing it into the fraction of 0x6400; subtracting 1032 leaves
// the signed code, exactly; code * scale has at most 3 + 8 significant bits: exact in FP16 too.
__device__ __forceinline__ v4u dequant8_int4(uint32_t w, v2h s) {
  const uint32_t x = w ^ 0x88888888u, y = x >> 4;
  const v2h bias = {(_Float16)1032.0f, (_Float16)1032.0f};
  union { v2h h[4]; v4u u; uint32_t d[4]; } c;
  // (permuted & 0x000F000F) | 0x64006400 as one v_and_or_b32 each (the compiler emits an and and an or)
  const uint32_t mask = 0x000F000Fu, magic = 0x64006400u;
  const uint32_t p0 = __builtin_amdgcn_perm(y, x, 0x0C040C00u), p1 = __builtin_amdgcn_perm(y, x, 0x0C050C01u);
  const uint32_t p2 = __builtin_amdgcn_perm(y, x, 0x0C060C02u), p3 = __builtin_amdgcn_perm(y, x, 0x0C070C03u);
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(c.d[0]) : "v"(p0), "s"(mask), "v"(magic));
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(c.d[1]) : "v"(p1), "s"(mask), "v"(magic));
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(c.d[2]) : "v"(p2), "s"(mask), "v"(magic));
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(c.d[3]) : "v"(p3), "s"(mask), "v"(magic));
#pragma unroll
  for (int i = 0; i < 4; ++i) c.h[i] = (c.h[i] - bias) * s;
  return c.u;
}

constexpr int kNvfp4 = 0, kInt4 = 1;

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
  static constexpr int kOpsPerTask = FMT == kNvfp4 ? 9 : 19;   // micro-operations per 8 codes
  v2h h[4];
  uint32_t x, y, p[4];
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
    else if constexpr (U == 1) c.y = c.x >> 4;
    else if constexpr (U < 6) c.p[U - 2] = __builtin_amdgcn_perm(c.y, c.x, 0x0C040C00u + 0x00010001u * (U - 2));
    else if constexpr (U < 10) {
      uint32_t d;
      const uint32_t mask = 0x000F000Fu, magic = 0x64006400u;
      asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(d) : "v"(c.p[U - 6]), "s"(mask), "v"(magic));
      union { uint32_t u; v2h h; } t;
      t.u = d;
      c.h[U - 6] = t.h;
    } else if constexpr (U < 14) {
      const v2h bias = {(_Float16)1032.0f, (_Float16)1032.0f};
      c.h[U - 10] = c.h[U - 10] - bias;
    } else if constexpr (U < 18) c.h[U - 14] = c.h[U - 14] * s;
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
  if ((ntiles & 7) == 0) id = (id & 7) * (ntiles >> 3) + (id >> 3);
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
  const RowAddr ax = row_addr(Xq, Xs, rowX, K, tiled), aw = row_addr(Wq, Ws, rowW, K, tiled);
  Raw ax_, aw_, bx_, bw_;
  load_raw(ax_, ax, 0);
  load_raw(aw_, aw, 0);
  convert(ax_, aw_, lds);
  load_raw(ax_, ax, min(1, KT - 1));
  load_raw(aw_, aw, min(1, KT - 1));
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
      const int kl = min(kt + 2, KT - 1);
      load_raw(bx_, ax, kl);
      load_raw(bw_, aw, kl);
    }
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

template <bool OUT_F32, int CB, int FMT>
hipError_t launch_shape(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws,
                        const float* tsw, int64_t M, int64_t N, int64_t K, int tiled, void* Y, int64_t ldy,
                        hipStream_t stream) {
  static bool configured = false;  // per instantiation
  if (!configured) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(w4_f16_gemm_kernel<OUT_F32, CB, FMT>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    configured = true;
  }
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
  if (const char* f = getenv("WUSH_NVFP4_WIDTH")) {  // tests: force a tile width (output channels / 64)
    if (f[0] >= '2' && f[0] <= '4' && f[1] == 0) best = f[0] - '0';
  }
#define WUSH_NV_LAUNCH(F32, CB) launch_shape<F32, CB, FMT>(Xq, Xs, tsx, Wq, Ws, tsw, M, N, K, tiled, Y, ldy, stream)
  if (out_f32) return best == 4 ? WUSH_NV_LAUNCH(true, 4) : best == 3 ? WUSH_NV_LAUNCH(true, 3) : WUSH_NV_LAUNCH(true, 2);
  return best == 4 ? WUSH_NV_LAUNCH(false, 4) : best == 3 ? WUSH_NV_LAUNCH(false, 3) : WUSH_NV_LAUNCH(false, 2);
#undef WUSH_NV_LAUNCH
}

}  // namespace

hipError_t launch_nvfp4_gemm(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws,
                             const float* tsw, int64_t M, int64_t N, int64_t K, int out_f32, int tiled, void* Y,
                             int64_t ldy, hipStream_t stream) {
  return launch_w4_f16_gemm<kNvfp4>(Xq, Xs, tsx, Wq, Ws, tsw, M, N, K, out_f32, tiled, Y, ldy, stream);
}

hipError_t launch_int4_gemm(const void* Xq, const void* Xs, const void* Wq, const void* Ws, int64_t M, int64_t N,
                            int64_t K, int out_f32, int tiled, void* Y, int64_t ldy, hipStream_t stream) {
  return launch_w4_f16_gemm<kInt4>(Xq, Xs, nullptr, Wq, Ws, nullptr, M, N, K, out_f32, tiled, Y, ldy, stream);
}

}  // namespace wush
