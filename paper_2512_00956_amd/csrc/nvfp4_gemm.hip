// NVFP4 x NVFP4 GEMM with FP32 accumulation for gfx950:
//   Y = tsx tsw * deq(Xq, Xs) . deq(Wq, Ws)^T
// (the sum over blocks of the layer forward-pass equation, in the NVFP4 variant
// of the paper's experiments: E2M1 elements, E4M3 scale per 16, FP32 tensor scale).
//
// CDNA4's block-scaled MFMA takes power-of-two (E8M0) scales per 32 elements; an
// E4M3 scale per 16 has no hardware path.  The product element * group-scale,
// however, has at most 2 + 4 significant bits and lies in [2^-10, 2688], so it is
// EXACT in FP16.  The kernel therefore dequantizes while staging: packed codes and
// scale bytes travel HBM -> registers, become FP16 (hardware fp4 -> f16 convert,
// one packed multiply by the group scale), land in LDS in MFMA operand order, and
// the contraction runs on v_mfma_f32_32x32x16_f16.  Nothing but the FP32
// accumulation order separates the result from the exact one.
//
// Tiling: one workgroup (4 waves, 2 x 2) per 256 x 256 output tile, K in steps of
// 64 (= 4 scale groups); each thread converts one X row and one W row of the step
// (interleaved with the MFMAs of the previous step); two LDS stages (2 x 64 KiB),
// two register stages for the packed loads.
#include "wush_device.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kOperandBytes = 8 * 256 * 16;      // [k chunk of 8][row][16 B]
constexpr int kStageBytes = 2 * kOperandBytes;   // X part, then W part
constexpr int kLdsBytes = 2 * kStageBytes;       // 128 KiB

struct Raw {
  v4u q[2];    // 64 codes of one row
  uint32_t s;  // their 4 scale bytes
};

__device__ __forceinline__ void load_raw(Raw& r, const uint8_t* __restrict__ q, const uint8_t* __restrict__ s,
                                         int64_t row, int K, int kt) {
  const uint8_t* p = q + row * (K / 2) + kt * 32;
  r.q[0] = *reinterpret_cast<const v4u*>(p);
  r.q[1] = *reinterpret_cast<const v4u*>(p + 16);
  r.s = *reinterpret_cast<const uint32_t*>(s + row * (K / 16) + kt * 4);
}

// E4M3 byte (non-negative, finite) -> FP16; every such value is an FP16 normal.
__device__ __forceinline__ _Float16 e4m3_to_f16(uint32_t byte) {
  const float f = byte < 8 ? (float)byte * 0.001953125f
                           : __uint_as_float(((byte >> 3) + 120u) << 23 | (byte & 7u) << 20);
  return (_Float16)f;
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

// Group g (16 elements) of a row's K step: two 16-byte LDS chunks, k = 16g + 8hh + 0..7.
__device__ __forceinline__ void convert_group(const Raw& r, int g, char* operand, int row) {
  const _Float16 sc = e4m3_to_f16((r.s >> (8 * g)) & 0xFFu);
  const v2h s = {sc, sc};
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {
    const uint32_t w = r.q[g >> 1][(g & 1) * 2 + hh];
    *reinterpret_cast<v4u*>(operand + ((2 * g + hh) * 256 + row) * 16) = dequant8(w, s);
  }
}

template <bool OUT_F32>
__global__ __launch_bounds__(256) void nvfp4_gemm_kernel(
    const uint8_t* __restrict__ Xq, const uint8_t* __restrict__ Xs, const float* __restrict__ tsx,
    const uint8_t* __restrict__ Wq, const uint8_t* __restrict__ Ws, const float* __restrict__ tsw,
    void* __restrict__ Yv, int64_t ldy, int M, int N, int K, int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
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
  const int64_t rowW = min(n0 + tid, N - 1);
  const int KT = K / kBK;

  Raw rx[2], rw[2];
  load_raw(rx[0], Xq, Xs, rowX, K, 0);
  load_raw(rw[0], Wq, Ws, rowW, K, 0);
  if (KT > 1) {
    load_raw(rx[1], Xq, Xs, rowX, K, 1);
    load_raw(rw[1], Wq, Ws, rowW, K, 1);
  }
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    convert_group(rx[0], g, lds, tid);
    convert_group(rw[0], g, lds + kOperandBytes, tid);
  }
  if (KT > 2) {
    load_raw(rx[0], Xq, Xs, rowX, K, 2);
    load_raw(rw[0], Wq, Ws, rowW, K, 2);
  }
  __syncthreads();

  v16f acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = (v16f){0};

  // One K step: MFMAs on stage `cur`; meanwhile convert step kt+1 (registers set
  // (kt+1)&1) into the other stage and refill that register set with step kt+3.
  auto step = [&](int kt, Raw& nx, Raw& nw) {
    const char* cur = lds + (kt & 1) * kStageBytes;
    char* nxt = lds + ((kt + 1) & 1) * kStageBytes;
    const bool have_next = kt + 1 < KT;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      v8h a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        a[i] = *reinterpret_cast<const v8h*>(cur + ((2 * g + h) * 256 + wm * 128 + 32 * i + l32) * 16);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        b[j] = *reinterpret_cast<const v8h*>(cur + kOperandBytes + ((2 * g + h) * 256 + wn * 128 + 32 * j + l32) * 16);
      if (have_next) {
        convert_group(nx, g, nxt, tid);
        convert_group(nw, g, nxt + kOperandBytes, tid);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 3 < KT) {
      load_raw(nx, Xq, Xs, rowX, K, kt + 3);
      load_raw(nw, Wq, Ws, rowW, K, kt + 3);
    }
    __syncthreads();
  };

  int kt = 0;
  for (; kt + 1 < KT; kt += 2) {
    step(kt, rx[1], rw[1]);
    step(kt + 1, rx[0], rw[0]);
  }
  if (kt < KT) step(kt, rx[1], rw[1]);

  const float scale = *tsx * *tsw;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + wn * 128 + 32 * j + l32;
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

}  // namespace

hipError_t launch_nvfp4_gemm(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws,
                             const float* tsw, int64_t M, int64_t N, int64_t K, int out_f32, void* Y, int64_t ldy,
                             hipStream_t stream) {
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(nvfp4_gemm_kernel<false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(nvfp4_gemm_kernel<true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles_m = (int)((M + kBM - 1) / kBM), tiles_n = (int)((N + kBN - 1) / kBN);
  const dim3 grid((unsigned)(tiles_m * tiles_n)), block(256);
  if (out_f32)
    nvfp4_gemm_kernel<true><<<grid, block, kLdsBytes, stream>>>((const uint8_t*)Xq, (const uint8_t*)Xs, tsx,
                                                                (const uint8_t*)Wq, (const uint8_t*)Ws, tsw, Y, ldy,
                                                                (int)M, (int)N, (int)K, tiles_m, tiles_n);
  else
    nvfp4_gemm_kernel<false><<<grid, block, kLdsBytes, stream>>>((const uint8_t*)Xq, (const uint8_t*)Xs, tsx,
                                                                 (const uint8_t*)Wq, (const uint8_t*)Ws, tsw, Y, ldy,
                                                                 (int)M, (int)N, (int)K, tiles_m, tiles_n);
  return hipGetLastError();
}

}  // namespace wush
