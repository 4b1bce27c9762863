// Host-side launchers of the gfx950 kernels.  Arguments are assumed valid:
// the C-ABI layer checks shapes, alignment and formats before calling these.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace wush {

// Compute units of the current device (queried once per device).
int device_cu_count();

// Process-wide switches for tests and measurements (set through wush_debug_set, never from the
// environment): which kernel or tile shape a launcher takes where it would otherwise choose by itself.
// -1 = unset = the library's own choice.  The numbering is that of the WUSH_DEBUG_* constants of wush.h.
enum DebugOption {
  kDbgGemmTile = 0,          // tiled MXFP4 GEMM: 0..3 = 256x256, 128x384, 128x256, 128x128
  kDbgGemmSkinny = 1,        // MXFP4 GEMM, up to 128 tokens: 1 = weight-streaming kernel, 0 = tiled kernel
  kDbgGemmSimple = 2,        // canonical layout: 1 = the one-wave-per-tile kernel
  kDbgW4Width = 3,           // NVFP4 / INT4 tiled GEMM: tile width 2..4 (x 64 output channels)
  kDbgW4Skinny = 4,          // NVFP4 / INT4 GEMM, up to 128 tokens: 0 = tiled kernel, 1, 2 = weight-streaming kernel (K split,
                             // shared X)
  kDbgDecodeFused = 5,       // wush_layer_decode: 1 = single launch with a grid-wide barrier
  kDbgDecodeTestTimeout = 6, // wush_layer_decode: 1 = the barrier wait gives up at once (error-path test)
  kDbgCount
};
int debug_option(int opt);

// Raises a kernel's dynamic LDS limit, once per device: the attribute belongs to the device's copy of
// the code object, so a process that drives several GPUs has to set it on each.  One object per
// kernel instantiation (a function-local static of its launcher).
class DynamicLdsLimit {
 public:
  hipError_t ensure(const void* kernel, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < 64;
    if (tracked && (done_.load(std::memory_order_acquire) >> dev & 1)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && tracked) done_.fetch_or(uint64_t(1) << dev, std::memory_order_release);
    return e;
  }

 private:
  std::atomic<uint64_t> done_{0};
};
// Token tiles per workgroup of the fused transform + quantize kernels (ntiles 32-token tiles,
// col_groups workgroups across the channels).
int token_walk(int ntiles, int col_groups);
// The same for kernels whose workgroups can hold two groups of waves that walk alternate tiles:
// tiles per workgroup and the number of groups (1 or 2).
struct Walk {
  int tiles_per_wg, groups;
};
Walk token_walk_groups(int ntiles, int col_groups);

// `tiled` != 0 selects the fragment-order layout of wush_device.hpp (K % 256 == 0).
hipError_t launch_transform_quant(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T,
                                  int rule, int tiled, void* Xq, void* Xs, float* dbg, hipStream_t stream);

hipError_t launch_quantize_f32(const float* Y, int64_t M, int64_t K, int rule, int tiled, void* q, void* s,
                               hipStream_t stream);

hipError_t launch_unpack_tiled(const void* qt, const void* st, int64_t rows, int64_t K, void* q, void* s,
                               hipStream_t stream);

// workspace layout: [C][32][32] FP64 inverses, then one int32 status word.
size_t weight_prep_workspace_bytes(int64_t N, int64_t K);
size_t weight_prep_status_offset(int64_t K);
hipError_t launch_weight_prep(const void* W, int64_t N, int64_t K, int64_t ldw, const void* T,
                              int rule, int tiled, void* Wq, void* Ws, void* workspace, hipStream_t stream);

hipError_t launch_mxfp4_gemm(const void* Xq, const void* Xs, const void* Wq, const void* Ws,
                             int64_t M, int64_t N, int64_t K, int out_f32, int tiled, void* Y, int64_t ldy,
                             hipStream_t stream);

// Alg. 1 / Alg. 2 (RTN case) transform construction; workspace = partial moments + status word.
size_t build_transforms_workspace_bytes(int64_t K);
size_t build_transforms_status_offset(int64_t K);
hipError_t launch_build_transforms(const void* W, int64_t N, int64_t ldw, const void* X, int64_t Mc, int64_t ldx,
                                   int64_t K, double lambda, int block, void* T_out, double* T_f64, void* workspace,
                                   hipStream_t stream);   // block = 32, or 16 for the NVFP4 variant

// Operands in the fragment-order layout (K % 256 == 0).
hipError_t launch_mxfp4_gemm_frag(const void* Xq, const void* Xs, const void* Wq, const void* Ws,
                                  int64_t M, int64_t N, int64_t K, int out_f32, void* Y, int64_t ldy,
                                  hipStream_t stream);

// Alg. 2, GPTQ case: transforms (unless given) and pre-quantized weights.  Workspace: FP64 Hessian factor,
// its inverse, a working copy of W, per-block scratch, status word.
size_t gptq_prep_workspace_bytes(int64_t N, int64_t K);
size_t gptq_prep_status_offset(int64_t N, int64_t K);
hipError_t launch_gptq_prep(const void* W, int64_t N, int64_t K, int64_t ldw, const void* Xc, int64_t Mc, int64_t ldx,
                            double lambda, int transform_given, int rule, int tiled, void* T_blocks, void* Wq, void* Ws,
                            void* workspace, hipStream_t stream);

// Decode-sized paths (GEMM: M <= 128; fused layer: M <= 64; fragment-order operands).
hipError_t launch_mxfp4_gemm_skinny(const void* Xq, const void* Xs, const void* Wq, const void* Ws, int64_t M,
                                    int64_t N, int64_t K, int out_f32, void* Y, int64_t ldy, hipStream_t stream);
// workspace layout: Xq for 64 tokens | Xs | barrier words (generation, error flag, arrival and release slots).
size_t layer_decode_workspace_bytes(int64_t K);
size_t layer_decode_scales_offset(int64_t K);
size_t layer_decode_state_offset(int64_t K);
size_t layer_decode_error_offset(int64_t K);
hipError_t launch_layer_decode_init(void* workspace, int64_t K, hipStream_t stream);
// test_timeout != 0: the barrier expects one workgroup more than launched and gives up after a few polls.
hipError_t launch_layer_decode(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T, const void* Wq,
                               const void* Ws, int64_t N, int rule, int out_f32, void* Y, int64_t ldy,
                               void* workspace, int test_timeout, hipStream_t stream);

// NVFP4 variant (E2M1, E4M3 scale per 16, FP32 tensor scale in device memory; 16 x 16 transforms).
// `tiled` != 0 selects the layout of nvfp4_layout.hpp (K % 64 == 0, buffers of a multiple of 32 rows).
hipError_t launch_nvfp4_transform_quant(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T16,
                                        const float* tscale, int tiled, void* Xq, void* Xs, float* dbg,
                                        hipStream_t stream);
// AbsMax of T X over the batch / (6 * 448) -> *ts_out (device float).
hipError_t launch_nvfp4_calibrate(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T16, float* ts_out,
                                  hipStream_t stream);
hipError_t launch_nvfp4_quantize_f32(const float* Y, int64_t M, int64_t K, const float* tscale, int tiled, void* q,
                                     void* s, hipStream_t stream);
hipError_t launch_nvfp4_unpack_tiled(const void* qt, const void* st, int64_t rows, int64_t K, void* q, void* s,
                                     hipStream_t stream);
// workspace: [K/16][16][16] FP64 inverses | u64 AbsMax bits | int32 status
size_t nvfp4_weight_prep_workspace_bytes(int64_t K);
size_t nvfp4_weight_prep_status_offset(int64_t K);
hipError_t launch_nvfp4_weight_prep(const void* W, int64_t N, int64_t K, int64_t ldw, const void* T16, int tiled,
                                    void* Wq, void* Ws, float* ts_out, void* workspace, hipStream_t stream);
// K % 64 == 0
hipError_t launch_nvfp4_gemm(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws,
                             const float* tsw, int64_t M, int64_t N, int64_t K, int out_f32, int tiled, void* Y,
                             int64_t ldy, hipStream_t stream);

// Weight-streaming GEMMs of the two formats for M <= 128, tiled layout only (w4_gemm_skinny.hip).
hipError_t launch_nvfp4_gemm_skinny(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws,
                                    const float* tsw, int64_t M, int64_t N, int64_t K, int out_f32, void* Y,
                                    int64_t ldy, hipStream_t stream);
hipError_t launch_int4_gemm_skinny(const void* Xq, const void* Xs, const void* Wq, const void* Ws, int64_t M, int64_t N,
                                   int64_t K, int out_f32, void* Y, int64_t ldy, hipStream_t stream);

// INT4 variant (two's-complement codes, BF16 scale per 32, 32 x 32 transforms); layouts as for NVFP4
// (the 4 scale bytes of a K step of 64 are two BF16 numbers).  Weight workspace: as launch_weight_prep.
hipError_t launch_int4_transform_quant(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T, int tiled,
                                       void* Xq, void* Xs, float* dbg, hipStream_t stream);
hipError_t launch_int4_quantize_f32(const float* Y, int64_t M, int64_t K, int tiled, void* q, void* s,
                                    hipStream_t stream);
hipError_t launch_int4_weight_prep(const void* W, int64_t N, int64_t K, int64_t ldw, const void* T, int tiled, void* Wq,
                                   void* Ws, void* workspace, hipStream_t stream);
// K % 64 == 0
hipError_t launch_int4_gemm(const void* Xq, const void* Xs, const void* Wq, const void* Ws, int64_t M, int64_t N,
                            int64_t K, int out_f32, int tiled, void* Y, int64_t ldy, hipStream_t stream);

}  // namespace wush
