// C ABI of the library: argument validation, then kernel launches on the
// caller's stream.  No allocation, no host synchronization (except the *_status
// calls, which are documented to block).  Process-wide state: the switches of
// wush_debug_set and the per-device caches named in the header.
#include "../../include/wush.h"

#include <hip/hip_runtime.h>
#include <atomic>

#include "wush_kernels.hpp"

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline wush_status check_fmt(const wush_fmt& f) {
  if (f.block != 32 || f.elem != WUSH_E2M1 || f.scale != WUSH_E8M0) return WUSH_ERR_FMT;
  if (f.scale_rule != WUSH_SCALE_NOSAT && f.scale_rule != WUSH_SCALE_OCP_FLOOR) return WUSH_ERR_FMT;
  if (f.out_dtype != WUSH_OUT_BF16 && f.out_dtype != WUSH_OUT_F32) return WUSH_ERR_FMT;
  if (f.layout != WUSH_LAYOUT_CANONICAL && f.layout != WUSH_LAYOUT_TILED) return WUSH_ERR_FMT;
  return WUSH_OK;
}

// The tiled layout exists only for K a multiple of 256.
inline wush_status check_layout(const wush_fmt& f, int64_t K) {
  return (f.layout == WUSH_LAYOUT_TILED && K % 256 != 0) ? WUSH_ERR_SHAPE : WUSH_OK;
}

// Kernel index arithmetic uses 32-bit row/column counters, 64-bit offsets of rows and tiles, and
// 32-bit offsets inside a tile of at most 256 rows (256 rows of packed codes must stay below 4 GiB);
// a GEMM launches one workgroup per output tile of at least 128 x 128.
constexpr int64_t kMaxDim = (int64_t)1 << 30;    // rows: M, N, calibration tokens
constexpr int64_t kMaxK = (int64_t)1 << 22;      // channels
constexpr int64_t kMaxOutputs = (int64_t)1 << 40;   // M * N of one GEMM

inline bool gemm_too_large(int64_t M, int64_t N, int64_t K) {
  return M > kMaxDim || N > kMaxDim || K > kMaxK || M * N > kMaxOutputs;   // M, N <= 2^30: the product fits
}

inline wush_status check_rows(int64_t rows, int64_t K, int64_t ld) {
  if (rows <= 0 || K <= 0 || rows > kMaxDim || K > kMaxK) return WUSH_ERR_SHAPE;
  if (K % 32 != 0) return WUSH_ERR_SHAPE;
  if (ld < K || ld % 8 != 0) return WUSH_ERR_SHAPE;
  return WUSH_OK;
}

inline wush_status from_hip(hipError_t e) { return e == hipSuccess ? WUSH_OK : WUSH_ERR_DEVICE; }

// wush_debug_set's switches: 0 = unset, otherwise value + 1 (so that the array needs no initializer).
std::atomic<int> g_debug[wush::kDbgCount];

}  // namespace

namespace wush {
int debug_option(int opt) { return opt >= 0 && opt < kDbgCount ? g_debug[opt].load(std::memory_order_relaxed) - 1 : -1; }
}  // namespace wush

extern "C" {

wush_fmt wush_default_fmt(void) {
  wush_fmt f;
  f.block = 32;
  f.elem = WUSH_E2M1;
  f.scale = WUSH_E8M0;
  f.scale_rule = WUSH_SCALE_NOSAT;
  f.out_dtype = WUSH_OUT_BF16;
  f.layout = WUSH_LAYOUT_CANONICAL;
  return f;
}

wush_status wush_quantize_act(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T_blocks,
                              wush_fmt fmt, void* Xq, void* Xs, float* dbg_Yt, void* stream) {
  if (!X || !T_blocks || !Xq || !Xs) return WUSH_ERR_NULL;
  if (wush_status s = check_fmt(fmt)) return s;
  if (wush_status s = check_rows(M, K, ldx)) return s;
  if (wush_status s = check_layout(fmt, K)) return s;
  if (!aligned16(X) || !aligned16(T_blocks) || !aligned16(Xq) || !aligned16(Xs) || !aligned16(dbg_Yt))
    return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_transform_quant(X, M, K, ldx, T_blocks, fmt.scale_rule,
                                               fmt.layout == WUSH_LAYOUT_TILED, Xq, Xs, dbg_Yt,
                                               static_cast<hipStream_t>(stream)));
}

size_t wush_prepare_weight_workspace(int64_t N, int64_t K) {
  if (N <= 0 || K <= 0 || K % 32 != 0) return 0;
  return wush::weight_prep_workspace_bytes(N, K);
}

wush_status wush_prepare_weight(const void* W, int64_t N, int64_t K, int64_t ldw, const void* T_blocks,
                                wush_fmt fmt, void* Wq, void* Ws, void* workspace,
                                size_t workspace_bytes, void* stream) {
  if (!W || !T_blocks || !Wq || !Ws) return WUSH_ERR_NULL;
  if (wush_status s = check_fmt(fmt)) return s;
  if (wush_status s = check_rows(N, K, ldw)) return s;
  if (wush_status s = check_layout(fmt, K)) return s;
  if (!aligned16(W) || !aligned16(T_blocks) || !aligned16(Wq) || !aligned16(Ws)) return WUSH_ERR_ALIGN;
  if (!workspace || workspace_bytes < wush::weight_prep_workspace_bytes(N, K)) return WUSH_ERR_WORKSPACE;
  if (!aligned16(workspace)) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_weight_prep(W, N, K, ldw, T_blocks, fmt.scale_rule,
                                           fmt.layout == WUSH_LAYOUT_TILED, Wq, Ws, workspace,
                                           static_cast<hipStream_t>(stream)));
}

wush_status wush_workspace_status(const void* workspace, int64_t K, void* stream) {
  if (!workspace) return WUSH_ERR_NULL;
  if (K <= 0 || K % 32 != 0) return WUSH_ERR_SHAPE;
  int flag = 0;
  const char* p = static_cast<const char*>(workspace) + wush::weight_prep_status_offset(K);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(&flag, p, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess) return WUSH_ERR_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return WUSH_ERR_DEVICE;
  return flag ? WUSH_ERR_SINGULAR : WUSH_OK;
}

size_t wush_build_transforms_workspace(int64_t K) {
  if (K <= 0 || K % 32 != 0 || K > kMaxK) return 0;
  return wush::build_transforms_workspace_bytes(K);
}

wush_status wush_build_transforms(const void* W, int64_t N, int64_t ldw, const void* X_cal, int64_t M_cal,
                                  int64_t ldx, int64_t K, double lambda, void* T_blocks, double* T_f64,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (!W || !X_cal || !T_blocks) return WUSH_ERR_NULL;
  if (wush_status s = check_rows(N, K, ldw)) return s;
  if (wush_status s = check_rows(M_cal, K, ldx)) return s;
  if (!(lambda >= 0.0) || !(lambda < 1e6)) return WUSH_ERR_SHAPE;
  if (!aligned16(W) || !aligned16(X_cal) || !aligned16(T_blocks) || !aligned16(T_f64)) return WUSH_ERR_ALIGN;
  if (!workspace || workspace_bytes < wush::build_transforms_workspace_bytes(K)) return WUSH_ERR_WORKSPACE;
  if (!aligned16(workspace)) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_build_transforms(W, N, ldw, X_cal, M_cal, ldx, K, lambda, 32, T_blocks, T_f64, workspace,
                                                static_cast<hipStream_t>(stream)));
}

wush_status wush_build_transforms_nvfp4(const void* W, int64_t N, int64_t ldw, const void* X_cal, int64_t M_cal,
                                        int64_t ldx, int64_t K, double lambda, void* T16, double* T_f64,
                                        void* workspace, size_t workspace_bytes, void* stream) {
  if (!W || !X_cal || !T16) return WUSH_ERR_NULL;
  if (wush_status s = check_rows(N, K, ldw)) return s;
  if (wush_status s = check_rows(M_cal, K, ldx)) return s;
  if (!(lambda >= 0.0) || !(lambda < 1e6)) return WUSH_ERR_SHAPE;
  if (!aligned16(W) || !aligned16(X_cal) || !aligned16(T16) || !aligned16(T_f64)) return WUSH_ERR_ALIGN;
  if (!workspace || workspace_bytes < wush::build_transforms_workspace_bytes(K)) return WUSH_ERR_WORKSPACE;
  if (!aligned16(workspace)) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_build_transforms(W, N, ldw, X_cal, M_cal, ldx, K, lambda, 16, T16, T_f64, workspace,
                                                static_cast<hipStream_t>(stream)));
}

wush_status wush_build_transforms_status(const void* workspace, int64_t K, void* stream) {
  if (!workspace) return WUSH_ERR_NULL;
  if (K <= 0 || K % 32 != 0 || K > kMaxK) return WUSH_ERR_SHAPE;
  int flag = 0;
  const char* p = static_cast<const char*>(workspace) + wush::build_transforms_status_offset(K);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(&flag, p, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess) return WUSH_ERR_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return WUSH_ERR_DEVICE;
  return flag ? WUSH_ERR_SINGULAR : WUSH_OK;
}

wush_status wush_linear(const void* Xq, const void* Xs, const void* Wq, const void* Ws, int64_t M,
                        int64_t N, int64_t K, wush_fmt fmt, void* Y, int64_t ldy, void* stream) {
  if (!Xq || !Xs || !Wq || !Ws || !Y) return WUSH_ERR_NULL;
  if (wush_status s = check_fmt(fmt)) return s;
  if (M <= 0 || N <= 0 || K <= 0 || gemm_too_large(M, N, K) || K % 32 != 0) return WUSH_ERR_SHAPE;
  if (ldy < N) return WUSH_ERR_SHAPE;
  if (wush_status s = check_layout(fmt, K)) return s;
  if (!aligned16(Xq) || !aligned16(Xs) || !aligned16(Wq) || !aligned16(Ws)) return WUSH_ERR_ALIGN;
  const uintptr_t elem = fmt.out_dtype == WUSH_OUT_F32 ? 4 : 2;
  if (reinterpret_cast<uintptr_t>(Y) % elem != 0) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_mxfp4_gemm(Xq, Xs, Wq, Ws, M, N, K, fmt.out_dtype == WUSH_OUT_F32,
                                          fmt.layout == WUSH_LAYOUT_TILED, Y, ldy,
                                          static_cast<hipStream_t>(stream)));
}

size_t wush_prepare_weight_gptq_workspace(int64_t N, int64_t K) {
  if (N <= 0 || K <= 0 || K % 32 != 0 || N > kMaxDim || K > kMaxK) return 0;
  return wush::gptq_prep_workspace_bytes(N, K);
}

wush_status wush_prepare_weight_gptq(const void* W, int64_t N, int64_t K, int64_t ldw, const void* X_cal,
                                     int64_t M_cal, int64_t ldx, double lambda, int32_t transform_given,
                                     wush_fmt fmt, void* T_blocks, void* Wq, void* Ws, void* workspace,
                                     size_t workspace_bytes, void* stream) {
  if (!W || !X_cal || !T_blocks || !Wq || !Ws) return WUSH_ERR_NULL;
  if (wush_status s = check_fmt(fmt)) return s;
  if (wush_status s = check_rows(N, K, ldw)) return s;
  if (wush_status s = check_rows(M_cal, K, ldx)) return s;
  if (wush_status s = check_layout(fmt, K)) return s;
  if (!(lambda >= 0.0) || !(lambda < 1e6)) return WUSH_ERR_SHAPE;
  if (transform_given != 0 && transform_given != 1) return WUSH_ERR_FMT;
  if (!aligned16(W) || !aligned16(X_cal) || !aligned16(T_blocks) || !aligned16(Wq) || !aligned16(Ws)) return WUSH_ERR_ALIGN;
  if (!workspace || workspace_bytes < wush::gptq_prep_workspace_bytes(N, K)) return WUSH_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_gptq_prep(W, N, K, ldw, X_cal, M_cal, ldx, lambda, transform_given, fmt.scale_rule,
                                         fmt.layout == WUSH_LAYOUT_TILED, T_blocks, Wq, Ws, workspace,
                                         static_cast<hipStream_t>(stream)));
}

wush_status wush_prepare_weight_gptq_status(const void* workspace, int64_t N, int64_t K, void* stream) {
  if (!workspace) return WUSH_ERR_NULL;
  if (N <= 0 || K <= 0 || K % 32 != 0 || N > kMaxDim || K > kMaxK) return WUSH_ERR_SHAPE;
  int flag = 0;
  const char* p = static_cast<const char*>(workspace) + wush::gptq_prep_status_offset(N, K);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(&flag, p, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess) return WUSH_ERR_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return WUSH_ERR_DEVICE;
  return flag ? WUSH_ERR_SINGULAR : WUSH_OK;
}

size_t wush_layer_decode_workspace(int64_t K) {
  if (K <= 0 || K % 256 != 0 || K > kMaxK) return 0;
  return wush::layer_decode_workspace_bytes(K);
}

wush_status wush_layer_decode_init(void* workspace, size_t workspace_bytes, int64_t K, void* stream) {
  if (!workspace) return WUSH_ERR_NULL;
  if (K <= 0 || K % 256 != 0 || K > kMaxK) return WUSH_ERR_SHAPE;
  if (workspace_bytes < wush::layer_decode_workspace_bytes(K)) return WUSH_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_layer_decode_init(workspace, K, static_cast<hipStream_t>(stream)));
}

wush_status wush_layer_decode(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T_blocks,
                              const void* Wq, const void* Ws, int64_t N, wush_fmt fmt, void* Y, int64_t ldy,
                              void* workspace, size_t workspace_bytes, void* stream) {
  if (!X || !T_blocks || !Wq || !Ws || !Y) return WUSH_ERR_NULL;
  if (wush_status s = check_fmt(fmt)) return s;
  if (fmt.layout != WUSH_LAYOUT_TILED) return WUSH_ERR_FMT;
  if (wush_status s = check_rows(M, K, ldx)) return s;
  if (M > 64 || K % 256 != 0 || N <= 0 || N > kMaxDim || ldy < N) return WUSH_ERR_SHAPE;
  if (!aligned16(X) || !aligned16(T_blocks) || !aligned16(Wq) || !aligned16(Ws)) return WUSH_ERR_ALIGN;
  const uintptr_t elem = fmt.out_dtype == WUSH_OUT_F32 ? 4 : 2;
  if (reinterpret_cast<uintptr_t>(Y) % elem != 0) return WUSH_ERR_ALIGN;
  if (!workspace || workspace_bytes < wush::layer_decode_workspace_bytes(K)) return WUSH_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return WUSH_ERR_ALIGN;
  // WUSH_DEBUG_DECODE_TEST_TIMEOUT (tests only): make every workgroup's barrier wait expire at once.
  const int test_timeout = wush::debug_option(wush::kDbgDecodeTestTimeout) == 1;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int out_f32 = fmt.out_dtype == WUSH_OUT_F32;
  // Two launches by default.  With the host's launch cost out of the picture (graph
  // replay) two back-to-back kernels are 1.5-2 us apart, while the single-launch
  // form pays 4-6 us for its grid-wide barrier across the eight XCDs: measured
  // 6.4 against 9.5 us on 4096 x 6144, 40 against 55 us on 8192 x 57344 (M = 1).
  // wush_debug_set(WUSH_DEBUG_DECODE_FUSED, 1) selects the single launch.
  const bool fused = wush::debug_option(wush::kDbgDecodeFused) == 1;
  if (fused || test_timeout)
    return from_hip(wush::launch_layer_decode(X, M, K, ldx, T_blocks, Wq, Ws, N, fmt.scale_rule, out_f32, Y, ldy,
                                              workspace, test_timeout, st));
  // two launches through the same workspace (same Xq/Xs layout and positions)
  char* wsb = static_cast<char*>(workspace);
  void* Xq = wsb;
  void* Xs = wsb + wush::layer_decode_scales_offset(K);
  if (hipError_t e = wush::launch_transform_quant(X, M, K, ldx, T_blocks, fmt.scale_rule, 1, Xq, Xs, nullptr, st))
    return from_hip(e);
  return from_hip(wush::launch_mxfp4_gemm_skinny(Xq, Xs, Wq, Ws, M, N, K, out_f32, Y, ldy, st));
}

// ---------------------------------------------------------------------------
// wush_layer_decode_static: wush_layer_decode (two-launch form) for callers that can neither
// allocate nor pass a workspace.  The quantized activations live in a file-scope device array;
// every GPU the library runs on holds its own copy of it at its own address, looked up once per
// device with hipGetSymbolAddress (the array's name is only a host-side stand-in: host code
// must never pass it to a kernel) and kept in scratch_ptr[].
// ---------------------------------------------------------------------------
namespace {

constexpr int64_t kStaticDecodeMaxK = 32768;
// codes of two 32-token row blocks, then their scales: (K / 256) * (2 * 4096 + 2 * 256) bytes
constexpr size_t kStaticScratchBytes = (size_t)(kStaticDecodeMaxK / 256) * (2 * 4096 + 2 * 256);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::atomic<unsigned char*> scratch_ptr[64];   // per device; zero-initialized

wush_status scratch_of_current_device(unsigned char** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return WUSH_ERR_DEVICE;
  const bool tracked = dev >= 0 && dev < 64;
  unsigned char* p = tracked ? scratch_ptr[dev].load(std::memory_order_acquire) : nullptr;
  if (!p) {
    if (hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)) != hipSuccess || !p) return WUSH_ERR_DEVICE;
    if (tracked) scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return WUSH_OK;
}

}  // namespace

wush_status wush_layer_decode_static(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T_blocks,
                                     const void* Wq, const void* Ws, int64_t N, wush_fmt fmt, void* Y, int64_t ldy,
                                     void* stream) {
  if (!X || !T_blocks || !Wq || !Ws || !Y) return WUSH_ERR_NULL;
  if (wush_status s = check_fmt(fmt)) return s;
  if (fmt.layout != WUSH_LAYOUT_TILED) return WUSH_ERR_FMT;
  if (wush_status s = check_rows(M, K, ldx)) return s;
  if (M > 64 || K % 256 != 0 || N <= 0 || N > kMaxDim || ldy < N) return WUSH_ERR_SHAPE;
  if (K > kStaticDecodeMaxK) return WUSH_ERR_TOO_LARGE;
  if (!aligned16(X) || !aligned16(T_blocks) || !aligned16(Wq) || !aligned16(Ws)) return WUSH_ERR_ALIGN;
  const uintptr_t elem = fmt.out_dtype == WUSH_OUT_F32 ? 4 : 2;
  if (reinterpret_cast<uintptr_t>(Y) % elem != 0) return WUSH_ERR_ALIGN;
  unsigned char* sc = nullptr;
  if (wush_status s = scratch_of_current_device(&sc)) return s;
  // Same positions inside the scratch as inside a wush_layer_decode workspace of this K.  Nothing has
  // to start at zero: the quantizer writes every row below M of the row blocks the GEMM reads, and the
  // rows from M to the end of the last block (whatever an earlier call left there: valid codes and
  // scale bytes, or the zeros the array starts with) only reach output rows that are never stored.
  void* Xq = sc;
  void* Xs = sc + wush::layer_decode_scales_offset(K);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hipError_t e = wush::launch_transform_quant(X, M, K, ldx, T_blocks, fmt.scale_rule, 1, Xq, Xs, nullptr, st))
    return from_hip(e);
  return from_hip(wush::launch_mxfp4_gemm_skinny(Xq, Xs, Wq, Ws, M, N, K, fmt.out_dtype == WUSH_OUT_F32, Y, ldy, st));
}

wush_status wush_layer_decode_status(const void* workspace, int64_t K, void* stream) {
  if (!workspace) return WUSH_ERR_NULL;
  if (K <= 0 || K % 256 != 0 || K > kMaxK) return WUSH_ERR_SHAPE;
  unsigned flag = 0;
  const char* p = static_cast<const char*>(workspace) + wush::layer_decode_error_offset(K);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(&flag, p, sizeof(flag), hipMemcpyDeviceToHost, st) != hipSuccess) return WUSH_ERR_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return WUSH_ERR_DEVICE;
  return flag ? WUSH_ERR_TIMEOUT : WUSH_OK;
}

static inline wush_status check_nv_layout(int32_t layout, int64_t K) {
  if (layout != WUSH_LAYOUT_CANONICAL && layout != WUSH_LAYOUT_TILED) return WUSH_ERR_FMT;
  return (layout == WUSH_LAYOUT_TILED && K % 64 != 0) ? WUSH_ERR_SHAPE : WUSH_OK;
}

wush_status wush_quantize_act_nvfp4(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T16,
                                    const float* tensor_scale, int32_t layout, void* Xq, void* Xs, float* dbg_Yt,
                                    void* stream) {
  if (!X || !T16 || !tensor_scale || !Xq || !Xs) return WUSH_ERR_NULL;
  if (wush_status s = check_rows(M, K, ldx)) return s;
  if (wush_status s = check_nv_layout(layout, K)) return s;
  if (!aligned16(X) || !aligned16(T16) || !aligned16(Xq) || !aligned16(Xs) || !aligned16(dbg_Yt)) return WUSH_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(tensor_scale) % 4 != 0) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_nvfp4_transform_quant(X, M, K, ldx, T16, tensor_scale, layout == WUSH_LAYOUT_TILED, Xq,
                                                     Xs, dbg_Yt, static_cast<hipStream_t>(stream)));
}

wush_status wush_calibrate_act_nvfp4(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T16,
                                     float* tensor_scale, void* stream) {
  if (!X || !T16 || !tensor_scale) return WUSH_ERR_NULL;
  if (wush_status s = check_rows(M, K, ldx)) return s;
  if (!aligned16(X) || !aligned16(T16)) return WUSH_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(tensor_scale) % 4 != 0) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_nvfp4_calibrate(X, M, K, ldx, T16, tensor_scale, static_cast<hipStream_t>(stream)));
}

size_t wush_prepare_weight_nvfp4_workspace(int64_t K) {
  if (K <= 0 || K % 32 != 0 || K > kMaxK) return 0;
  return wush::nvfp4_weight_prep_workspace_bytes(K);
}

wush_status wush_prepare_weight_nvfp4(const void* W, int64_t N, int64_t K, int64_t ldw, const void* T16,
                                      int32_t layout, void* Wq, void* Ws, float* tensor_scale, void* workspace,
                                      size_t workspace_bytes, void* stream) {
  if (!W || !T16 || !Wq || !Ws || !tensor_scale) return WUSH_ERR_NULL;
  if (wush_status s = check_rows(N, K, ldw)) return s;
  if (wush_status s = check_nv_layout(layout, K)) return s;
  if (!aligned16(W) || !aligned16(T16) || !aligned16(Wq) || !aligned16(Ws)) return WUSH_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(tensor_scale) % 4 != 0) return WUSH_ERR_ALIGN;
  if (!workspace || workspace_bytes < wush::nvfp4_weight_prep_workspace_bytes(K)) return WUSH_ERR_WORKSPACE;
  if (!aligned16(workspace)) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_nvfp4_weight_prep(W, N, K, ldw, T16, layout == WUSH_LAYOUT_TILED, Wq, Ws, tensor_scale,
                                                 workspace, static_cast<hipStream_t>(stream)));
}

wush_status wush_prepare_weight_nvfp4_status(const void* workspace, int64_t K, void* stream) {
  if (!workspace) return WUSH_ERR_NULL;
  if (K <= 0 || K % 32 != 0 || K > kMaxK) return WUSH_ERR_SHAPE;
  int flag = 0;
  const char* p = static_cast<const char*>(workspace) + wush::nvfp4_weight_prep_status_offset(K);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(&flag, p, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess) return WUSH_ERR_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return WUSH_ERR_DEVICE;
  return flag ? WUSH_ERR_SINGULAR : WUSH_OK;
}

wush_status wush_linear_nvfp4(const void* Xq, const void* Xs, const float* tsx, const void* Wq, const void* Ws,
                              const float* tsw, int64_t M, int64_t N, int64_t K, int32_t layout, int32_t out_dtype,
                              void* Y, int64_t ldy, void* stream) {
  if (!Xq || !Xs || !tsx || !Wq || !Ws || !tsw || !Y) return WUSH_ERR_NULL;
  if (out_dtype != WUSH_OUT_BF16 && out_dtype != WUSH_OUT_F32) return WUSH_ERR_FMT;
  if (layout != WUSH_LAYOUT_CANONICAL && layout != WUSH_LAYOUT_TILED) return WUSH_ERR_FMT;
  if (M <= 0 || N <= 0 || K <= 0 || gemm_too_large(M, N, K) || K % 64 != 0) return WUSH_ERR_SHAPE;
  if (ldy < N) return WUSH_ERR_SHAPE;
  if (!aligned16(Xq) || !aligned16(Xs) || !aligned16(Wq) || !aligned16(Ws)) return WUSH_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(tsx) % 4 != 0 || reinterpret_cast<uintptr_t>(tsw) % 4 != 0) return WUSH_ERR_ALIGN;
  const uintptr_t elem = out_dtype == WUSH_OUT_F32 ? 4 : 2;
  if (reinterpret_cast<uintptr_t>(Y) % elem != 0) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_nvfp4_gemm(Xq, Xs, tsx, Wq, Ws, tsw, M, N, K, out_dtype == WUSH_OUT_F32,
                                          layout == WUSH_LAYOUT_TILED, Y, ldy, static_cast<hipStream_t>(stream)));
}

wush_status wush_quantize_f32_nvfp4(const float* Yt, int64_t M, int64_t K, const float* tensor_scale, int32_t layout,
                                    void* q, void* s, void* stream) {
  if (!Yt || !tensor_scale || !q || !s) return WUSH_ERR_NULL;
  if (M <= 0 || K <= 0 || M > kMaxDim || K > kMaxK || K % 32 != 0) return WUSH_ERR_SHAPE;
  if (wush_status st = check_nv_layout(layout, K)) return st;
  if (!aligned16(Yt) || !aligned16(q) || !aligned16(s)) return WUSH_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(tensor_scale) % 4 != 0) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_nvfp4_quantize_f32(Yt, M, K, tensor_scale, layout == WUSH_LAYOUT_TILED, q, s,
                                                  static_cast<hipStream_t>(stream)));
}

wush_status wush_packed_sizes_nvfp4(int64_t rows, int64_t K, int32_t layout, size_t* code_bytes, size_t* scale_bytes) {
  if (!code_bytes || !scale_bytes) return WUSH_ERR_NULL;
  if (rows <= 0 || K <= 0 || rows > kMaxDim || K > kMaxK || K % 32 != 0) return WUSH_ERR_SHAPE;
  if (wush_status st = check_nv_layout(layout, K)) return st;
  const int64_t r = layout == WUSH_LAYOUT_TILED ? (rows + 31) / 32 * 32 : rows;
  *code_bytes = (size_t)r * (size_t)(K / 2);
  *scale_bytes = (size_t)r * (size_t)(K / 16);
  return WUSH_OK;
}

wush_status wush_unpack_tiled_nvfp4(const void* q_tiled, const void* s_tiled, int64_t rows, int64_t K, void* q, void* s,
                                    void* stream) {
  if (!q_tiled || !s_tiled || !q || !s) return WUSH_ERR_NULL;
  if (rows <= 0 || K <= 0 || rows > kMaxDim || K > kMaxK || K % 64 != 0) return WUSH_ERR_SHAPE;
  if (!aligned16(q_tiled) || !aligned16(s_tiled) || !aligned16(q) || !aligned16(s)) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_nvfp4_unpack_tiled(q_tiled, s_tiled, rows, K, q, s, static_cast<hipStream_t>(stream)));
}

wush_status wush_quantize_act_int4(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T_blocks,
                                   int32_t layout, void* Xq, void* Xs, float* dbg_Yt, void* stream) {
  if (!X || !T_blocks || !Xq || !Xs) return WUSH_ERR_NULL;
  if (wush_status s = check_rows(M, K, ldx)) return s;
  if (wush_status s = check_nv_layout(layout, K)) return s;
  if (!aligned16(X) || !aligned16(T_blocks) || !aligned16(Xq) || !aligned16(Xs) || !aligned16(dbg_Yt))
    return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_int4_transform_quant(X, M, K, ldx, T_blocks, layout == WUSH_LAYOUT_TILED, Xq, Xs, dbg_Yt,
                                                    static_cast<hipStream_t>(stream)));
}

wush_status wush_prepare_weight_int4(const void* W, int64_t N, int64_t K, int64_t ldw, const void* T_blocks,
                                     int32_t layout, void* Wq, void* Ws, void* workspace, size_t workspace_bytes,
                                     void* stream) {
  if (!W || !T_blocks || !Wq || !Ws) return WUSH_ERR_NULL;
  if (wush_status s = check_rows(N, K, ldw)) return s;
  if (wush_status s = check_nv_layout(layout, K)) return s;
  if (!aligned16(W) || !aligned16(T_blocks) || !aligned16(Wq) || !aligned16(Ws)) return WUSH_ERR_ALIGN;
  if (!workspace || workspace_bytes < wush::weight_prep_workspace_bytes(N, K)) return WUSH_ERR_WORKSPACE;
  if (!aligned16(workspace)) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_int4_weight_prep(W, N, K, ldw, T_blocks, layout == WUSH_LAYOUT_TILED, Wq, Ws, workspace,
                                                static_cast<hipStream_t>(stream)));
}

wush_status wush_linear_int4(const void* Xq, const void* Xs, const void* Wq, const void* Ws, int64_t M, int64_t N,
                             int64_t K, int32_t layout, int32_t out_dtype, void* Y, int64_t ldy, void* stream) {
  if (!Xq || !Xs || !Wq || !Ws || !Y) return WUSH_ERR_NULL;
  if (out_dtype != WUSH_OUT_BF16 && out_dtype != WUSH_OUT_F32) return WUSH_ERR_FMT;
  if (layout != WUSH_LAYOUT_CANONICAL && layout != WUSH_LAYOUT_TILED) return WUSH_ERR_FMT;
  if (M <= 0 || N <= 0 || K <= 0 || gemm_too_large(M, N, K) || K % 64 != 0) return WUSH_ERR_SHAPE;
  if (ldy < N) return WUSH_ERR_SHAPE;
  if (!aligned16(Xq) || !aligned16(Xs) || !aligned16(Wq) || !aligned16(Ws)) return WUSH_ERR_ALIGN;
  const uintptr_t elem = out_dtype == WUSH_OUT_F32 ? 4 : 2;
  if (reinterpret_cast<uintptr_t>(Y) % elem != 0) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_int4_gemm(Xq, Xs, Wq, Ws, M, N, K, out_dtype == WUSH_OUT_F32,
                                         layout == WUSH_LAYOUT_TILED, Y, ldy, static_cast<hipStream_t>(stream)));
}

wush_status wush_quantize_f32_int4(const float* Yt, int64_t M, int64_t K, int32_t layout, void* q, void* s,
                                   void* stream) {
  if (!Yt || !q || !s) return WUSH_ERR_NULL;
  if (M <= 0 || K <= 0 || M > kMaxDim || K > kMaxK || K % 32 != 0) return WUSH_ERR_SHAPE;
  if (wush_status st = check_nv_layout(layout, K)) return st;
  if (!aligned16(Yt) || !aligned16(q) || !aligned16(s)) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_int4_quantize_f32(Yt, M, K, layout == WUSH_LAYOUT_TILED, q, s,
                                                 static_cast<hipStream_t>(stream)));
}

wush_status wush_quantize_f32(const float* Yt, int64_t M, int64_t K, wush_fmt fmt, void* q, void* s,
                              void* stream) {
  if (!Yt || !q || !s) return WUSH_ERR_NULL;
  if (wush_status st = check_fmt(fmt)) return st;
  if (M <= 0 || K <= 0 || M > kMaxDim || K > kMaxK || K % 32 != 0) return WUSH_ERR_SHAPE;
  if (wush_status st = check_layout(fmt, K)) return st;
  if (!aligned16(Yt) || !aligned16(q) || !aligned16(s)) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_quantize_f32(Yt, M, K, fmt.scale_rule, fmt.layout == WUSH_LAYOUT_TILED, q, s,
                                            static_cast<hipStream_t>(stream)));
}

wush_status wush_packed_sizes(int64_t rows, int64_t K, wush_fmt fmt, size_t* code_bytes, size_t* scale_bytes) {
  if (!code_bytes || !scale_bytes) return WUSH_ERR_NULL;
  if (wush_status st = check_fmt(fmt)) return st;
  if (rows <= 0 || K <= 0 || rows > kMaxDim || K > kMaxK || K % 32 != 0) return WUSH_ERR_SHAPE;
  if (wush_status st = check_layout(fmt, K)) return st;
  const int64_t padded = fmt.layout == WUSH_LAYOUT_TILED ? (rows + 255) / 256 * 256 : rows;
  *code_bytes = (size_t)(padded * (K / 2));
  *scale_bytes = (size_t)(padded * (K / 32));
  return WUSH_OK;
}

wush_status wush_unpack_tiled(const void* q_tiled, const void* s_tiled, int64_t rows, int64_t K, void* q,
                              void* s, void* stream) {
  if (!q_tiled || !s_tiled || !q || !s) return WUSH_ERR_NULL;
  if (rows <= 0 || K <= 0 || rows > kMaxDim || K > kMaxK || K % 256 != 0) return WUSH_ERR_SHAPE;
  if (!aligned16(q_tiled) || !aligned16(s_tiled) || !aligned16(q) || !aligned16(s)) return WUSH_ERR_ALIGN;
  return from_hip(wush::launch_unpack_tiled(q_tiled, s_tiled, rows, K, q, s, static_cast<hipStream_t>(stream)));
}

wush_status wush_debug_set(int32_t option, int32_t value) {
  if (option < 0 || option >= wush::kDbgCount) return WUSH_ERR_FMT;
  if (value < -1 || value > 1023) return WUSH_ERR_SHAPE;
  g_debug[option].store(value + 1, std::memory_order_relaxed);
  return WUSH_OK;
}

const char* wush_status_string(wush_status st) {
  switch (st) {
    case WUSH_OK: return "ok";
    case WUSH_ERR_NULL: return "null pointer";
    case WUSH_ERR_SHAPE: return "bad shape or leading dimension";
    case WUSH_ERR_ALIGN: return "pointer not 16-byte aligned";
    case WUSH_ERR_FMT: return "unsupported format";
    case WUSH_ERR_WORKSPACE: return "workspace missing or too small";
    case WUSH_ERR_DEVICE: return "HIP runtime error";
    case WUSH_ERR_SINGULAR: return "singular transform block";
    case WUSH_ERR_TIMEOUT: return "grid barrier wait expired";
    case WUSH_ERR_TOO_LARGE: return "size beyond the fixed scratch of this entry point";
  }
  return "unknown status";
}

const char* wush_version(void) { return "0.10"; }

}  // extern "C"
