/*
 * wush.h -- C ABI of the MI355X (gfx950) W4A4 WUSH linear-layer library.
 *
 * The library computes the per-layer forward of a weight+activation MXFP4
 * quantized linear layer with block-diagonal, data-aware transforms (paper:
 * Methodology, "Block-independent constraint", the WUSH construction equation,
 * Alg. 2 RTN case, and the layer forward-pass equation; kernels: section
 * "GPU Kernel Support").
 *
 * Notation (ours <-> paper).  Tensors are row-major with channels last:
 *   X [M][K]  activations, M = d_batch tokens, K = d_in channels (paper: X^T)
 *   W [N][K]  weights, N = d_out (paper: W^T)
 *   block b = channels 32b .. 32b+31, C = K/32 blocks, d = 32
 *   T [C][32][32]  T[b][j][k] = (T_wush of block b)[j][k]: input channel k ->
 *                  transformed channel j
 *
 *   Yt[m,32b+j] = sum_k X[m,32b+k] T[b][j][k]                (T_wush X)
 *   Wt[n,32b+j] = sum_k W[n,32b+k] inv(T[b])[k][j]           (T_wush^{-T} W)
 *   Y [m,n]     = sum_kappa deq(q(Yt))[m,kappa] deq(q(Wt))[n,kappa]
 *
 * Quantizer q (RTN with AbsMax scale per group of 32 consecutive channels):
 *   element E2M1: 4-bit pattern s|e1 e0|m, codes 0..7 = 0,.5,1,1.5,2,3,4,6;
 *   scale E8M0: byte s means 2^(s-127), s in 0..254 (255 is never written);
 *   WUSH_SCALE_NOSAT : smallest power of two with AbsMax <= 6*2^e (no clipping)
 *   WUSH_SCALE_OCP_FLOOR : e = floor(log2 AbsMax) - 2 (maxima in (6,8)*2^e clip)
 *   rounding to nearest, ties to the even code; the input's sign bit is kept
 *   even if the magnitude rounds to zero; an all-zero group gets byte 0.
 *   NaN/Inf inputs are undefined behaviour.
 *
 * Packed layouts.
 *   WUSH_LAYOUT_CANONICAL (default; the reference layout every test reads):
 *     codes  [rows][K/2] bytes, element k in byte k/2, even k = low nibble;
 *     scales [rows][K/32] bytes.
 *   WUSH_LAYOUT_TILED (opaque, fast; K % 256 == 0): the same 16-byte groups and
 *     scale bytes, reordered into the lane order of the block-scaled MFMA
 *     operands so that the GEMM reads them with contiguous 128-bit accesses.
 *     Buffers are padded to a multiple of 256 rows (wush_packed_sizes gives the
 *     sizes; padding rows may be read but never reach a valid output).  The quantizers
 *     write it and wush_linear reads it when fmt.layout says so; both operands
 *     of one wush_linear call use the same layout.  wush_unpack_tiled converts
 *     it back to canonical.
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates nothing.  What it keeps between calls, per process and device: the
 *     compute-unit count, which kernels had their LDS limit raised, the fixed
 *     scratch array of wush_layer_decode_static, and the switches of wush_debug_set;
 *     no call's result depends on an earlier call.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls only
 *     enqueue work and return; results are valid after the stream is
 *     synchronized.
 *   - All arguments are validated before any launch.  On any error nothing is
 *     launched and no output byte is touched; the return value says why.
 *   - Requirements: M, N, K > 0; K % 32 == 0; data pointers 16-byte aligned;
 *     input leading dimensions (in elements) >= K and a multiple of 8;
 *     fmt.block == 32, fmt.elem == WUSH_E2M1, fmt.scale == WUSH_E8M0.
 *   - Largest sizes: row counts (M, N, calibration tokens) up to 2^30, K up to
 *     2^22, M * N of one GEMM up to 2^40; beyond that WUSH_ERR_SHAPE (the
 *     workspace-size queries return 0).
 */
#ifndef WUSH_H_
#define WUSH_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  WUSH_OK = 0,
  WUSH_ERR_NULL = 1,      /* a required pointer is NULL */
  WUSH_ERR_SHAPE = 2,     /* non-positive or too large size, K % 32 != 0, bad leading dimension */
  WUSH_ERR_ALIGN = 3,     /* pointer not 16-byte aligned */
  WUSH_ERR_FMT = 4,       /* unsupported format descriptor */
  WUSH_ERR_WORKSPACE = 5, /* workspace missing or too small */
  WUSH_ERR_DEVICE = 6,    /* the HIP runtime reported a launch error */
  WUSH_ERR_SINGULAR = 7,  /* a transform block is singular / a moment not positive definite */
  WUSH_ERR_TIMEOUT = 8,   /* wush_layer_decode: a workgroup gave up waiting at the grid-wide barrier */
  WUSH_ERR_TOO_LARGE = 9  /* wush_layer_decode_static: K beyond what its fixed scratch holds */
} wush_status;

enum { WUSH_E2M1 = 1 };
enum { WUSH_E8M0 = 1 };
enum { WUSH_SCALE_NOSAT = 0, WUSH_SCALE_OCP_FLOOR = 1 };
enum { WUSH_OUT_BF16 = 0, WUSH_OUT_F32 = 1 };
enum { WUSH_LAYOUT_CANONICAL = 0, WUSH_LAYOUT_TILED = 1 };

typedef struct {
  int32_t block;      /* 32 */
  int32_t elem;       /* WUSH_E2M1 */
  int32_t scale;      /* WUSH_E8M0 */
  int32_t scale_rule; /* WUSH_SCALE_NOSAT (default) or WUSH_SCALE_OCP_FLOOR */
  int32_t out_dtype;  /* wush_linear only: WUSH_OUT_BF16 (default) or WUSH_OUT_F32 */
  int32_t layout;     /* packed codes/scales: WUSH_LAYOUT_CANONICAL (default) or WUSH_LAYOUT_TILED */
} wush_fmt;

/* The default descriptor: MXFP4, block 32, no-saturation scale, BF16 output. */
wush_fmt wush_default_fmt(void);

/*
 * Fused activation transform + quantization: q(T_wush X) of the layer
 * forward-pass equation, one fused kernel as in "GPU Kernel Support".
 *   X        in   bf16 [M][ldx] (device), K contiguous channels per row
 *   T_blocks in   bf16 [K/32][32][32] (device)
 *   Xq       out  u8 [M][K/2] packed E2M1 codes   } canonical shapes; sizes for the
 *   Xs       out  u8 [M][K/32] E8M0 scale bytes   } tiled layout: wush_packed_sizes
 *   dbg_Yt   out  optional (may be NULL): f32 [M][K], the transformed values
 *                 exactly as the kernel fed them to its quantizer (FP32 MFMA
 *                 accumulators).  Test tap; costs 4 B/element of extra writes.
 */
wush_status wush_quantize_act(const void* X, int64_t M, int64_t K, int64_t ldx,
                              const void* T_blocks, wush_fmt fmt,
                              void* Xq, void* Xs, float* dbg_Yt, void* stream);

/*
 * Offline weight preparation (Alg. 2, RTN case, last two steps):
 * T_xvsh = T_wush^{-T}, then q(T_xvsh W).  The inverse of every 32x32 block
 * is taken in FP64 on the device (Gauss-Jordan, partial pivoting), the product
 * W_blk inv(T_b) is formed in FP64 and quantized with the same rules as the
 * activations.
 *   W        in   bf16 [N][ldw] (device)
 *   T_blocks in   bf16 [K/32][32][32] (device), the SAME tensor the
 *                 activation side uses
 *   Wq, Ws   out  u8 [N][K/2], u8 [N][K/32]
 *   workspace     device scratch of at least wush_prepare_weight_workspace(N,K)
 *                 bytes, 16-byte aligned; holds the inverses and a status word.
 * A singular block (no usable pivot) cannot be reported synchronously; it sets
 * a flag in the workspace that wush_workspace_status reads back.
 */
wush_status wush_prepare_weight(const void* W, int64_t N, int64_t K, int64_t ldw,
                                const void* T_blocks, wush_fmt fmt,
                                void* Wq, void* Ws,
                                void* workspace, size_t workspace_bytes, void* stream);

size_t wush_prepare_weight_workspace(int64_t N, int64_t K);

/*
 * Synchronizes `stream`, copies the status word of a workspace last used by
 * wush_prepare_weight (for input size K) to the host and returns WUSH_OK or
 * WUSH_ERR_SINGULAR.  This is the only entry point that blocks.
 */
wush_status wush_workspace_status(const void* workspace, int64_t K, void* stream);

/*
 * Offline construction of the transforms on the device (Alg. 2, RTN case:
 * per-block second moments of the ORIGINAL weight block and of the calibration
 * activations, then Alg. 1: damped Cholesky factors, SVD of W'^T X', and
 * T_wush = H S^(-1/2) U^T W'^T with the normalized Sylvester Hadamard matrix),
 * all in FP64, result rounded to BF16.  Conventions that make T unique:
 * singular values descending, the largest-magnitude entry of every column of U
 * positive.
 *   W        in   bf16 [N][ldw] (device)
 *   X_cal    in   bf16 [M_cal][ldx] (device), calibration tokens
 *   lambda        damping ratio (>= 0): lambda * tr(M)/32 is added to the diagonal
 *   T_blocks out  bf16 [K/32][32][32]
 *   T_f64    out  optional (may be NULL): f64 [K/32][32][32], T before rounding
 *   workspace     device scratch, >= wush_build_transforms_workspace(K) bytes,
 *                 16-byte aligned
 * A moment that is not positive definite after damping sets a flag that
 * wush_build_transforms_status reads back (it synchronizes the stream).
 */
size_t wush_build_transforms_workspace(int64_t K);
wush_status wush_build_transforms(const void* W, int64_t N, int64_t ldw,
                                  const void* X_cal, int64_t M_cal, int64_t ldx,
                                  int64_t K, double lambda,
                                  void* T_blocks, double* T_f64,
                                  void* workspace, size_t workspace_bytes, void* stream);
wush_status wush_build_transforms_status(const void* workspace, int64_t K, void* stream);

/*
 * Offline weight preparation, GPTQ case of Alg. 2: the transforms are built
 * block after block from the second moment of the UPDATED weight block and the
 * diagonal block of the activation Hessian H = M_cal^-1 X_cal^T X_cal (Alg. 1),
 * the transformed block is quantized by the GPTQ subroutine (intra-block error
 * propagation under the transformed block Hessian) and the error, mapped back
 * to the original space, is propagated to the remaining blocks through the
 * Cholesky factor of inv(H + lambda tr(H)/K I).  All in FP64 on the device.
 * Readings of what the paper leaves open: T_i is rounded to BF16 before it is
 * used; the MXFP4 group of an output channel is the block itself and its scale
 * is taken from the transformed weights before any intra-block update (later
 * values saturate); channels of a block are processed in index order.
 *   W        in   bf16 [N][ldw] (device)
 *   X_cal    in   bf16 [M_cal][ldx] (device), calibration tokens
 *   lambda        damping ratio of both the Hessian and Alg. 1
 *   transform_given  0: T_blocks is an OUTPUT (the algorithm above);
 *                 1: T_blocks is an INPUT (e.g. Hadamard or identity blocks) and
 *                 only the GPTQ schedule runs -- the baselines of the paper's tables
 *   T_blocks      bf16 [K/32][32][32]
 *   Wq, Ws   out  packed codes / scales in fmt.layout, as wush_prepare_weight writes
 *   workspace     device scratch, >= wush_prepare_weight_gptq_workspace(N, K)
 *                 bytes (two K x K and one N x K FP64 matrices), 256-byte aligned
 * A Hessian or moment that is not positive definite, or a singular T_i, sets a
 * flag that wush_prepare_weight_gptq_status reads back (it synchronizes).
 */
size_t wush_prepare_weight_gptq_workspace(int64_t N, int64_t K);
wush_status wush_prepare_weight_gptq(const void* W, int64_t N, int64_t K, int64_t ldw,
                                     const void* X_cal, int64_t M_cal, int64_t ldx,
                                     double lambda, int32_t transform_given, wush_fmt fmt,
                                     void* T_blocks, void* Wq, void* Ws,
                                     void* workspace, size_t workspace_bytes, void* stream);
wush_status wush_prepare_weight_gptq_status(const void* workspace, int64_t N, int64_t K, void* stream);

/*
 * MXFP4 x MXFP4 GEMM with FP32 accumulation: the sum over blocks of the layer
 * forward-pass equation, Y = deq(Xq,Xs) . deq(Wq,Ws)^T, on block-scaled MFMA.
 *   Xq, Xs   in   u8 [M][K/2], u8 [M][K/32]
 *   Wq, Ws   in   u8 [N][K/2], u8 [N][K/32]
 *   Y        out  [M][ldy], bf16 (fmt.out_dtype == WUSH_OUT_BF16, rounded to
 *                 nearest even from the FP32 accumulator) or f32
 * ldy >= N (elements); Y aligned to its element size.  The tiled kernel needs
 * Y 16-byte aligned and ldy a multiple of 8; other layouts take a slower
 * general kernel.  In the tiled layout M <= 64 (and M <= 128 unless the layer is
 * very large) takes a weight-streaming kernel
 * (one workgroup per 32 output channels) instead of 256 x 256 tiles.
 */
wush_status wush_linear(const void* Xq, const void* Xs, const void* Wq, const void* Ws,
                        int64_t M, int64_t N, int64_t K, wush_fmt fmt,
                        void* Y, int64_t ldy, void* stream);

/*
 * Decode-sized layer forward in one call (M <= 64 tokens): the whole layer
 * forward-pass equation  Y = sum_i Wq(i)^T q(T(i) X(i))  -- activation transform,
 * MXFP4 quantization and MXFP4 GEMM.  Results are those of wush_quantize_act
 * followed by wush_linear: identical codes and scales, identical FP32
 * accumulation order per output.  The quantized activations live only in the
 * workspace, and the GEMM is the weight-streaming kernel for few tokens.
 * Two forms exist.  The default enqueues two kernels (quantizer, GEMM).  After
 * wush_debug_set(WUSH_DEBUG_DECODE_FUSED, 1) the call is ONE kernel launch:
 * quantization, a grid-wide barrier, then the GEMM, with the weight stream
 * started before the barrier.  On MI355X the barrier across the eight XCDs costs
 * more (4-6 us) than the gap between two kernels of one stream (1.5-2 us), so
 * the single launch only pays where launches are expensive for the caller.
 *   X        in   bf16 [M][ldx] (device), 1 <= M <= 64
 *   T_blocks in   bf16 [K/32][32][32] (device)
 *   Wq, Ws   in   prepared weights in WUSH_LAYOUT_TILED (fmt.layout must say so;
 *                 K % 256 == 0), as written by wush_prepare_weight
 *   Y        out  [M][ldy] bf16 or f32 (fmt.out_dtype), ldy >= N
 *   workspace     device memory, >= wush_layer_decode_workspace(K) bytes, 256-byte
 *                 aligned: the quantized activations and the barrier words.
 *                 wush_layer_decode_init must have run on it once (and again
 *                 after a WUSH_ERR_TIMEOUT); one call at a time per workspace.
 * The single-launch form holds all its workgroups resident (one per CU) and
 * synchronizes them once through the workspace; every wait is bounded.  If a wait
 * expires (the GPU was shared with work that kept this kernel's workgroups from
 * running together) the workgroup sets a flag, Y is left incomplete, and
 * wush_layer_decode_status (which synchronizes the stream) returns
 * WUSH_ERR_TIMEOUT; otherwise WUSH_OK.
 */
size_t wush_layer_decode_workspace(int64_t K);
wush_status wush_layer_decode_init(void* workspace, size_t workspace_bytes, int64_t K, void* stream);
wush_status wush_layer_decode(const void* X, int64_t M, int64_t K, int64_t ldx,
                              const void* T_blocks, const void* Wq, const void* Ws, int64_t N,
                              wush_fmt fmt, void* Y, int64_t ldy,
                              void* workspace, size_t workspace_bytes, void* stream);
wush_status wush_layer_decode_status(const void* workspace, int64_t K, void* stream);

/*
 * wush_layer_decode for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments without the workspace, same results bit for bit (it enqueues
 * the same two kernels: quantizer, weight-streaming GEMM).  The quantized activations
 * live in a fixed device array inside the library (1 088 KiB; each GPU the library runs
 * on holds its own copy until the process ends), which limits K:
 *   K <= 32768, otherwise WUSH_ERR_TOO_LARGE (nothing is launched).
 * The call allocates nothing, frees nothing and needs no init call.  Every call on a GPU
 * uses that GPU's one array: calls that overlap on one GPU (two streams, two threads)
 * race and give undefined results; calls on one stream are ordered and safe.  The array
 * keeps the previous call's contents; no call depends on them.
 */
wush_status wush_layer_decode_static(const void* X, int64_t M, int64_t K, int64_t ldx,
                                     const void* T_blocks, const void* Wq, const void* Ws, int64_t N,
                                     wush_fmt fmt, void* Y, int64_t ldy, void* stream);

/*
 * ---------------------------------------------------------------------------
 * NVFP4 variant (paper: "Layerwise Quantization Loss" and the accuracy tables run
 * the method with NVFP4 as well: group size 16, transform block size matched to
 * the group size).  Format: E2M1 elements; one FP8 E4M3 scale byte (bias 7, no
 * infinities, largest value 448 = 0x7E, never negative) per 16 consecutive
 * channels; one FP32 scale per tensor.  A stored element is worth
 *   E2M1(code) * E4M3(byte) * tensor_scale.
 * Transforms are T16 bf16 [K/16][16][16], T16[b][j][k] as for the 32-blocks.
 * Packed layouts (argument `layout`): WUSH_LAYOUT_CANONICAL: codes u8 [rows][K/2]
 * (even k = low nibble), scales u8 [rows][K/16].  WUSH_LAYOUT_TILED (opaque, fast;
 * K % 64 == 0; buffers hold a multiple of 32 rows, wush_packed_sizes_nvfp4 gives the
 * sizes): the same 16-byte chunks and scale dwords, ordered [row block of 32][K step
 * of 64][half][row] so that a GEMM tile reads contiguous runs; both operands of one
 * wush_linear_nvfp4 call use the same layout; wush_unpack_tiled_nvfp4 converts back.
 * Tensor scales live in DEVICE memory (one float) so that no call has to synchronize.
 * Quantizer (readings of what the paper leaves open): group scale byte =
 * nearest E4M3 (ties to even, saturating) of AbsMax / (6 * tensor_scale);
 * elements = nearest E2M1 (ties to even, saturating) of
 * value / (E4M3(byte) * tensor_scale); the input's sign bit is kept; scale byte 0
 * or tensor scale 0 give magnitude 0.  Each step is one IEEE operation, in FP32
 * for activations and FP64 for weights:
 *   c = 1/(6 ts), r = AbsMax c, d = E4M3(byte) ts, rcp = 1/d, code = E2M1(v rcp).
 * Requirements as above (K % 32 == 0 for the quantizers, K % 64 == 0 for
 * wush_linear_nvfp4, 16-byte aligned data pointers, 4-byte aligned scales).
 * ---------------------------------------------------------------------------
 */

/*
 * Fused activation transform (16 x 16 blocks) + NVFP4 quantization: q(T X) of the
 * layer forward-pass equation.
 *   X            in   bf16 [M][ldx] (device)
 *   T16          in   bf16 [K/16][16][16] (device)
 *   tensor_scale in   float (device): the activation tensor's second-level scale,
 *                     e.g. AbsMax of T X over calibration data / (6 * 448)
 *   Xq, Xs       out  u8 [M][K/2], u8 [M][K/16]
 *   dbg_Yt       out  optional: f32 [M][K], the transformed values as quantized
 */
wush_status wush_quantize_act_nvfp4(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T16,
                                    const float* tensor_scale, int32_t layout, void* Xq, void* Xs,
                                    float* dbg_Yt, void* stream);

/*
 * Offline construction of the 16 x 16 transforms on the device: wush_build_transforms with
 * d = 16 (Alg. 1 per block of 16 channels, Hadamard matrix of order 16).  Same workspace size
 * (wush_build_transforms_workspace) and status call (wush_build_transforms_status).
 *   T16      out  bf16 [K/16][16][16]
 *   T_f64    out  optional: f64 [K/16][16][16], T before rounding
 */
wush_status wush_build_transforms_nvfp4(const void* W, int64_t N, int64_t ldw,
                                        const void* X_cal, int64_t M_cal, int64_t ldx,
                                        int64_t K, double lambda,
                                        void* T16, double* T_f64,
                                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Calibration of the activation tensor scale (offline, on a calibration batch; or online, once
 * before wush_quantize_act_nvfp4, when the batch's own maximum is wanted): AbsMax of T X over
 * the batch / (6 * 448), with the quantizer's own transform arithmetic (BF16 MFMA, FP32
 * accumulators).
 *   X            in   bf16 [M][ldx] (device)
 *   T16          in   bf16 [K/16][16][16] (device)
 *   tensor_scale out  float (device)
 */
wush_status wush_calibrate_act_nvfp4(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T16,
                                     float* tensor_scale, void* stream);

/*
 * Offline weight side in NVFP4 (Alg. 2, RTN case, d = 16): FP64 inverse of every
 * block of T16, W_blk inv(T_b) in FP64, tensor scale = AbsMax of the transformed
 * weights / (6 * 448) rounded to FP32, then the quantizer above in FP64.
 *   W            in   bf16 [N][ldw] (device)
 *   Wq, Ws       out  u8 [N][K/2], u8 [N][K/16]
 *   tensor_scale out  float (device)
 *   workspace         device scratch, >= wush_prepare_weight_nvfp4_workspace(K) bytes,
 *                     16-byte aligned
 * A singular block sets a flag that wush_prepare_weight_nvfp4_status reads back
 * (it synchronizes the stream): WUSH_OK or WUSH_ERR_SINGULAR.
 */
size_t wush_prepare_weight_nvfp4_workspace(int64_t K);
wush_status wush_prepare_weight_nvfp4(const void* W, int64_t N, int64_t K, int64_t ldw, const void* T16,
                                      int32_t layout, void* Wq, void* Ws, float* tensor_scale,
                                      void* workspace, size_t workspace_bytes, void* stream);
wush_status wush_prepare_weight_nvfp4_status(const void* workspace, int64_t K, void* stream);

/*
 * NVFP4 x NVFP4 GEMM, FP32 accumulation: Y = tsx tsw deq(Xq,Xs) . deq(Wq,Ws)^T.
 * CDNA4's block-scaled MFMA has no E4M3-per-16 scale path; element * group scale
 * is exact in FP16, so the kernel dequantizes into LDS and contracts on the FP16
 * MFMA (FP32 accumulators): results differ from the exact product only by the
 * FP32 accumulation order.
 *   Xq, Xs, tsx  in   u8 [M][K/2], u8 [M][K/16] (or tiled), float (device)
 *   Wq, Ws, tsw  in   u8 [N][K/2], u8 [N][K/16] (or tiled), float (device)
 *   layout            of all four packed buffers; the tiled one is about a quarter faster
 *                     (a 256-row tile of a row-major operand touches 256 cache lines per load)
 *   out_dtype         WUSH_OUT_BF16 or WUSH_OUT_F32
 *   Y            out  [M][ldy], ldy >= N, aligned to its element size
 */
wush_status wush_linear_nvfp4(const void* Xq, const void* Xs, const float* tsx,
                              const void* Wq, const void* Ws, const float* tsw,
                              int64_t M, int64_t N, int64_t K, int32_t layout, int32_t out_dtype,
                              void* Y, int64_t ldy, void* stream);

/* Test tap: the NVFP4 quantizer alone on FP32 values. Yt f32 [M][K] -> q, s in `layout`. */
wush_status wush_quantize_f32_nvfp4(const float* Yt, int64_t M, int64_t K, const float* tensor_scale,
                                    int32_t layout, void* q, void* s, void* stream);

/* Buffer sizes (bytes) of a packed NVFP4 [rows][K] operand in `layout`.  Host pointers out. */
wush_status wush_packed_sizes_nvfp4(int64_t rows, int64_t K, int32_t layout,
                                    size_t* code_bytes, size_t* scale_bytes);

/* Tiled -> canonical copy of one packed NVFP4 operand (device pointers); for inspection and tests. */
wush_status wush_unpack_tiled_nvfp4(const void* q_tiled, const void* s_tiled, int64_t rows, int64_t K,
                                    void* q, void* s, void* stream);

/*
 * ---------------------------------------------------------------------------
 * INT4 variant (paper, "Layerwise Quantization Loss" / Table 1: "4-bit integers with
 * Gaussian MSE clipping and BF16 scales of group size 32"; transform blocks of 32 as
 * for MXFP4, same T_blocks tensor).  Codes: two's-complement nibbles -8 .. 7 (even k =
 * low nibble); one BF16 scale per 32 consecutive channels; value = code * scale.
 * Readings: scale = BF16(STEP * root-mean-square of the group), STEP = 0.33860793 = the
 * step that minimizes the mean squared error of this 16-level grid on a unit Gaussian
 * (values beyond -8.5 / 7.5 steps are clipped); code = clip(round-half-even(v / scale));
 * a scale below BF16's normal range is stored as 0 and gives code 0.  One IEEE
 * operation per step, FP32 for activations and FP64 for weights, no fused multiply-add
 * in the sum of squares (channels 0..15 left to right, 16..31 left to right, the two
 * sums added; sigma = sqrt(ss / 32); rcp = 1 / scale; v * rcp rounded).
 * Packed layouts: canonical = codes u8 [rows][K/2], scales u16 [rows][K/32]; tiled = the
 * NVFP4 tiled layout (the 4 scale bytes of a K step of 64 are its two BF16 scales;
 * K % 64 == 0); wush_packed_sizes_nvfp4 / wush_unpack_tiled_nvfp4 serve both formats
 * (same geometry: 4 bits per code, 4 scale bytes per 64 channels).
 * ---------------------------------------------------------------------------
 */
wush_status wush_quantize_act_int4(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T_blocks,
                                   int32_t layout, void* Xq, void* Xs, float* dbg_Yt, void* stream);

/*
 * Offline weight side in INT4 (Alg. 2, RTN case): as wush_prepare_weight (FP64 inverse
 * of every block, W_blk inv(T_b) in FP64), then the quantizer above in FP64.  Workspace
 * and status: wush_prepare_weight_workspace / wush_workspace_status.
 */
wush_status wush_prepare_weight_int4(const void* W, int64_t N, int64_t K, int64_t ldw, const void* T_blocks,
                                     int32_t layout, void* Wq, void* Ws,
                                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * INT4 x INT4 GEMM, FP32 accumulation: Y = deq(Xq,Xs) . deq(Wq,Ws)^T, by the kernel of
 * wush_linear_nvfp4 with another dequantization (code * scale is exact in FP16 while
 * the scale lies in FP16's normal range, 2^-14 .. 8188; smaller scales lose bits below
 * 2^-24, larger ones overflow: rescale the tensor by a power of two beforehand).
 * K % 64 == 0.
 */
wush_status wush_linear_int4(const void* Xq, const void* Xs, const void* Wq, const void* Ws,
                             int64_t M, int64_t N, int64_t K, int32_t layout, int32_t out_dtype,
                             void* Y, int64_t ldy, void* stream);

/* Test tap: the INT4 quantizer alone on FP32 values. Yt f32 [M][K] -> q, s in `layout`. */
wush_status wush_quantize_f32_int4(const float* Yt, int64_t M, int64_t K, int32_t layout,
                                   void* q, void* s, void* stream);

/*
 * Test tap: the quantizer alone on FP32 values (same device function the fused
 * kernel uses).  Yt f32 [M][K] (device) -> q u8 [M][K/2], s u8 [M][K/32].
 */
wush_status wush_quantize_f32(const float* Yt, int64_t M, int64_t K, wush_fmt fmt,
                              void* q, void* s, void* stream);

/*
 * Buffer sizes (bytes) of the packed codes and scales of a [rows][K] operand
 * in the layout fmt.layout (quantizer outputs, wush_linear inputs).  Host
 * pointers out.
 */
wush_status wush_packed_sizes(int64_t rows, int64_t K, wush_fmt fmt,
                              size_t* code_bytes, size_t* scale_bytes);

/*
 * Tiled -> canonical copy of one packed operand (device pointers; q, s are
 * canonical u8 [rows][K/2], u8 [rows][K/32]).  For inspection and tests: the
 * hot path never needs it.
 */
wush_status wush_unpack_tiled(const void* q_tiled, const void* s_tiled, int64_t rows, int64_t K,
                              void* q, void* s, void* stream);

/*
 * Switches for tests and measurements: which kernel or tile shape a call takes where the
 * library would otherwise choose by itself.  Process-wide, read by every later call on any
 * thread; value -1 restores the library's own choice.  Results do not depend on them beyond
 * the accumulation order of a GEMM; nothing reads the environment.
 *   WUSH_DEBUG_GEMM_TILE            wush_linear, tiled layout: 0..3 = 256x256, 128x384, 128x256, 128x128 tiles
 *   WUSH_DEBUG_GEMM_SKINNY          wush_linear up to 128 tokens: 1 = weight-streaming kernel, 0 = tiled kernel
 *   WUSH_DEBUG_GEMM_SIMPLE          wush_linear, canonical layout: 1 = the general one-wave-per-tile kernel
 *   WUSH_DEBUG_W4_WIDTH             wush_linear_nvfp4 / _int4: tile width 2..4 (x 64 output channels)
 *   WUSH_DEBUG_W4_SKINNY            wush_linear_nvfp4 / _int4 up to 128 tokens: 0 = tiled kernel; weight-streaming kernel with
 *                                   1 = K split over a workgroup's waves, 2 = activations shared through LDS (65..128 tokens;
 *                                   with fewer it is 1)
 *   WUSH_DEBUG_DECODE_FUSED         wush_layer_decode: 1 = one launch with a grid-wide barrier
 *   WUSH_DEBUG_DECODE_TEST_TIMEOUT  wush_layer_decode: 1 = the barrier wait gives up at once (error-path test)
 * Returns WUSH_ERR_FMT for an unknown option, WUSH_ERR_SHAPE for a value outside -1 .. 1023.
 */
enum {
  WUSH_DEBUG_GEMM_TILE = 0, WUSH_DEBUG_GEMM_SKINNY = 1, WUSH_DEBUG_GEMM_SIMPLE = 2, WUSH_DEBUG_W4_WIDTH = 3,
  WUSH_DEBUG_W4_SKINNY = 4, WUSH_DEBUG_DECODE_FUSED = 5, WUSH_DEBUG_DECODE_TEST_TIMEOUT = 6
};
wush_status wush_debug_set(int32_t option, int32_t value);

/* Human-readable name of a status code; static storage, never NULL. */
const char* wush_status_string(wush_status st);

/* Library version, "major.minor"; static storage. */
const char* wush_version(void);

#ifdef __cplusplus
}
#endif
#endif /* WUSH_H_ */
