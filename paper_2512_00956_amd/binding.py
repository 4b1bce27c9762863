"""ctypes binding of include/wush.h: argument marshalling only.

Tensor arguments are torch tensors on the GPU (torch is used for device memory
and streams); each wrapper passes `data_ptr()`s, sizes and the current HIP
stream to the C entry point of the same name and raises `WushError` on a
non-zero status.  No fallback exists: if `libwush.so` is missing the first call
raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_double, c_int32, c_int64, c_size_t, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libwush.so"

WUSH_SCALE_NOSAT, WUSH_SCALE_OCP_FLOOR = 0, 1
WUSH_OUT_BF16, WUSH_OUT_F32 = 0, 1
WUSH_LAYOUT_CANONICAL, WUSH_LAYOUT_TILED = 0, 1
(WUSH_DEBUG_GEMM_TILE, WUSH_DEBUG_GEMM_SKINNY, WUSH_DEBUG_GEMM_SIMPLE, WUSH_DEBUG_W4_WIDTH, WUSH_DEBUG_W4_SKINNY,
 WUSH_DEBUG_DECODE_FUSED, WUSH_DEBUG_DECODE_TEST_TIMEOUT) = range(7)

STATUS_NAMES = {
    0: "WUSH_OK", 1: "WUSH_ERR_NULL", 2: "WUSH_ERR_SHAPE", 3: "WUSH_ERR_ALIGN", 4: "WUSH_ERR_FMT",
    5: "WUSH_ERR_WORKSPACE", 6: "WUSH_ERR_DEVICE", 7: "WUSH_ERR_SINGULAR", 8: "WUSH_ERR_TIMEOUT",
    9: "WUSH_ERR_TOO_LARGE",
}

# every symbol include/wush.h declares
EXPORTS = (
    "wush_default_fmt", "wush_quantize_act", "wush_prepare_weight", "wush_prepare_weight_workspace",
    "wush_workspace_status", "wush_linear", "wush_quantize_f32", "wush_status_string", "wush_version",
    "wush_packed_sizes", "wush_unpack_tiled",
    "wush_build_transforms", "wush_build_transforms_workspace", "wush_build_transforms_status",
    "wush_layer_decode", "wush_layer_decode_workspace", "wush_layer_decode_init", "wush_layer_decode_status",
    "wush_layer_decode_static", "wush_debug_set",
    "wush_prepare_weight_gptq", "wush_prepare_weight_gptq_workspace", "wush_prepare_weight_gptq_status",
    "wush_quantize_act_nvfp4", "wush_prepare_weight_nvfp4", "wush_prepare_weight_nvfp4_workspace",
    "wush_prepare_weight_nvfp4_status", "wush_linear_nvfp4", "wush_quantize_f32_nvfp4",
    "wush_packed_sizes_nvfp4", "wush_unpack_tiled_nvfp4",
    "wush_calibrate_act_nvfp4", "wush_build_transforms_nvfp4",
    "wush_quantize_act_int4", "wush_prepare_weight_int4", "wush_linear_int4", "wush_quantize_f32_int4",
)


class WushFmt(ctypes.Structure):
    _fields_ = [("block", c_int32), ("elem", c_int32), ("scale", c_int32),
                ("scale_rule", c_int32), ("out_dtype", c_int32), ("layout", c_int32)]


class WushError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {STATUS_NAMES.get(code, code)} ({wush_status_string(code)})")


_lib = None


def lib_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def lib() -> ctypes.CDLL:
    """The loaded C library (loads it on first use)."""
    global _lib
    if _lib is None:
        p = lib_path()
        if not os.path.exists(p):
            raise RuntimeError(
                f"{p} not found: build it first (python -m paper_2512_00956_amd.build); "
                "there is no fallback path")
        L = ctypes.CDLL(p)
        L.wush_default_fmt.restype = WushFmt
        L.wush_default_fmt.argtypes = []
        L.wush_quantize_act.restype = c_int32
        L.wush_quantize_act.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, WushFmt,
                                        c_void_p, c_void_p, c_void_p, c_void_p]
        L.wush_prepare_weight.restype = c_int32
        L.wush_prepare_weight.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, WushFmt,
                                          c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
        L.wush_prepare_weight_workspace.restype = c_size_t
        L.wush_prepare_weight_workspace.argtypes = [c_int64, c_int64]
        L.wush_workspace_status.restype = c_int32
        L.wush_workspace_status.argtypes = [c_void_p, c_int64, c_void_p]
        L.wush_linear.restype = c_int32
        L.wush_linear.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64,
                                  WushFmt, c_void_p, c_int64, c_void_p]
        L.wush_quantize_f32.restype = c_int32
        L.wush_quantize_f32.argtypes = [c_void_p, c_int64, c_int64, WushFmt, c_void_p, c_void_p, c_void_p]
        L.wush_status_string.restype = c_char_p
        L.wush_status_string.argtypes = [c_int32]
        L.wush_version.restype = c_char_p
        L.wush_version.argtypes = []
        L.wush_build_transforms_workspace.restype = c_size_t
        L.wush_build_transforms_workspace.argtypes = [c_int64]
        L.wush_build_transforms.restype = c_int32
        L.wush_build_transforms.argtypes = [c_void_p, c_int64, c_int64, c_void_p, c_int64, c_int64, c_int64, c_double,
                                            c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
        L.wush_build_transforms_status.restype = c_int32
        L.wush_build_transforms_status.argtypes = [c_void_p, c_int64, c_void_p]
        L.wush_packed_sizes.restype = c_int32
        L.wush_packed_sizes.argtypes = [c_int64, c_int64, WushFmt, POINTER(c_size_t), POINTER(c_size_t)]
        L.wush_unpack_tiled.restype = c_int32
        L.wush_unpack_tiled.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_void_p, c_void_p, c_void_p]
        L.wush_layer_decode_workspace.restype = c_size_t
        L.wush_layer_decode_workspace.argtypes = [c_int64]
        L.wush_layer_decode_init.restype = c_int32
        L.wush_layer_decode_init.argtypes = [c_void_p, c_size_t, c_int64, c_void_p]
        L.wush_layer_decode.restype = c_int32
        L.wush_layer_decode.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_int64,
                                        WushFmt, c_void_p, c_int64, c_void_p, c_size_t, c_void_p]
        L.wush_layer_decode_static.restype = c_int32
        L.wush_layer_decode_static.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_int64,
                                               WushFmt, c_void_p, c_int64, c_void_p]
        L.wush_debug_set.restype = c_int32
        L.wush_debug_set.argtypes = [c_int32, c_int32]
        L.wush_layer_decode_status.restype = c_int32
        L.wush_layer_decode_status.argtypes = [c_void_p, c_int64, c_void_p]
        L.wush_prepare_weight_gptq_workspace.restype = c_size_t
        L.wush_prepare_weight_gptq_workspace.argtypes = [c_int64, c_int64]
        L.wush_prepare_weight_gptq.restype = c_int32
        L.wush_prepare_weight_gptq.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, c_int64, c_int64, c_double,
                                               c_int32, WushFmt, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t,
                                               c_void_p]
        L.wush_prepare_weight_gptq_status.restype = c_int32
        L.wush_prepare_weight_gptq_status.argtypes = [c_void_p, c_int64, c_int64, c_void_p]
        L.wush_quantize_act_int4.restype = c_int32
        L.wush_quantize_act_int4.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, c_int32, c_void_p, c_void_p,
                                             c_void_p, c_void_p]
        L.wush_prepare_weight_int4.restype = c_int32
        L.wush_prepare_weight_int4.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, c_int32, c_void_p, c_void_p,
                                               c_void_p, c_size_t, c_void_p]
        L.wush_linear_int4.restype = c_int32
        L.wush_linear_int4.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int32,
                                       c_int32, c_void_p, c_int64, c_void_p]
        L.wush_quantize_f32_int4.restype = c_int32
        L.wush_quantize_f32_int4.argtypes = [c_void_p, c_int64, c_int64, c_int32, c_void_p, c_void_p, c_void_p]
        L.wush_build_transforms_nvfp4.restype = c_int32
        L.wush_build_transforms_nvfp4.argtypes = L.wush_build_transforms.argtypes
        L.wush_calibrate_act_nvfp4.restype = c_int32
        L.wush_calibrate_act_nvfp4.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, c_void_p, c_void_p]
        L.wush_quantize_act_nvfp4.restype = c_int32
        L.wush_quantize_act_nvfp4.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, c_void_p, c_int32, c_void_p,
                                              c_void_p, c_void_p, c_void_p]
        L.wush_prepare_weight_nvfp4_workspace.restype = c_size_t
        L.wush_prepare_weight_nvfp4_workspace.argtypes = [c_int64]
        L.wush_prepare_weight_nvfp4.restype = c_int32
        L.wush_prepare_weight_nvfp4.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, c_int32, c_void_p, c_void_p,
                                                c_void_p, c_void_p, c_size_t, c_void_p]
        L.wush_prepare_weight_nvfp4_status.restype = c_int32
        L.wush_prepare_weight_nvfp4_status.argtypes = [c_void_p, c_int64, c_void_p]
        L.wush_linear_nvfp4.restype = c_int32
        L.wush_linear_nvfp4.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64,
                                        c_int64, c_int32, c_int32, c_void_p, c_int64, c_void_p]
        L.wush_quantize_f32_nvfp4.restype = c_int32
        L.wush_quantize_f32_nvfp4.argtypes = [c_void_p, c_int64, c_int64, c_void_p, c_int32, c_void_p, c_void_p, c_void_p]
        L.wush_packed_sizes_nvfp4.restype = c_int32
        L.wush_packed_sizes_nvfp4.argtypes = [c_int64, c_int64, c_int32, POINTER(c_size_t), POINTER(c_size_t)]
        L.wush_unpack_tiled_nvfp4.restype = c_int32
        L.wush_unpack_tiled_nvfp4.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_void_p, c_void_p, c_void_p]
        _lib = L
    return _lib


def default_fmt(scale_rule: int = WUSH_SCALE_NOSAT, out_dtype: int = WUSH_OUT_BF16,
                layout: int = WUSH_LAYOUT_CANONICAL) -> WushFmt:
    f = lib().wush_default_fmt()
    f.scale_rule = scale_rule
    f.out_dtype = out_dtype
    f.layout = layout
    return f


def wush_packed_sizes(rows: int, K: int, fmt: WushFmt | None = None):
    """(code_bytes, scale_bytes) of a packed [rows][K] operand in fmt.layout."""
    cb, sb = c_size_t(0), c_size_t(0)
    _check(lib().wush_packed_sizes(rows, K, fmt or default_fmt(), ctypes.byref(cb), ctypes.byref(sb)),
           "wush_packed_sizes")
    return cb.value, sb.value


def wush_unpack_tiled(q_tiled, s_tiled, rows: int, K: int, q, s, stream=None):
    """Tiled -> canonical copy (q u8 [rows][K/2], s u8 [rows][K/32])."""
    _check(lib().wush_unpack_tiled(_ptr(q_tiled), _ptr(s_tiled), rows, K, _ptr(q), _ptr(s), _stream(stream)),
           "wush_unpack_tiled")


def wush_debug_set(option: int, value: int):
    """Test / measurement switch (WUSH_DEBUG_*): force a kernel or tile shape; value -1 = the library's choice."""
    _check(lib().wush_debug_set(int(option), int(value)), "wush_debug_set")


def wush_status_string(code: int) -> str:
    return lib().wush_status_string(int(code)).decode()


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return c_void_p(torch.cuda.current_stream().cuda_stream)
    return c_void_p(stream if isinstance(stream, int) else stream.cuda_stream)


def _check(code: int, where: str):
    if code != 0:
        raise WushError(code, where)


def wush_quantize_act(X, T_blocks, Xq, Xs, fmt: WushFmt | None = None, dbg_Yt=None, stream=None):
    """X bf16 [M][K] (row stride X.stride(0)), T_blocks bf16 [K/32][32][32] ->
    Xq u8 [M][K/2], Xs u8 [M][K/32] (pre-allocated by the caller)."""
    M, K = X.shape
    _check(lib().wush_quantize_act(_ptr(X), M, K, X.stride(0), _ptr(T_blocks), fmt or default_fmt(),
                                   _ptr(Xq), _ptr(Xs), _ptr(dbg_Yt), _stream(stream)), "wush_quantize_act")


def wush_prepare_weight_workspace(N: int, K: int) -> int:
    return int(lib().wush_prepare_weight_workspace(N, K))


def wush_prepare_weight(W, T_blocks, Wq, Ws, workspace, fmt: WushFmt | None = None, stream=None):
    """W bf16 [N][K] -> Wq u8 [N][K/2], Ws u8 [N][K/32]; workspace: u8 tensor of
    at least wush_prepare_weight_workspace(N, K) bytes."""
    N, K = W.shape
    _check(lib().wush_prepare_weight(_ptr(W), N, K, W.stride(0), _ptr(T_blocks), fmt or default_fmt(),
                                     _ptr(Wq), _ptr(Ws), _ptr(workspace),
                                     0 if workspace is None else workspace.numel() * workspace.element_size(),
                                     _stream(stream)), "wush_prepare_weight")


def wush_workspace_status(workspace, K: int, stream=None):
    _check(lib().wush_workspace_status(_ptr(workspace), K, _stream(stream)), "wush_workspace_status")


def wush_linear(Xq, Xs, Wq, Ws, Y, fmt: WushFmt | None = None, stream=None, K: int | None = None):
    """Y [M][N] (bf16 or f32 per fmt.out_dtype, row stride Y.stride(0)) =
    deq(Xq, Xs) . deq(Wq, Ws)^T.  M and N come from Y; K from the canonical
    shape of Xq unless given (the tiled layout has no 2-D shape to read it from)."""
    M, N = Y.shape
    if K is None:
        K = 2 * Xq.shape[-1]
    _check(lib().wush_linear(_ptr(Xq), _ptr(Xs), _ptr(Wq), _ptr(Ws), M, N, K, fmt or default_fmt(),
                             _ptr(Y), Y.stride(0), _stream(stream)), "wush_linear")


def wush_build_transforms_workspace(K: int) -> int:
    return int(lib().wush_build_transforms_workspace(K))


def wush_build_transforms(W, X_cal, lam: float, T_blocks, workspace, T_f64=None, stream=None):
    """Alg. 1 + Alg. 2 (RTN case) on the device: W bf16 [N][K], X_cal bf16 [M_cal][K]
    -> T_blocks bf16 [K/32][32][32] (and the unrounded f64 T if T_f64 is given)."""
    N, K = W.shape
    Mc = X_cal.shape[0]
    _check(lib().wush_build_transforms(_ptr(W), N, W.stride(0), _ptr(X_cal), Mc, X_cal.stride(0), K, float(lam),
                                       _ptr(T_blocks), _ptr(T_f64), _ptr(workspace),
                                       0 if workspace is None else workspace.numel() * workspace.element_size(),
                                       _stream(stream)), "wush_build_transforms")


def wush_build_transforms_nvfp4(W, X_cal, lam: float, T16, workspace, T_f64=None, stream=None):
    """The same with 16 x 16 blocks (NVFP4 variant): -> T16 bf16 [K/16][16][16]."""
    N, K = W.shape
    Mc = X_cal.shape[0]
    _check(lib().wush_build_transforms_nvfp4(_ptr(W), N, W.stride(0), _ptr(X_cal), Mc, X_cal.stride(0), K, float(lam),
                                             _ptr(T16), _ptr(T_f64), _ptr(workspace),
                                             0 if workspace is None else workspace.numel() * workspace.element_size(),
                                             _stream(stream)), "wush_build_transforms_nvfp4")


def wush_build_transforms_status(workspace, K: int, stream=None):
    _check(lib().wush_build_transforms_status(_ptr(workspace), K, _stream(stream)), "wush_build_transforms_status")


def wush_quantize_f32(Yt, q, s, fmt: WushFmt | None = None, stream=None):
    """Quantizer-only test tap: Yt f32 [M][K] -> q u8 [M][K/2], s u8 [M][K/32]."""
    M, K = Yt.shape
    _check(lib().wush_quantize_f32(_ptr(Yt), M, K, fmt or default_fmt(), _ptr(q), _ptr(s), _stream(stream)),
           "wush_quantize_f32")


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def wush_layer_decode_workspace(K: int) -> int:
    return int(lib().wush_layer_decode_workspace(K))


def wush_layer_decode_init(workspace, K: int, stream=None):
    """Zero the barrier words of a wush_layer_decode workspace (once after allocation)."""
    _check(lib().wush_layer_decode_init(_ptr(workspace), _nbytes(workspace), K, _stream(stream)),
           "wush_layer_decode_init")


def wush_layer_decode(X, T_blocks, Wq, Ws, Y, workspace, fmt: WushFmt | None = None, stream=None):
    """One-launch layer forward for M <= 64 tokens: X bf16 [M][K], prepared tiled
    weights Wq/Ws -> Y [M][N] (N from Y)."""
    M, K = X.shape
    N = Y.shape[1]
    _check(lib().wush_layer_decode(_ptr(X), M, K, X.stride(0), _ptr(T_blocks), _ptr(Wq), _ptr(Ws), N,
                                   fmt or default_fmt(layout=WUSH_LAYOUT_TILED), _ptr(Y), Y.stride(0),
                                   _ptr(workspace), _nbytes(workspace), _stream(stream)), "wush_layer_decode")


def wush_layer_decode_static(X, T_blocks, Wq, Ws, Y, fmt: WushFmt | None = None, stream=None):
    """wush_layer_decode without a workspace (K <= 32768): the library's own fixed scratch holds the
    quantized activations; allocates nothing."""
    M, K = X.shape
    N = Y.shape[1]
    _check(lib().wush_layer_decode_static(_ptr(X), M, K, X.stride(0), _ptr(T_blocks), _ptr(Wq), _ptr(Ws), N,
                                          fmt or default_fmt(layout=WUSH_LAYOUT_TILED), _ptr(Y), Y.stride(0),
                                          _stream(stream)), "wush_layer_decode_static")


def wush_layer_decode_status(workspace, K: int, stream=None):
    _check(lib().wush_layer_decode_status(_ptr(workspace), K, _stream(stream)), "wush_layer_decode_status")


def wush_prepare_weight_gptq_workspace(N: int, K: int) -> int:
    return int(lib().wush_prepare_weight_gptq_workspace(N, K))


def wush_prepare_weight_gptq(W, X_cal, lam: float, T_blocks, Wq, Ws, workspace, fmt: WushFmt | None = None,
                             transform_given: bool = False, stream=None):
    """Alg. 2, GPTQ case: W bf16 [N][K], X_cal bf16 [M_cal][K] -> T_blocks (output unless
    transform_given), Wq, Ws."""
    N, K = W.shape
    _check(lib().wush_prepare_weight_gptq(_ptr(W), N, K, W.stride(0), _ptr(X_cal), X_cal.shape[0], X_cal.stride(0),
                                          float(lam), int(bool(transform_given)), fmt or default_fmt(), _ptr(T_blocks),
                                          _ptr(Wq), _ptr(Ws), _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "wush_prepare_weight_gptq")


def wush_prepare_weight_gptq_status(workspace, N: int, K: int, stream=None):
    _check(lib().wush_prepare_weight_gptq_status(_ptr(workspace), N, K, _stream(stream)),
           "wush_prepare_weight_gptq_status")


# ---------------------------------------------------------------------------
# NVFP4 variant (E2M1, E4M3 scale per 16, FP32 tensor scale held in a 1-element
# float tensor on the GPU; transforms bf16 [K/16][16][16]).  `layout`:
# WUSH_LAYOUT_CANONICAL (default) or WUSH_LAYOUT_TILED.
# ---------------------------------------------------------------------------
def wush_quantize_act_nvfp4(X, T16, tensor_scale, Xq, Xs, layout: int = WUSH_LAYOUT_CANONICAL, dbg_Yt=None,
                            stream=None):
    """X bf16 [M][K] -> Xq u8 [M][K/2], Xs u8 [M][K/16] (canonical shapes); tensor_scale: float32 tensor
    (1 element, GPU)."""
    M, K = X.shape
    _check(lib().wush_quantize_act_nvfp4(_ptr(X), M, K, X.stride(0), _ptr(T16), _ptr(tensor_scale), layout, _ptr(Xq),
                                         _ptr(Xs), _ptr(dbg_Yt), _stream(stream)), "wush_quantize_act_nvfp4")


def wush_calibrate_act_nvfp4(X, T16, tensor_scale, stream=None):
    """tensor_scale (float32 tensor, 1 element, written) = AbsMax of T X over the batch / (6 * 448)."""
    M, K = X.shape
    _check(lib().wush_calibrate_act_nvfp4(_ptr(X), M, K, X.stride(0), _ptr(T16), _ptr(tensor_scale), _stream(stream)),
           "wush_calibrate_act_nvfp4")


def wush_prepare_weight_nvfp4_workspace(K: int) -> int:
    return int(lib().wush_prepare_weight_nvfp4_workspace(K))


def wush_prepare_weight_nvfp4(W, T16, Wq, Ws, tensor_scale, workspace, layout: int = WUSH_LAYOUT_CANONICAL,
                              stream=None):
    """W bf16 [N][K] -> Wq, Ws in `layout`, tensor_scale (float32 tensor, 1 element, written)."""
    N, K = W.shape
    _check(lib().wush_prepare_weight_nvfp4(_ptr(W), N, K, W.stride(0), _ptr(T16), layout, _ptr(Wq), _ptr(Ws),
                                           _ptr(tensor_scale), _ptr(workspace),
                                           0 if workspace is None else workspace.numel() * workspace.element_size(),
                                           _stream(stream)), "wush_prepare_weight_nvfp4")


def wush_prepare_weight_nvfp4_status(workspace, K: int, stream=None):
    _check(lib().wush_prepare_weight_nvfp4_status(_ptr(workspace), K, _stream(stream)),
           "wush_prepare_weight_nvfp4_status")


def wush_linear_nvfp4(Xq, Xs, tsx, Wq, Ws, tsw, Y, layout: int = WUSH_LAYOUT_CANONICAL,
                      out_dtype: int = WUSH_OUT_BF16, stream=None, K: int | None = None):
    """Y [M][N] = tsx tsw deq(Xq, Xs) . deq(Wq, Ws)^T; K from the canonical shape of Xq unless given."""
    M, N = Y.shape
    if K is None:
        K = 2 * Xq.shape[-1]
    _check(lib().wush_linear_nvfp4(_ptr(Xq), _ptr(Xs), _ptr(tsx), _ptr(Wq), _ptr(Ws), _ptr(tsw), M, N, K, layout,
                                   out_dtype, _ptr(Y), Y.stride(0), _stream(stream)), "wush_linear_nvfp4")


def wush_quantize_f32_nvfp4(Yt, tensor_scale, q, s, layout: int = WUSH_LAYOUT_CANONICAL, stream=None):
    M, K = Yt.shape
    _check(lib().wush_quantize_f32_nvfp4(_ptr(Yt), M, K, _ptr(tensor_scale), layout, _ptr(q), _ptr(s),
                                         _stream(stream)), "wush_quantize_f32_nvfp4")


def wush_packed_sizes_nvfp4(rows: int, K: int, layout: int = WUSH_LAYOUT_CANONICAL):
    """(code_bytes, scale_bytes) of a packed NVFP4 [rows][K] operand in `layout`."""
    cb, sb = c_size_t(0), c_size_t(0)
    _check(lib().wush_packed_sizes_nvfp4(rows, K, layout, ctypes.byref(cb), ctypes.byref(sb)),
           "wush_packed_sizes_nvfp4")
    return cb.value, sb.value


def wush_unpack_tiled_nvfp4(q_tiled, s_tiled, rows: int, K: int, q, s, stream=None):
    """Tiled -> canonical copy (q u8 [rows][K/2], s u8 [rows][K/16])."""
    _check(lib().wush_unpack_tiled_nvfp4(_ptr(q_tiled), _ptr(s_tiled), rows, K, _ptr(q), _ptr(s), _stream(stream)),
           "wush_unpack_tiled_nvfp4")


# ---------------------------------------------------------------------------
# INT4 variant (two's-complement codes, BF16 scale per 32; transforms bf16 [K/32][32][32]).
# Packed sizes / unpacking: wush_packed_sizes_nvfp4, wush_unpack_tiled_nvfp4 (same geometry).
# ---------------------------------------------------------------------------
def wush_quantize_act_int4(X, T_blocks, Xq, Xs, layout: int = WUSH_LAYOUT_CANONICAL, dbg_Yt=None, stream=None):
    """X bf16 [M][K] -> Xq u8 [M][K/2], Xs: BF16 scales [M][K/32] (2 bytes each; canonical shapes)."""
    M, K = X.shape
    _check(lib().wush_quantize_act_int4(_ptr(X), M, K, X.stride(0), _ptr(T_blocks), layout, _ptr(Xq), _ptr(Xs),
                                        _ptr(dbg_Yt), _stream(stream)), "wush_quantize_act_int4")


def wush_prepare_weight_int4(W, T_blocks, Wq, Ws, workspace, layout: int = WUSH_LAYOUT_CANONICAL, stream=None):
    """W bf16 [N][K] -> Wq, Ws in `layout`; workspace as for wush_prepare_weight."""
    N, K = W.shape
    _check(lib().wush_prepare_weight_int4(_ptr(W), N, K, W.stride(0), _ptr(T_blocks), layout, _ptr(Wq), _ptr(Ws),
                                          _ptr(workspace),
                                          0 if workspace is None else workspace.numel() * workspace.element_size(),
                                          _stream(stream)), "wush_prepare_weight_int4")


def wush_linear_int4(Xq, Xs, Wq, Ws, Y, layout: int = WUSH_LAYOUT_CANONICAL, out_dtype: int = WUSH_OUT_BF16,
                     stream=None, K: int | None = None):
    """Y [M][N] = deq(Xq, Xs) . deq(Wq, Ws)^T; K from the canonical shape of Xq unless given."""
    M, N = Y.shape
    if K is None:
        K = 2 * Xq.shape[-1]
    _check(lib().wush_linear_int4(_ptr(Xq), _ptr(Xs), _ptr(Wq), _ptr(Ws), M, N, K, layout, out_dtype, _ptr(Y),
                                  Y.stride(0), _stream(stream)), "wush_linear_int4")


def wush_quantize_f32_int4(Yt, q, s, layout: int = WUSH_LAYOUT_CANONICAL, stream=None):
    M, K = Yt.shape
    _check(lib().wush_quantize_f32_int4(_ptr(Yt), M, K, layout, _ptr(q), _ptr(s), _stream(stream)),
           "wush_quantize_f32_int4")
