"""MI355X-native W4A4 WUSH linear-layer hot path.

The package is a thin ctypes binding over the C-ABI library `libwush.so`
(hand-written HIP kernels for gfx950).  Nothing here computes: every step of the
path runs inside the library.  Importing the package does not load the
library; the first call does, and fails loudly if it has not been built.
"""
from .binding import (  # noqa: F401
    WushError,
    WushFmt,
    default_fmt,
    lib,
    lib_path,
    wush_build_transforms,
    wush_build_transforms_nvfp4,
    wush_build_transforms_status,
    wush_build_transforms_workspace,
    wush_calibrate_act_nvfp4,
    wush_layer_decode,
    wush_layer_decode_init,
    wush_layer_decode_static,
    wush_layer_decode_status,
    wush_layer_decode_workspace,
    wush_linear,
    wush_linear_int4,
    wush_linear_nvfp4,
    wush_packed_sizes,
    wush_packed_sizes_nvfp4,
    wush_unpack_tiled,
    wush_unpack_tiled_nvfp4,
    wush_prepare_weight,
    wush_prepare_weight_gptq,
    wush_prepare_weight_gptq_status,
    wush_prepare_weight_gptq_workspace,
    wush_prepare_weight_int4,
    wush_prepare_weight_nvfp4,
    wush_prepare_weight_nvfp4_status,
    wush_prepare_weight_nvfp4_workspace,
    wush_prepare_weight_workspace,
    wush_quantize_act,
    wush_quantize_act_int4,
    wush_quantize_act_nvfp4,
    wush_quantize_f32,
    wush_quantize_f32_int4,
    wush_quantize_f32_nvfp4,
    wush_status_string,
    wush_workspace_status,
)

__all__ = [
    "WushError", "WushFmt", "default_fmt", "lib", "lib_path", "wush_linear", "wush_prepare_weight",
    "wush_prepare_weight_workspace", "wush_quantize_act", "wush_quantize_f32", "wush_status_string",
    "wush_workspace_status", "wush_packed_sizes", "wush_unpack_tiled", "wush_build_transforms",
    "wush_build_transforms_status", "wush_build_transforms_workspace", "wush_layer_decode",
    "wush_layer_decode_init", "wush_layer_decode_static", "wush_layer_decode_status", "wush_layer_decode_workspace",
    "wush_prepare_weight_gptq", "wush_prepare_weight_gptq_status", "wush_prepare_weight_gptq_workspace",
    "wush_quantize_act_nvfp4", "wush_prepare_weight_nvfp4", "wush_prepare_weight_nvfp4_status",
    "wush_prepare_weight_nvfp4_workspace", "wush_linear_nvfp4", "wush_quantize_f32_nvfp4",
    "wush_packed_sizes_nvfp4", "wush_unpack_tiled_nvfp4", 
    "wush_calibrate_act_nvfp4", "wush_build_transforms_nvfp4", "wush_quantize_act_int4", "wush_prepare_weight_int4", "wush_linear_int4", "wush_quantize_f32_int4",
]
