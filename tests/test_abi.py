"""C-ABI checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before any launch (so fake,
never-dereferenced device addresses are enough here)."""
import ctypes
import os
import re

import pytest

import paper_2512_00956_amd as P
from paper_2512_00956_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(P.lib_path()):
        from paper_2512_00956_amd.build import build
        build()
    return P.lib()


def test_header_symbols_are_exported(L):
    text = open(os.path.join(ROOT, "include", "wush.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(wush_[a-z0-9_]+)\s*\(", text))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None
    assert L.wush_version() == b"0.10"


def test_default_fmt_and_status_strings(L):
    f = P.default_fmt()
    assert (f.block, f.elem, f.scale, f.scale_rule, f.out_dtype, f.layout) == (32, 1, 1, 0, 0, 0)
    names = {P.wush_status_string(c) for c in range(9)}
    assert len(names) == 9 and "ok" in names
    assert P.wush_status_string(99) == "unknown status"


A = 0x10000  # a 16-byte aligned fake address; never dereferenced on error paths


def test_quantize_act_validation(L):
    f = P.default_fmt()
    q = lambda *a: L.wush_quantize_act(*a)
    assert q(None, 4, 64, 64, A, f, A, A, None, None) == 1          # null X
    assert q(A, 4, 64, 64, None, f, A, A, None, None) == 1          # null T
    assert q(A, 4, 64, 64, A, f, None, A, None, None) == 1
    assert q(A, 0, 64, 64, A, f, A, A, None, None) == 2             # M = 0
    assert q(A, 4, 48, 48, A, f, A, A, None, None) == 2             # K % 32
    assert q(A, 4, 64, 56, A, f, A, A, None, None) == 2             # ldx < K
    assert q(A, 4, 64, 68, A, f, A, A, None, None) == 2             # ldx % 8
    assert q(A + 2, 4, 64, 64, A, f, A, A, None, None) == 3         # misaligned
    assert q(A, 4, 64, 64, A, f, A, A + 8, None, None) == 3
    assert q(A, 4, 64, 64, A, f, A, A, A + 4, None) == 3            # misaligned debug tap
    t = P.default_fmt(layout=1)
    assert q(A, 4, 128, 128, A, t, A, A, None, None) == 2           # tiled layout needs K % 256 == 0
    for field, val in (("block", 16), ("elem", 2), ("scale", 0), ("scale_rule", 2), ("out_dtype", 5), ("layout", 2)):
        g = P.default_fmt()
        setattr(g, field, val)
        assert q(A, 4, 64, 64, A, g, A, A, None, None) == 4


def test_prepare_weight_validation(L):
    f = P.default_fmt()
    need = L.wush_prepare_weight_workspace(8, 64)
    assert need >= 2 * 32 * 32 * 8 + 4
    assert L.wush_prepare_weight_workspace(8, 48) == 0
    w = lambda *a: L.wush_prepare_weight(*a)
    assert w(A, 8, 64, 64, A, f, A, A, None, need, None) == 5       # no workspace
    assert w(A, 8, 64, 64, A, f, A, A, A, need - 1, None) == 5      # too small
    assert w(A, 8, 64, 64, A, f, A, A, A + 4, need, None) == 3
    assert w(None, 8, 64, 64, A, f, A, A, A, need, None) == 1
    assert w(A, 8, 40, 64, A, f, A, A, A, need, None) == 2
    assert L.wush_workspace_status(None, 64, None) == 1
    assert L.wush_workspace_status(A, 50, None) == 2


def test_linear_and_tap_validation(L):
    f = P.default_fmt()
    g = P.default_fmt(out_dtype=1)
    lin = lambda *a: L.wush_linear(*a)
    assert lin(A, A, A, A, 4, 8, 64, f, None, 8, None) == 1
    assert lin(A, A, A, A, 4, 8, 96 + 16, f, A, 8, None) == 2       # K % 32
    assert lin(A, A, A, A, 4, 9, 64, f, A, 8, None) == 2            # ldy < N
    assert lin(A, A, A, A, 4, 9, 64, f, A + 1, 12, None) == 3       # bf16 Y at an odd address
    assert lin(A, A, A, A, 4, 9, 64, g, A + 2, 12, None) == 3       # f32 Y not 4-byte aligned
    assert lin(A, A, A, A, -1, 9, 64, f, A, 16, None) == 2
    assert lin(A, A + 1, A, A, 4, 8, 64, f, A, 8, None) == 3
    tap = lambda *a: L.wush_quantize_f32(*a)
    assert tap(None, 4, 64, f, A, A, None) == 1
    assert tap(A, 4, 65, f, A, A, None) == 2
    assert tap(A + 4, 4, 64, f, A, A, None) == 3


def test_binding_raises_typed_error(L):
    class Fake:
        def __init__(self, shape, stride0, ptr=A):
            self.shape, self._s, self._p = shape, stride0, ptr

        def stride(self, i):
            return self._s

        def data_ptr(self):
            return self._p

    with pytest.raises(P.WushError) as ei:
        P.wush_quantize_act(Fake((4, 48), 48), Fake((1, 32, 32), 1024), Fake((4, 24), 24), Fake((4, 1), 1), stream=0)
    assert ei.value.code == 2 and "WUSH_ERR_SHAPE" in str(ei.value)


def test_packed_sizes_and_unpack_validation(L):
    assert P.wush_packed_sizes(100, 512) == (100 * 256, 100 * 16)
    assert P.wush_packed_sizes(100, 512, P.default_fmt(layout=1)) == (256 * 256, 256 * 16)
    assert P.wush_packed_sizes(257, 256, P.default_fmt(layout=1)) == (512 * 128, 512 * 8)
    with pytest.raises(P.WushError):
        P.wush_packed_sizes(100, 128, P.default_fmt(layout=1))
    assert L.wush_unpack_tiled(A, A, 4, 128, A, A, None) == 2
    assert L.wush_unpack_tiled(None, A, 4, 256, A, A, None) == 1
    assert L.wush_unpack_tiled(A, A, 4, 256, A + 3, A, None) == 3


def test_build_transforms_validation(L):
    need = L.wush_build_transforms_workspace(64)
    assert need >= 2 * 2 * 1024 * 8 + 4 and L.wush_build_transforms_workspace(48) == 0
    bt = lambda *a: L.wush_build_transforms(*a)
    assert bt(None, 8, 64, A, 16, 64, 64, 0.01, A, None, A, need, None) == 1
    assert bt(A, 8, 64, A, 16, 64, 48, 0.01, A, None, A, need, None) == 2     # K % 32
    assert bt(A, 8, 64, A, 0, 64, 64, 0.01, A, None, A, need, None) == 2      # no calibration tokens
    assert bt(A, 8, 64, A, 16, 64, 64, -1.0, A, None, A, need, None) == 2     # negative damping
    assert bt(A, 8, 64, A, 16, 64, 64, 0.01, A, A + 8, A, need, None) == 3    # misaligned f64 tap
    assert bt(A, 8, 64, A, 16, 64, 64, 0.01, A, None, A, need - 1, None) == 5
    assert bt(A, 8, 64, A, 16, 64, 64, 0.01, A, None, None, need, None) == 5
    assert L.wush_build_transforms_status(None, 64, None) == 1


def test_layer_decode_validation(L):
    t = P.default_fmt(layout=1)
    need = L.wush_layer_decode_workspace(512)
    assert need >= 2 * (2 * 4096 + 2 * 256) + 64
    assert L.wush_layer_decode_workspace(288) == 0                # K % 256
    B = 0x10000                                                   # 256-byte aligned fake address
    dec = lambda *a: L.wush_layer_decode(*a)
    assert dec(None, 4, 512, 512, A, A, A, 64, t, A, 64, B, need, None) == 1
    assert dec(A, 4, 512, 512, A, A, A, 64, P.default_fmt(), A, 64, B, need, None) == 4   # canonical weights
    assert dec(A, 65, 512, 512, A, A, A, 64, t, A, 64, B, need, None) == 2                # M > 64
    assert dec(A, 4, 480, 480, A, A, A, 64, t, A, 64, B, need, None) == 2                 # K % 256
    assert dec(A, 4, 512, 512, A, A, A, 64, t, A, 60, B, need, None) == 2                 # ldy < N
    assert dec(A, 4, 512, 512, A, A + 8, A, 64, t, A, 64, B, need, None) == 3
    assert dec(A, 4, 512, 512, A, A, A, 64, t, A, 64, B, need - 1, None) == 5
    assert dec(A, 4, 512, 512, A, A, A, 64, t, A, 64, B + 16, need, None) == 3            # workspace alignment
    assert L.wush_layer_decode_init(None, need, 512, None) == 1
    assert L.wush_layer_decode_init(B, need - 1, 512, None) == 5
    assert L.wush_layer_decode_status(None, 512, None) == 1


def test_debug_set_validation(L):
    assert L.wush_debug_set(0, 2) == 0 and L.wush_debug_set(0, -1) == 0
    assert L.wush_debug_set(7, 1) == 4 and L.wush_debug_set(-1, 1) == 4       # unknown option
    assert L.wush_debug_set(0, -2) == 2 and L.wush_debug_set(0, 5000) == 2    # value out of range


def test_nvfp4_validation(L):
    q = lambda *a: L.wush_quantize_act_nvfp4(*a)
    assert q(None, 4, 64, 64, A, A, 0, A, A, None, None) == 1          # null X
    assert q(A, 4, 64, 64, A, None, 0, A, A, None, None) == 1          # null tensor scale
    assert q(A, 4, 48, 48, A, A, 0, A, A, None, None) == 2             # K % 32
    assert q(A, 4, 96, 96, A, A, 1, A, A, None, None) == 2             # tiled layout needs K % 64 == 0
    assert q(A, 4, 64, 64, A, A, 3, A, A, None, None) == 4             # unknown layout
    assert q(A, 4, 64, 64, A, A + 2, 0, A, A, None, None) == 3         # tensor scale not 4-byte aligned
    assert q(A, 4, 64, 64, A + 8, A, 0, A, A, None, None) == 3
    need = L.wush_prepare_weight_nvfp4_workspace(64)
    assert need >= 4 * 256 * 8 + 12 and L.wush_prepare_weight_nvfp4_workspace(40) == 0
    w = lambda *a: L.wush_prepare_weight_nvfp4(*a)
    assert w(A, 8, 64, 64, A, 0, A, A, None, A, need, None) == 1       # null tensor scale (output)
    assert w(A, 8, 64, 64, A, 0, A, A, A, None, need, None) == 5
    assert w(A, 8, 64, 64, A, 0, A, A, A, A, need - 1, None) == 5
    assert w(A, 8, 64, 64, A, 2, A, A, A, A, need, None) == 4
    assert L.wush_prepare_weight_nvfp4_status(None, 64, None) == 1
    lin = lambda *a: L.wush_linear_nvfp4(*a)
    assert lin(A, A, None, A, A, A, 4, 8, 64, 0, 0, A, 8, None) == 1
    assert lin(A, A, A, A, A, A, 4, 8, 96, 0, 0, A, 8, None) == 2      # K % 64
    assert lin(A, A, A, A, A, A, 4, 9, 64, 0, 0, A, 8, None) == 2      # ldy < N
    assert lin(A, A, A, A, A, A, 4, 8, 64, 0, 2, A, 8, None) == 4      # output type
    assert lin(A, A, A, A, A, A, 4, 8, 64, 5, 0, A, 8, None) == 4      # layout
    assert lin(A, A, A, A, A, A, 4, 8, 64, 0, 1, A + 2, 8, None) == 3  # f32 Y not 4-byte aligned
    assert L.wush_calibrate_act_nvfp4(A, 4, 64, 64, A, None, None) == 1
    assert L.wush_calibrate_act_nvfp4(A, 4, 64, 60, A, A, None) == 2
    need_bt = L.wush_build_transforms_workspace(64)
    assert L.wush_build_transforms_nvfp4(A, 8, 64, A, 16, 64, 64, 0.01, A, None, A, need_bt - 1, None) == 5
    assert L.wush_build_transforms_nvfp4(A, 8, 64, None, 16, 64, 64, 0.01, A, None, A, need_bt, None) == 1
    assert P.wush_packed_sizes_nvfp4(100, 512) == (100 * 256, 100 * 32)
    assert P.wush_packed_sizes_nvfp4(100, 512, 1) == (128 * 256, 128 * 32)
    with pytest.raises(P.WushError):
        P.wush_packed_sizes_nvfp4(100, 96, 1)
    assert L.wush_unpack_tiled_nvfp4(A, A, 4, 96, A, A, None) == 2


def test_int4_validation(L):
    q = lambda *a: L.wush_quantize_act_int4(*a)
    assert q(None, 4, 64, 64, A, 0, A, A, None, None) == 1
    assert q(A, 4, 48, 48, A, 0, A, A, None, None) == 2
    assert q(A, 4, 96, 96, A, 1, A, A, None, None) == 2                # tiled layout needs K % 64 == 0
    assert q(A, 4, 64, 64, A, 9, A, A, None, None) == 4
    assert q(A, 4, 64, 64, A, 0, A + 4, A, None, None) == 3
    need = L.wush_prepare_weight_workspace(8, 64)
    w = lambda *a: L.wush_prepare_weight_int4(*a)
    assert w(A, 8, 64, 64, A, 0, A, A, A, need - 1, None) == 5
    assert w(A, 8, 64, 64, None, 0, A, A, A, need, None) == 1
    lin = lambda *a: L.wush_linear_int4(*a)
    assert lin(A, A, A, None, 4, 8, 64, 0, 0, A, 8, None) == 1
    assert lin(A, A, A, A, 4, 8, 32, 0, 0, A, 8, None) == 2            # K % 64
    assert lin(A, A, A, A, 4, 8, 64, 0, 0, A + 1, 8, None) == 3
    tap = lambda *a: L.wush_quantize_f32_int4(*a)
    assert tap(A, 4, 64, 0, None, A, None) == 1 and tap(A, 4, 65, 0, A, A, None) == 2


def test_size_limits(L):
    """Row counts up to 2^30, K up to 2^22, M * N of a GEMM up to 2^40: anything larger is a shape error
    before any launch (kernel index arithmetic is sized for these)."""
    f = P.default_fmt()
    big_rows, big_k = (1 << 30) + 1, (1 << 22) + 32
    assert L.wush_quantize_act(A, big_rows, 64, 64, A, f, A, A, None, None) == 2
    assert L.wush_quantize_act(A, 4, big_k, big_k, A, f, A, A, None, None) == 2
    assert L.wush_linear(A, A, A, A, 1 << 21, 1 << 20, 64, f, A, 1 << 20, None) == 2        # M * N = 2^41
    assert L.wush_linear(A, A, A, A, 4, 8, big_k, f, A, 8, None) == 2
    assert L.wush_linear_nvfp4(A, A, A, A, A, A, 1 << 21, 1 << 20, 64, 0, 0, A, 1 << 20, None) == 2
    assert L.wush_linear_int4(A, A, A, A, 1 << 21, 1 << 20, 64, 0, 0, A, 1 << 20, None) == 2
    assert L.wush_linear_int4(A, A, A, A, 4, 8, big_k + 32, 0, 0, A, 8, None) == 2
    assert L.wush_build_transforms_workspace(big_k) == 0
    assert L.wush_prepare_weight_gptq_workspace(big_rows, 64) == 0
