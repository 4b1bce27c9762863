"""wush_layer_decode_static (the entry point that allocates nothing: its scratch is a fixed device
array inside the library) against wush_layer_decode on the same inputs: two calls in a row through
the C ABI, the second with a smaller input, each bit-identical to the workspace-taking call, and the
first also within the layer tolerance of the CPU oracle.  Runs last: the array keeps what the calls
before it left there, which no result may depend on.
"""
import ctypes

import numpy as np
import pytest

import wush_inputs as I
from oracle import wush_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2512_00956_amd as P
    P.lib()
    return P


@pytest.fixture(scope="module")
def G():
    from tests import gpu_util
    return gpu_util


def _layer(P, G, K, N, seed):
    import torch
    cfg = I.scaled(I.CONFIGS["c2"], M=64, K=K, N=N, calib_tokens=8, n_outlier=max(1, K // 256))
    L = I.make_layer(cfg)
    Tb = I.make_transforms_random(K // 32, seed)
    Td, Wd = G.bf16_dev(Tb), G.bf16_dev(L["W"])
    tiled = P.default_fmt(layout=1)
    cb, sb = P.wush_packed_sizes(N, K, tiled)
    Wq, Ws = G.empty_u8(cb), G.empty_u8(sb)
    wsp = G.empty_u8(P.wush_prepare_weight_workspace(N, K))
    P.wush_prepare_weight(Wd, Td, Wq, Ws, wsp, tiled)
    P.wush_workspace_status(wsp, K)
    torch.cuda.synchronize()
    return L, Tb, Td, Wq, Ws


def _ref_call(P, G, Xd, Td, Wq, Ws, N, K, out_dtype):
    import torch
    fmt = P.default_fmt(layout=1, out_dtype=out_dtype)
    Y = torch.full((Xd.shape[0], N), float("nan"), dtype=torch.float32 if out_dtype else torch.bfloat16, device="cuda")
    dws = G.empty_u8(P.wush_layer_decode_workspace(K))
    P.wush_layer_decode_init(dws, K)
    P.wush_layer_decode(Xd, Td, Wq, Ws, Y, dws, fmt)
    P.wush_layer_decode_status(dws, K)
    return G.host(Y)


def _static_call_c_abi(P, Xd, Td, Wq, Ws, Y, fmt):
    """Straight through the C symbol: plain pointers and sizes."""
    import torch
    M, K = Xd.shape
    N = Y.shape[1]
    vp = ctypes.c_void_p
    rc = P.lib().wush_layer_decode_static(vp(Xd.data_ptr()), M, K, Xd.stride(0), vp(Td.data_ptr()), vp(Wq.data_ptr()),
                                          vp(Ws.data_ptr()), N, fmt, vp(Y.data_ptr()), Y.stride(0),
                                          vp(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, P.wush_status_string(rc)


@pytest.mark.parametrize("out_dtype", [0, 1])
def test_static_scratch_call_equals_workspace_call_twice(P, G, out_dtype):
    import torch
    K1, N1, M1 = 2048, 1000, 61       # two row blocks, ragged N
    K2, N2, M2 = 512, 96, 7           # smaller on every axis: most of the first call's scratch stays behind
    fmt = P.default_fmt(layout=1, out_dtype=out_dtype)
    dt = torch.float32 if out_dtype else torch.bfloat16
    L1, Tb1, Td1, Wq1, Ws1 = _layer(P, G, K1, N1, 21)
    L2, Tb2, Td2, Wq2, Ws2 = _layer(P, G, K2, N2, 22)
    X1, X2 = G.bf16_dev(L1["X"][:M1]), G.bf16_dev(L2["X"][:M2])
    r1 = _ref_call(P, G, X1, Td1, Wq1, Ws1, N1, K1, out_dtype)
    r2 = _ref_call(P, G, X2, Td2, Wq2, Ws2, N2, K2, out_dtype)
    Y1 = torch.full((M1, N1), float("nan"), dtype=dt, device="cuda")
    Y2 = torch.full((M2, N2), float("nan"), dtype=dt, device="cuda")
    _static_call_c_abi(P, X1, Td1, Wq1, Ws1, Y1, fmt)
    _static_call_c_abi(P, X2, Td2, Wq2, Ws2, Y2, fmt)
    torch.cuda.synchronize()
    y1, y2 = G.host(Y1), G.host(Y2)
    assert np.array_equal(y1.view(np.uint8), r1.view(np.uint8))
    assert np.array_equal(y2.view(np.uint8), r2.view(np.uint8))
    # The same pair once more, now that the runtime has loaded everything it loads lazily (code object,
    # symbol table): the device's free memory must not move, and what the first pair left in the scratch
    # must not matter.
    Y1.fill_(float("nan"))
    Y2.fill_(float("nan"))
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    _static_call_c_abi(P, X1, Td1, Wq1, Ws1, Y1, fmt)
    _static_call_c_abi(P, X2, Td2, Wq2, Ws2, Y2, fmt)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before
    assert np.array_equal(G.host(Y1).view(np.uint8), r1.view(np.uint8))
    assert np.array_equal(G.host(Y2).view(np.uint8), r2.view(np.uint8))
    # and the oracle, end to end (BF16 output: 2e-3; FP32: the quantized path's own accuracy is the same
    # on both sides, only the accumulation order differs)
    for y, L, Tb, M in ((y1, L1, Tb1, M1), (y2, L2, Tb2, M2)):
        X, W, T = (O.bf16_bits_to_f64(a) for a in (L["X"][:M], L["W"], Tb))
        ref = O.layer_forward(X, W, T)
        yv = O.bf16_bits_to_f64(y) if not out_dtype else y.astype(np.float64)
        assert O.rel_fro(yv, ref) <= 2e-3


def test_static_scratch_limits_and_validation(P, G):
    import torch
    L = P.lib()
    vp = ctypes.c_void_p
    A = vp(256)
    fmt = P.default_fmt(layout=1)
    call = L.wush_layer_decode_static
    assert call(A, 4, 32768 + 256, 32768 + 256, A, A, A, 64, fmt, A, 64, None) == 9      # beyond the fixed scratch
    assert P.wush_status_string(9) == "size beyond the fixed scratch of this entry point"
    assert call(None, 4, 512, 512, A, A, A, 64, fmt, A, 64, None) == 1
    assert call(A, 65, 512, 512, A, A, A, 64, fmt, A, 64, None) == 2
    assert call(A, 4, 480, 480, A, A, A, 64, fmt, A, 64, None) == 2
    assert call(A, 4, 512, 512, A, A, A, 64, P.default_fmt(layout=0), A, 64, None) == 4
    assert call(A, 4, 512, 512, A, vp(264), A, 64, fmt, A, 64, None) == 3
