"""GPU parity of the decode-sized paths (at most 64 tokens): the weight-streaming
GEMM that wush_linear takes for M <= 64 in the tiled layout, and the one-launch
layer forward wush_layer_decode (transform + quantize + GEMM behind a grid-wide
barrier).  The oracle is the same FP64 layer forward as everywhere else; the
fused call must in addition reproduce the two-call path bit for bit.
"""
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


def _poisoned(P, rows, K):
    import torch
    cb, sb = P.wush_packed_sizes(rows, K, P.default_fmt(layout=1))
    return (torch.full((cb,), 0xEE, dtype=torch.uint8, device="cuda"),
            torch.full((sb,), 0xEE, dtype=torch.uint8, device="cuda"))


def _prepared_layer(P, G, M, K, N, seed_shift=0):
    """Synthetic layer + random well-conditioned transforms, weights prepared in the tiled layout."""
    import torch
    cfg = I.scaled(I.CONFIGS["c2"], M=M, K=K, N=N, calib_tokens=8, n_outlier=max(1, K // 256))
    L = I.make_layer(cfg)
    Tb = I.make_transforms_random(K // 32, 11 + seed_shift)
    Td, Xd, Wd = G.bf16_dev(Tb), G.bf16_dev(L["X"]), G.bf16_dev(L["W"])
    tiled = P.default_fmt(layout=1)
    Wq, Ws = _poisoned(P, N, K)
    wsp = G.empty_u8(P.wush_prepare_weight_workspace(N, K))
    P.wush_prepare_weight(Wd, Td, Wq, Ws, wsp, tiled)
    P.wush_workspace_status(wsp, K)
    Wqc, Wsc = G.empty_u8(N, K // 2), G.empty_u8(N, K // 32)
    P.wush_unpack_tiled(Wq, Ws, N, K, Wqc, Wsc)
    torch.cuda.synchronize()
    return dict(L=L, Tb=Tb, Td=Td, Xd=Xd, Wq=Wq, Ws=Ws, wq=G.host(Wqc), ws=G.host(Wsc))


def _two_call(P, G, S, M, K, N, out_dtype):
    import torch
    Xq, Xs = _poisoned(P, M, K)
    P.wush_quantize_act(S["Xd"][:M], S["Td"], Xq, Xs, P.default_fmt(layout=1))
    Y = torch.full((M, N), float("nan"), dtype=torch.float32 if out_dtype else torch.bfloat16, device="cuda")
    P.wush_linear(Xq, Xs, S["Wq"], S["Ws"], Y, P.default_fmt(out_dtype=out_dtype, layout=1), K=K)
    xq, xs = G.empty_u8(M, K // 2), G.empty_u8(M, K // 32)
    P.wush_unpack_tiled(Xq, Xs, M, K, xq, xs)
    torch.cuda.synchronize()
    return Y, G.host(xq), G.host(xs)


SHAPES = [(64, 256, 32), (33, 1024, 96), (64, 1280, 45), (32, 2048, 520), (17, 4096, 6144), (64, 4096, 6144)]


@pytest.mark.parametrize("M,K,N", SHAPES)
def test_skinny_gemm_against_oracle(P, G, M, K, N):
    """wush_linear, tiled layout, M <= 64: FP32 and BF16 outputs against the
    oracle's FP64 product of the very codes the GPU holds."""
    S = _prepared_layer(P, G, M, K, N)
    Yf, xq, xs = _two_call(P, G, S, M, K, N, 1)
    Yb, _, _ = _two_call(P, G, S, M, K, N, 0)
    ref = O.dequantize(O.unpack_codes(xq), xs) @ O.dequantize(O.unpack_codes(S["wq"]), S["ws"]).T
    yf = G.host(Yf).astype(np.float64)
    assert np.isfinite(yf).all()
    assert O.rel_fro(yf, ref) <= 1e-5
    assert np.array_equal(O.bf16_bits_to_f64(G.host(Yb)), O.round_to_bf16(yf))
    assert O.rel_fro(O.bf16_bits_to_f64(G.host(Yb)), ref) <= 2e-3


@pytest.mark.parametrize("M,K,N", [(65, 512, 96), (100, 1280, 200), (128, 4096, 6144)])
def test_skinny_gemm_up_to_128_tokens(P, G, M, K, N):
    """65..128 tokens still take the weight-streaming kernel (four token blocks per workgroup)."""
    S = _prepared_layer(P, G, M, K, N)
    Yf, xq, xs = _two_call(P, G, S, M, K, N, 1)
    Yb, _, _ = _two_call(P, G, S, M, K, N, 0)
    ref = O.dequantize(O.unpack_codes(xq), xs) @ O.dequantize(O.unpack_codes(S["wq"]), S["ws"]).T
    yf = G.host(Yf).astype(np.float64)
    assert np.isfinite(yf).all()
    assert O.rel_fro(yf, ref) <= 1e-5
    assert np.array_equal(O.bf16_bits_to_f64(G.host(Yb)), O.round_to_bf16(yf))


def test_skinny_gemm_every_m(P, G):
    """Every M from 1 to 64 gives the rows of the M = 64 result (each token is independent)."""
    import torch
    K, N = 1024, 160
    S = _prepared_layer(P, G, 64, K, N)
    Y64, _, _ = _two_call(P, G, S, 64, K, N, 1)
    for M in list(range(1, 9)) + [15, 16, 31, 32, 33, 48, 63]:
        Y, _, _ = _two_call(P, G, S, M, K, N, 1)
        assert torch.equal(Y, Y64[:M]), M


@pytest.fixture(params=[1, 0], ids=["one_launch", "two_launches"])
def forced_form(request, P):
    """wush_layer_decode runs as one launch or as two (WUSH_DEBUG_DECODE_FUSED); both forms are
    checked on every shape."""
    P.wush_debug_set(P.WUSH_DEBUG_DECODE_FUSED, request.param)
    yield request.param
    P.wush_debug_set(P.WUSH_DEBUG_DECODE_FUSED, -1)


@pytest.mark.parametrize("M,K,N", SHAPES)
@pytest.mark.parametrize("out_dtype", [0, 1])
def test_layer_decode_equals_two_calls_and_oracle(P, G, M, K, N, out_dtype, forced_form):
    import torch
    S = _prepared_layer(P, G, M, K, N)
    Y2, xq, xs = _two_call(P, G, S, M, K, N, out_dtype)
    wsp = torch.full((P.wush_layer_decode_workspace(K),), 0xEE, dtype=torch.uint8, device="cuda")
    P.wush_layer_decode_init(wsp, K)
    fmt = P.default_fmt(out_dtype=out_dtype, layout=1)
    for rep in range(3):   # the barrier re-arms itself: several launches on one workspace
        Y = torch.full((M, N), float("nan"), dtype=Y2.dtype, device="cuda")
        P.wush_layer_decode(S["Xd"][:M], S["Td"], S["Wq"], S["Ws"], Y, wsp, fmt)
        P.wush_layer_decode_status(wsp, K)
        assert torch.equal(Y, Y2), rep
    # the activations the fused kernel quantized (first part of its workspace, tiled, 64 rows)
    KT = K // 256
    q, s = G.empty_u8(M, K // 2), G.empty_u8(M, K // 32)
    P.wush_unpack_tiled(wsp[:KT * 8192], wsp[KT * 8192:KT * 8192 + KT * 512], M, K, q, s)
    torch.cuda.synchronize()
    assert np.array_equal(G.host(q), xq) and np.array_equal(G.host(s), xs)
    # against the oracle's full FP64 layer forward (same bar as the large configurations:
    # exact on own codes, and within the boundary-flip allowance of the complete path)
    X = O.bf16_bits_to_f64(S["L"]["X"][:M])
    T = O.bf16_bits_to_f64(S["Tb"]).reshape(K // 32, 32, 32)
    Yt = O.transform_act(X, T)
    cr, sr = O.quantize_mxfp4(Yt)
    rate, unexplained = G.code_mismatch_report(Yt, O.unpack_codes(xq), xs, cr, sr)
    assert rate <= 1e-4 and unexplained == 0
    wdq = O.dequantize(O.unpack_codes(S["wq"]), S["ws"])
    y = G.host(Y).astype(np.float64) if out_dtype else O.bf16_bits_to_f64(G.host(Y))
    own = O.dequantize(O.unpack_codes(xq), xs) @ wdq.T
    assert O.rel_fro(y, own) <= (1e-5 if out_dtype else 2e-3)
    ref = O.dequantize(cr, sr) @ wdq.T
    exact = X @ O.bf16_bits_to_f64(S["L"]["W"]).T
    assert O.rel_fro(y, ref) <= max(2e-3, 0.05 * O.rel_fro(ref, exact))


def test_layer_decode_strided_and_alternating_inputs(P, G, forced_form):
    """Row strides on X and Y, and two different activations alternating on one workspace."""
    import torch
    M, K, N = 40, 1024, 200
    S = _prepared_layer(P, G, 64, K, N)
    wsp = G.empty_u8(P.wush_layer_decode_workspace(K))
    P.wush_layer_decode_init(wsp, K)
    Xwide = torch.zeros((64, K + 64), dtype=torch.bfloat16, device="cuda")
    Xwide[:, :K] = S["Xd"]
    Ywide = torch.full((M, N + 24), float("nan"), dtype=torch.bfloat16, device="cuda")
    for start in (0, 20, 0, 20):
        Xa = Xwide[start:start + M, :K]
        Y2 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        Xq, Xs = _poisoned(P, M, K)
        P.wush_quantize_act(Xa, S["Td"], Xq, Xs, P.default_fmt(layout=1))
        P.wush_linear(Xq, Xs, S["Wq"], S["Ws"], Y2, P.default_fmt(layout=1), K=K)
        P.wush_layer_decode(Xa, S["Td"], S["Wq"], S["Ws"], Ywide[:, :N], wsp)
        P.wush_layer_decode_status(wsp, K)
        assert torch.equal(Ywide[:, :N], Y2), start
    assert bool(Ywide[:, N:].isnan().all())     # nothing written past N


def test_layer_decode_barrier_timeout_is_reported(P, G):
    """The test hook makes the barrier expect one workgroup more than exist and give up after a
    few polls: every workgroup exits, the status call reports it, and after re-arming the
    workspace the next call is correct."""
    import torch
    M, K, N = 8, 512, 64
    S = _prepared_layer(P, G, M, K, N)
    Y2, _, _ = _two_call(P, G, S, M, K, N, 0)
    wsp = G.empty_u8(P.wush_layer_decode_workspace(K))
    P.wush_layer_decode_init(wsp, K)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    P.wush_debug_set(P.WUSH_DEBUG_DECODE_TEST_TIMEOUT, 1)
    try:
        P.wush_layer_decode(S["Xd"][:M], S["Td"], S["Wq"], S["Ws"], Y, wsp)
    finally:
        P.wush_debug_set(P.WUSH_DEBUG_DECODE_TEST_TIMEOUT, -1)
    with pytest.raises(P.WushError) as ei:
        P.wush_layer_decode_status(wsp, K)
    assert ei.value.code == 8
    assert bool(Y.isnan().all())                # Y untouched
    P.wush_layer_decode_init(wsp, K)
    P.wush_layer_decode(S["Xd"][:M], S["Td"], S["Wq"], S["Ws"], Y, wsp)
    P.wush_layer_decode_status(wsp, K)
    assert torch.equal(Y, Y2)


def test_layer_decode_default_form(P, G):
    """Without the override (two launches) the call gives the same result."""
    import torch
    M, K, N = 5, 4096, 1024
    S = _prepared_layer(P, G, M, K, N)
    Y2, _, _ = _two_call(P, G, S, M, K, N, 0)
    wsp = G.empty_u8(P.wush_layer_decode_workspace(K))
    P.wush_layer_decode_init(wsp, K)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    P.wush_layer_decode(S["Xd"][:M], S["Td"], S["Wq"], S["Ws"], Y, wsp)
    P.wush_layer_decode_status(wsp, K)
    assert torch.equal(Y, Y2)
