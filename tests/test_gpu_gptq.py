"""GPU parity of wush_prepare_weight_gptq (Alg. 2, GPTQ case) against the FP64 oracle.

The schedule is sequential with feedback: a transform entry that lands on the other side of a
BF16 rounding boundary, or a weight code that flips at an exact tie, changes everything after
it a little.  Both sides are FP64 with different summation orders (1e-16 relative), so such an
event needs a value within 1e-15 of a boundary: on the layers below none occurs and the outputs
are identical (also on the full c2 layer, 25 million codes).  The bars are set at that level:
at most 1e-4 of the transform entries (each one BF16 step apart), of the scales and of the codes
may differ -- on these sizes that is a handful of elements at most, where a wrong index in the
propagation of a single block shifts every later block (a tenth of all codes or more) -- and the
output error GPTQ minimizes must equal the oracle's to 1e-6 when nothing differs, 1e-3 otherwise.
"""
import numpy as np
import pytest

import wush_inputs as I
from oracle import wush_gptq_oracle as Q
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


def _layer(M, K, N, Mc, seed_mix=7, n_outlier=3):
    cfg = I.scaled(I.CONFIGS["c2"], M=M, K=K, N=N, calib_tokens=Mc, n_outlier=n_outlier)
    L = I.make_layer(cfg)
    # correlate the channels (the generator draws them independently; GPTQ's propagation acts on correlations);
    # the mixed calibration set is rounded to BF16 again because that is what both sides read
    rng = np.random.default_rng(seed_mix)
    mix = np.eye(K) + 0.3 * rng.standard_normal((K, K)) / np.sqrt(K)
    Xc = O.round_to_bf16(O.bf16_bits_to_f64(L["X_cal"]) @ mix)
    X = O.round_to_bf16(O.bf16_bits_to_f64(L["X"]) @ mix)
    return O.bf16_bits_to_f64(L["W"]), Xc, X


def _run_gpu(P, G, W, Xc, lam, layout=0, T_given=None):
    import torch
    N, K = W.shape
    fmt = P.default_fmt(layout=layout)
    Wd, Xd = G.bf16_dev(O.bf16_values_to_bits(W)), G.bf16_dev(O.bf16_values_to_bits(Xc))
    if T_given is None:
        Td = torch.full((K // 32, 32, 32), float("nan"), dtype=torch.bfloat16, device="cuda")
    else:
        Td = G.bf16_dev(O.bf16_values_to_bits(T_given))
    cb, sb = P.wush_packed_sizes(N, K, fmt)
    Wq = torch.full((cb,), 0xEE, dtype=torch.uint8, device="cuda")
    Ws = torch.full((sb,), 0xEE, dtype=torch.uint8, device="cuda")
    wsp = torch.empty(P.wush_prepare_weight_gptq_workspace(N, K), dtype=torch.uint8, device="cuda")
    P.wush_prepare_weight_gptq(Wd, Xd, lam, Td, Wq, Ws, wsp, fmt, transform_given=T_given is not None)
    P.wush_prepare_weight_gptq_status(wsp, N, K)
    if layout:
        q, s = G.empty_u8(N, K // 2), G.empty_u8(N, K // 32)
        P.wush_unpack_tiled(Wq, Ws, N, K, q, s)
    else:
        q, s = Wq.view(N, K // 2), Ws.view(N, K // 32)
    torch.cuda.synchronize()
    return O.bf16_bits_to_f64(G.host(Td)), O.unpack_codes(G.host(q)), G.host(s)


def _compare(T_gpu, c_gpu, s_gpu, T_ref, c_ref, s_ref, W, X, what):
    dT = T_gpu != T_ref
    step = np.abs(T_gpu - T_ref) / np.maximum(np.abs(T_ref), 1e-30)
    print(f"{what}: T entries differing {dT.mean():.2e} (max relative step {step.max():.2e}), "
          f"scales differing {np.mean(s_gpu != s_ref):.2e}, codes differing {np.mean(c_gpu != c_ref):.2e}")
    n_diff = int(dT.sum()) + int(np.sum(s_gpu != s_ref)) + int(np.sum(c_gpu != c_ref))
    assert dT.mean() <= 1e-4 and step.max() <= 2.0 ** -7          # at most one BF16 step
    assert np.mean(s_gpu != s_ref) <= 1e-4
    assert np.mean(c_gpu != c_ref) <= 1e-4
    l_gpu, l_ref = Q.proxy_loss(T_gpu, c_gpu, s_gpu, W, X), Q.proxy_loss(T_ref, c_ref, s_ref, W, X)
    print(f"{what}: weight-only output MSE  oracle {l_ref:.5e}  GPU {l_gpu:.5e}  ({n_diff} differing values)")
    assert abs(l_gpu - l_ref) <= (1e-6 if n_diff == 0 else 1e-3) * l_ref
    return l_gpu


@pytest.mark.parametrize("N,K,Mc,layout", [(48, 128, 400, 0), (300, 512, 1024, 1), (77, 416, 1000, 0)])
def test_gptq_wush_against_oracle(P, G, N, K, Mc, layout):
    W, Xc, X = _layer(64, K, N, Mc)
    T_ref, c_ref, s_ref = Q.gptq_wush_layer(W, Xc, 1e-2)
    T_gpu, c_gpu, s_gpu = _run_gpu(P, G, W, Xc, 1e-2, layout)
    l_gptq = _compare(T_gpu, c_gpu, s_gpu, T_ref, c_ref, s_ref, W, X, f"N={N} K={K}")
    # and it does what it is for: lower output error than the RTN case on the same layer
    T0 = O.round_to_bf16(O.build_transforms(W, Xc, 1e-2))
    c0, s0 = O.quantize_mxfp4(O.transform_weight(W, T0))
    assert l_gptq < Q.proxy_loss(T0, c0, s0, W, X)


@pytest.mark.parametrize("transform", ["hadamard", "identity"])
def test_gptq_with_a_given_transform(P, G, transform):
    N, K, Mc = 96, 256, 800
    W, Xc, X = _layer(64, K, N, Mc)
    T_ref, c_ref, s_ref = Q.gptq_wush_layer(W, Xc, 1e-2, transform=transform)
    T_gpu, c_gpu, s_gpu = _run_gpu(P, G, W, Xc, 1e-2, 0, T_given=T_ref)
    assert np.array_equal(T_gpu, T_ref)                            # an input: untouched
    _compare(T_gpu, c_gpu, s_gpu, T_ref, c_ref, s_ref, W, X, transform)


def test_gptq_reports_a_hessian_that_is_not_positive_definite(P, G):
    import torch
    N, K = 32, 64
    W, _, _ = _layer(8, K, N, 64)
    Xc = np.zeros((64, K))
    Wd, Xd = G.bf16_dev(O.bf16_values_to_bits(W)), G.bf16_dev(O.bf16_values_to_bits(Xc))
    Td = torch.zeros((K // 32, 32, 32), dtype=torch.bfloat16, device="cuda")
    Wq, Ws = G.empty_u8(N, K // 2), G.empty_u8(N, K // 32)
    wsp = torch.empty(P.wush_prepare_weight_gptq_workspace(N, K), dtype=torch.uint8, device="cuda")
    P.wush_prepare_weight_gptq(Wd, Xd, 0.0, Td, Wq, Ws, wsp)
    with pytest.raises(P.WushError) as ei:
        P.wush_prepare_weight_gptq_status(wsp, N, K)
    assert ei.value.code == 7


def test_gptq_layer_runs_through_the_online_path(P, G):
    """The outputs plug into the unchanged online path: quantize activations with the returned T,
    multiply with the returned codes; the W4A4 layer loss beats RTN + Hadamard (direction of the paper's tables)."""
    import torch
    M, K, N, Mc = 64, 512, 256, 2048
    W, Xc, X = _layer(M, K, N, Mc)
    fmt = P.default_fmt(layout=1)
    T_gpu, c_gpu, s_gpu = _run_gpu(P, G, W, Xc, 1e-2, 1)
    Td = G.bf16_dev(O.bf16_values_to_bits(T_gpu))
    Wd, Xcd = G.bf16_dev(O.bf16_values_to_bits(W)), G.bf16_dev(O.bf16_values_to_bits(Xc))
    cb, sb = P.wush_packed_sizes(N, K, fmt)
    Wq, Ws = G.empty_u8(cb), G.empty_u8(sb)
    wsp = torch.empty(P.wush_prepare_weight_gptq_workspace(N, K), dtype=torch.uint8, device="cuda")
    Td2 = torch.empty_like(Td)
    P.wush_prepare_weight_gptq(Wd, Xcd, 1e-2, Td2, Wq, Ws, wsp, fmt)
    assert torch.equal(Td2, Td)                                    # reproducible
    xcb, xsb = P.wush_packed_sizes(M, K, fmt)
    Xq, Xs = G.empty_u8(xcb), G.empty_u8(xsb)
    Xd = G.bf16_dev(O.bf16_values_to_bits(X))
    P.wush_quantize_act(Xd, Td, Xq, Xs, fmt)
    Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    P.wush_linear(Xq, Xs, Wq, Ws, Y, P.default_fmt(out_dtype=1, layout=1), K=K)
    torch.cuda.synchronize()
    y = G.host(Y).astype(np.float64)
    xc, xs = O.quantize_mxfp4(O.transform_act(X, T_gpu))
    ref = O.dequantize(xc, xs) @ O.dequantize(c_gpu, s_gpu).T
    assert O.rel_fro(y, ref) <= 2e-3
    exact = X @ W.T
    l_gw = O.layer_loss(y, exact)
    l_rh = O.layer_loss(O.layer_forward(X, W, O.round_to_bf16(O.hadamard_transforms(K // 32))), exact)
    print(f"W4A4 layer loss: RTN-H {l_rh:.4e}  GPTQ-WUSH (GPU) {l_gw:.4e}")
    assert l_gw < l_rh


def test_gptq_c2_full_size(P, G):
    """The c2 layer in full (K=4096, N=6144, 4096 calibration tokens): the oracle redoes the whole schedule."""
    import time
    cfg = I.CONFIGS["c2"]
    L = I.make_layer(cfg)
    W, Xc = O.bf16_bits_to_f64(L["W"]), O.bf16_bits_to_f64(L["X_cal"])
    X = O.bf16_bits_to_f64(L["X"][:256])
    t0 = time.perf_counter()
    T_gpu, c_gpu, s_gpu = _run_gpu(P, G, W, Xc, 1e-2, 1)
    t1 = time.perf_counter()
    T_ref, c_ref, s_ref = Q.gptq_wush_layer(W, Xc, 1e-2)
    t2 = time.perf_counter()
    print(f"c2 GPTQ case: GPU call incl. transfers {t1 - t0:.2f} s, oracle {t2 - t1:.1f} s")
    _compare(T_gpu, c_gpu, s_gpu, T_ref, c_ref, s_ref, W, X, "c2")
