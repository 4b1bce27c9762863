"""GPU parity of the on-device transform construction (Alg. 1 + the moment step
of Alg. 2, RTN case) against the oracle's FP64 construction.

The unrounded FP64 T must agree to ~1e-9 of the block's largest entry (both
sides are FP64; only summation order and the SVD algorithm differ).  The BF16
result must equal the oracle's rounded T except for entries whose FP64 value sits
within that distance of a BF16 rounding boundary.
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


CASES = {
    "c1": (I.CONFIGS["c1"], 1e-2),
    "c1_lam0": (I.CONFIGS["c1"], 0.0),
    "ragged_rows": (I.scaled(I.CONFIGS["c1"], K=32 * 5, N=77, calib_tokens=333, n_outlier=2), 1e-4),
    "c2_cut": (I.scaled(I.CONFIGS["c2"], K=1024, N=1536, calib_tokens=4096, n_outlier=5), 1e-2),
    "c3_cut": (I.scaled(I.CONFIGS["c3"], K=32 * 20, N=512, calib_tokens=3000, n_outlier=6), 1e-2),
}


def _gpu_transforms(P, G, L, lam):
    import torch
    cfg = L["cfg"]
    C = cfg.C
    T = torch.empty((C, 32, 32), dtype=torch.bfloat16, device="cuda")
    T64 = torch.full((C, 32, 32), float("nan"), dtype=torch.float64, device="cuda")
    ws = G.empty_u8(P.wush_build_transforms_workspace(cfg.K))
    P.wush_build_transforms(G.bf16_dev(L["W"]), G.bf16_dev(L["X_cal"]), lam, T, ws, T_f64=T64)
    P.wush_build_transforms_status(ws, cfg.K)
    return G.host(T), T64.cpu().numpy()


@pytest.mark.parametrize("name", list(CASES))
def test_build_transforms_matches_oracle(P, G, name):
    cfg, lam = CASES[name]
    L = I.make_layer(cfg)
    W, Xc = O.bf16_bits_to_f64(L["W"]), O.bf16_bits_to_f64(L["X_cal"])
    T_ref = O.build_transforms(W, Xc, lam)
    t_bits, t64 = _gpu_transforms(P, G, L, lam)
    assert np.isfinite(t64).all()
    scale = np.max(np.abs(T_ref), axis=(1, 2), keepdims=True)
    err = np.max(np.abs(t64 - T_ref) / scale)
    assert err <= 1e-9, err
    # BF16 output: identical to the oracle's rounding except at rounding boundaries
    ref_bits = O.bf16_values_to_bits(O.round_to_bf16(T_ref))
    diff = t_bits != ref_bits
    assert diff.mean() <= 1e-4
    if diff.any():
        ulp = np.abs(O.bf16_bits_to_f64(t_bits)[diff] - O.bf16_bits_to_f64(ref_bits)[diff])
        gap = np.abs(np.abs(t64[diff] - T_ref[diff]))
        assert np.all(ulp <= np.abs(T_ref[diff]) * 2.0 ** -7) and np.all(gap <= 1e-9 * scale.repeat(32, 1).repeat(32, 2)[diff])
    # the device-built transforms satisfy the paper's identities on their own
    b = cfg.C // 2
    sl = slice(32 * b, 32 * b + 32)
    Wp, Xp, U, s, V = O.wush_factors(O.second_moment(W[:, sl]), O.second_moment(Xc[:, sl]), lam)
    eq = t64[b] @ O.damped(O.second_moment(Xc[:, sl]), lam) @ t64[b].T
    assert np.allclose(np.diag(eq), s.sum() / 32, rtol=1e-8)
    assert O.fp_model_objective(t64[b], Wp, Xp) == pytest.approx(s.sum() ** 2 / 32, rel=1e-8)


def test_device_built_transforms_drive_the_layer(P, G):
    """Whole offline + online path on the device: build T, prepare W, quantize X, GEMM."""
    import torch
    cfg = CASES["c2_cut"][0]
    cfg = I.scaled(cfg, M=300)
    L = I.make_layer(cfg)
    M, K, N = cfg.M, cfg.K, cfg.N
    t_bits, _ = _gpu_transforms(P, G, L, 1e-2)
    T = O.bf16_bits_to_f64(t_bits)
    Td = G.bf16_dev(t_bits)
    Xq, Xs = G.empty_u8(M, K // 2), G.empty_u8(M, K // 32)
    Wq, Ws = G.empty_u8(N, K // 2), G.empty_u8(N, K // 32)
    ws = G.empty_u8(P.wush_prepare_weight_workspace(N, K))
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    P.wush_prepare_weight(G.bf16_dev(L["W"]), Td, Wq, Ws, ws)
    P.wush_workspace_status(ws, K)
    P.wush_quantize_act(G.bf16_dev(L["X"]), Td, Xq, Xs)
    P.wush_linear(Xq, Xs, Wq, Ws, Y)
    torch.cuda.synchronize()
    X, W = O.bf16_bits_to_f64(L["X"]), O.bf16_bits_to_f64(L["W"])
    y = O.bf16_bits_to_f64(G.host(Y))
    assert O.rel_fro(y, O.layer_forward(X, W, T)) <= 2e-3
    # and it beats the plain Hadamard transform on the same data, as the oracle does
    Th = O.round_to_bf16(O.hadamard_transforms(cfg.C))
    exact = X @ W.T
    assert O.layer_loss(y, exact) < O.layer_loss(O.layer_forward(X, W, Th), exact)


def test_build_transforms_flags_indefinite_moment(P, G):
    """lambda = 0 with fewer calibration tokens than channels: M_X is singular."""
    import torch
    cfg = I.scaled(I.CONFIGS["c1"], K=64, N=64, calib_tokens=8, n_outlier=1)
    L = I.make_layer(cfg)
    T = torch.empty((2, 32, 32), dtype=torch.bfloat16, device="cuda")
    ws = G.empty_u8(P.wush_build_transforms_workspace(64))
    P.wush_build_transforms(G.bf16_dev(L["W"]), G.bf16_dev(L["X_cal"]), 0.0, T, ws)
    with pytest.raises(P.WushError) as ei:
        P.wush_build_transforms_status(ws, 64)
    assert ei.value.code == 7


@pytest.mark.parametrize("name", ["c1", "c1_lam0", "ragged_rows", "c2_cut"])
def test_build_transforms_16_matches_oracle(P, G, name):
    """The same construction with 16 x 16 blocks (the NVFP4 variant)."""
    import torch
    cfg, lam = CASES[name]
    L = I.make_layer(cfg)
    W, Xc = O.bf16_bits_to_f64(L["W"]), O.bf16_bits_to_f64(L["X_cal"])
    C16 = cfg.K // 16
    T_ref = np.empty((C16, 16, 16))
    for b in range(C16):
        sl = slice(16 * b, 16 * b + 16)
        T_ref[b] = O.wush_block(O.second_moment(W[:, sl]), O.second_moment(Xc[:, sl]), lam)
    T = torch.empty((C16, 16, 16), dtype=torch.bfloat16, device="cuda")
    T64 = torch.full((C16, 16, 16), float("nan"), dtype=torch.float64, device="cuda")
    ws = G.empty_u8(P.wush_build_transforms_workspace(cfg.K))
    P.wush_build_transforms_nvfp4(G.bf16_dev(L["W"]), G.bf16_dev(L["X_cal"]), lam, T, ws, T_f64=T64)
    P.wush_build_transforms_status(ws, cfg.K)
    t_bits, t64 = G.host(T), T64.cpu().numpy()
    assert np.isfinite(t64).all()
    scale = np.max(np.abs(T_ref), axis=(1, 2), keepdims=True)
    assert np.max(np.abs(t64 - T_ref) / scale) <= 1e-9
    ref_bits = O.bf16_values_to_bits(O.round_to_bf16(T_ref))
    diff = t_bits != ref_bits
    assert diff.mean() <= 1e-4
    if diff.any():
        assert np.all(np.abs(t64[diff] - T_ref[diff]) <= 1e-9 * scale.repeat(16, 1).repeat(16, 2)[diff])
    # the identities of the construction hold for a 16-block as well
    b = C16 // 2
    sl = slice(16 * b, 16 * b + 16)
    Wp, Xp, U, s, V = O.wush_factors(O.second_moment(W[:, sl]), O.second_moment(Xc[:, sl]), lam)
    eq = t64[b] @ O.damped(O.second_moment(Xc[:, sl]), lam) @ t64[b].T
    assert np.allclose(np.diag(eq), s.sum() / 16, rtol=1e-8)
    assert O.fp_model_objective(t64[b], Wp, Xp) == pytest.approx(s.sum() ** 2 / 16, rel=1e-8)
