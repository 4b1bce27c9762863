"""Pins of the GPTQ-case oracle (Alg. 2, GPTQ case) against things other than itself:
the OBS/OBQ update written with explicit inverses of the remaining sub-Hessian, the
unblocked GPTQ recursion over all input channels, the special case with no correlations
(reduces to the RTN case, pinned elsewhere), and the direction of the loss."""
import numpy as np
import pytest

import wush_inputs as I
from oracle import wush_gptq_oracle as Q
from oracle import wush_oracle as O


def _spd(d, seed, cond=50.0):
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((4 * d, d)) * np.geomspace(1.0, cond ** 0.5, d)
    return A.T @ A / (4 * d)


def test_gptq_block_is_the_obs_update():
    """Quantizing coordinate r and compensating on the remaining ones must be the OBS step
    delta = -(w_r - q_r) / [inv(H_rest)]_rr * [inv(H_rest)]_r,rest with H_rest the Hessian restricted
    to the coordinates not yet quantized -- here with explicit inverses, no Cholesky."""
    d, N = 8, 5
    H = _spd(d, 1)
    rng = np.random.default_rng(2)
    W = rng.standard_normal((N, d)) * 3.0
    codes, sb, deq = Q.gptq_block(W, H)
    assert np.array_equal(sb, O.scale_bytes(np.max(np.abs(W), axis=1)))
    for n in range(N):
        w = W[n].copy()
        for r in range(d):
            Hinv = np.linalg.inv(H[r:, r:])
            c, q = Q.quantize_static(w[r:r + 1], sb[n:n + 1])
            assert c[0] == codes[n, r] and q[0] == deq[n, r]
            w[r + 1:] -= (w[r] - q[0]) / Hinv[0, 0] * Hinv[0, 1:]


def test_block_hessian_is_the_conditional_hessian():
    """(L_ii L_ii^T)^-1 must be the Hessian of block i once blocks < i are fixed:
    the inverse of the leading d x d block of inv(H[i:, i:])."""
    K, d = 96, 32
    H = _spd(K, 3)
    lam = 0.01
    Hd = H + lam * np.trace(H) / K * np.eye(K)
    L = Q.inverse_cholesky(H, lam)
    assert np.allclose(L @ L.T @ Hd, np.eye(K), atol=1e-9) and np.allclose(L, np.tril(L))
    for i in range(K // d):
        s = slice(d * i, d * i + d)
        cond = np.linalg.inv(np.linalg.inv(Hd[d * i:, d * i:])[:d, :d])
        blk = np.linalg.inv(L[s, s] @ L[s, s].T)
        assert np.allclose(blk, cond, rtol=1e-8, atol=1e-10)


def _unblocked_gptq(W, X_cal, lam):
    """Plain GPTQ over all K input channels, one at a time, with the full upper Cholesky factor
    of the inverse Hessian; the scale of a group is taken when its first channel is reached."""
    W = np.array(W, dtype=np.float64)
    N, K = W.shape
    H = Q.hessian(X_cal)
    Hd = H + lam * np.trace(H) / K * np.eye(K)
    R = np.linalg.cholesky(np.linalg.inv(Hd)).T
    codes = np.zeros((N, K), dtype=np.uint8)
    scales = np.zeros((N, K // 32), dtype=np.uint8)
    for c in range(K):
        g = c // 32
        if c % 32 == 0:
            scales[:, g] = O.scale_bytes(np.max(np.abs(W[:, c:c + 32]), axis=1))
        codes[:, c], q = Q.quantize_static(W[:, c], scales[:, g])
        err = (W[:, c] - q) / R[c, c]
        W[:, c + 1:] -= np.outer(err, R[c, c + 1:])
    return codes, scales


def test_blocked_schedule_equals_unblocked_gptq_for_the_identity_transform():
    cfg = I.scaled(I.CONFIGS["c1"], M=8, K=128, N=48, calib_tokens=400, n_outlier=2)
    L = I.make_layer(cfg)
    W, Xc = O.bf16_bits_to_f64(L["W"]), O.bf16_bits_to_f64(L["X_cal"])
    T, codes, scales = Q.gptq_wush_layer(W, Xc, 1e-2, transform="identity")
    c2, s2 = _unblocked_gptq(W, Xc, 1e-2)
    assert np.array_equal(scales, s2)
    assert np.mean(codes != c2) <= 1e-3        # FP64 rounding order differs; flips only at exact boundaries
    assert np.array_equal(T, np.broadcast_to(np.eye(32), T.shape))


def test_uncorrelated_activations_reduce_to_the_rtn_case():
    """With H = identity nothing propagates between blocks (L is diagonal): the transforms are the
    RTN case's.  Inside a block the transformed Hessian is T T^T, so an orthogonal transform
    (Hadamard) leaves nothing to propagate at all and the codes are the RTN codes; for WUSH the
    scales (taken before any update) and the first transformed channel of every block (no update
    reaches it) are the RTN case's."""
    K, N = 128, 40
    cfg = I.scaled(I.CONFIGS["c1"], M=8, K=K, N=N, calib_tokens=K, n_outlier=2)
    W = O.bf16_bits_to_f64(I.make_layer(cfg)["W"])
    Xc = np.sqrt(K) * np.eye(K)
    # the BF16-rounded Hadamard matrix is orthogonal only to 2^-9, hence a handful of boundary flips at most
    T, codes, scales = Q.gptq_wush_layer(W, Xc, 1e-2, transform="hadamard")
    TH = O.round_to_bf16(O.hadamard_transforms(K // 32))
    c_rtn, s_rtn = O.quantize_mxfp4(O.transform_weight(W, TH))
    assert np.array_equal(T, TH) and np.array_equal(scales, s_rtn)
    assert np.mean(codes != c_rtn) <= 5e-3
    T, codes, scales = Q.gptq_wush_layer(W, Xc, 1e-2)
    T_rtn = O.round_to_bf16(O.build_transforms(W, Xc, 1e-2))
    assert np.array_equal(T, T_rtn)
    c_rtn, s_rtn = O.quantize_mxfp4(O.transform_weight(W, T_rtn))
    assert np.array_equal(scales, s_rtn) and np.array_equal(codes[:, ::32], c_rtn[:, ::32])
    assert np.mean(codes != c_rtn) > 0.01      # and the rest does move


@pytest.mark.parametrize("transform", ["identity", "hadamard", "wush"])
def test_gptq_lowers_the_weight_only_output_error(transform):
    """GPTQ's propagation minimizes the output error under unquantized activations; on correlated
    synthetic activations it must beat RTN with the same kind of transform."""
    cfg = I.scaled(I.CONFIGS["c1"], M=256, K=256, N=96, calib_tokens=1024, n_outlier=3)
    L = I.make_layer(cfg)
    W, Xc, X = (O.bf16_bits_to_f64(L[k]) for k in ("W", "X_cal", "X"))
    rng = np.random.default_rng(5)
    mix = np.eye(256) + 0.3 * rng.standard_normal((256, 256)) / 16.0    # correlate the channels
    Xc, X = Xc @ mix, X @ mix
    T, codes, scales = Q.gptq_wush_layer(W, Xc, 1e-2, transform=transform)
    if transform == "wush":
        T0 = O.round_to_bf16(O.build_transforms(W, Xc, 1e-2))
    elif transform == "hadamard":
        T0 = O.round_to_bf16(O.hadamard_transforms(8))
    else:
        T0 = np.broadcast_to(np.eye(32), (8, 32, 32)).copy()
    c0, s0 = O.quantize_mxfp4(O.transform_weight(W, T0))
    gptq, rtn = Q.proxy_loss(T, codes, scales, W, X), Q.proxy_loss(T0, c0, s0, W, X)
    print(f"{transform}: weight-only output MSE  RTN {rtn:.4e}  GPTQ {gptq:.4e}")
    assert gptq < rtn


def test_w4a4_layer_loss_gptq_wush_vs_rtn_hadamard():
    """Direction of Table 1 / Table 2 on synthetic data: GPTQ + WUSH gives a lower W4A4 layer loss than
    RTN + Hadamard.  Absolute values are unpinned (the paper's need its models and data)."""
    cfg = I.scaled(I.CONFIGS["c1"], M=256, K=256, N=96, calib_tokens=1024, n_outlier=3)
    L = I.make_layer(cfg)
    W, Xc, X = (O.bf16_bits_to_f64(L[k]) for k in ("W", "X_cal", "X"))
    T, codes, scales = Q.gptq_wush_layer(W, Xc, 1e-2)
    xc, xs = O.quantize_mxfp4(O.transform_act(X, T))
    y_gw = O.dequantize(xc, xs) @ O.dequantize(codes, scales).T
    TH = O.round_to_bf16(O.hadamard_transforms(8))
    y_rh = O.layer_forward(X, W, TH)
    ref = X @ W.T
    l_gw, l_rh = O.layer_loss(y_gw, ref), O.layer_loss(y_rh, ref)
    print(f"W4A4 layer loss: RTN-H {l_rh:.4e}  GPTQ-WUSH {l_gw:.4e}")
    assert l_gw < l_rh
