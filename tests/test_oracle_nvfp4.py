"""Pins of the NVFP4 oracle (oracle/wush_nvfp4_oracle.py) to things other than itself:
the FP8 conversion of a library, exact rational arithmetic, brute force, values
worked by hand, and the direction the paper's Table 1 reports."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import wush_nvfp4_oracle as NV
from oracle import wush_oracle as O


# ---------------------------------------------------------------- E4M3 grid
def test_e4m3_values_match_the_library_dtype():
    lib = torch.arange(0, 127, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(NV.e4m3_value(np.arange(127)), lib)
    assert NV.e4m3_value(126) == 448.0 and NV.e4m3_value(1) == 2.0 ** -9


def test_round_e4m3_matches_the_library_conversion():
    rng = np.random.default_rng(1)
    # log-uniform over the whole range incl. subnormals, plus every grid point and midpoint
    r = np.exp(rng.uniform(np.log(2.0 ** -12), np.log(448.0), 200000))
    grid = NV.e4m3_value(np.arange(127))
    mids = (grid[1:] + grid[:-1]) / 2
    r = np.concatenate([r, grid, mids, np.nextafter(mids, 0), np.nextafter(mids, 1e9)]).astype(np.float32)
    lib = torch.from_numpy(r).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(NV.round_e4m3(r), lib)


def test_round_e4m3_saturates():
    assert np.array_equal(NV.round_e4m3(np.array([448.0, 464.0, 465.0, 1e6, 3.4e38])), [126] * 5)


def test_round_e2m1_agrees_with_the_mxfp4_oracle_rounding():
    v = np.linspace(-8, 8, 6401)
    assert np.array_equal(NV.round_e2m1(v), O.round_e2m1(v))


# ---------------------------------------------------------------- quantizer
def test_worked_groups():
    # ts = 1: group AbsMax 6 -> r = 1 -> byte of 1.0 = 7 << 3; the grid points map to themselves
    y = np.array([[0, .5, 1, 1.5, 2, 3, 4, 6, -0.5, -1, -1.5, -2, -3, -4, -6, 0.]], dtype=np.float32)
    c, s = NV.quantize_nvfp4(y, 1.0)
    assert s.tolist() == [[56]]
    assert c[0].tolist() == [0, 1, 2, 3, 4, 5, 6, 7, 9, 10, 11, 12, 13, 14, 15, 0]
    # AbsMax 6*448 with ts = 1 reaches the largest scale; anything larger saturates scale and element
    y2 = np.zeros((1, 16), dtype=np.float32)
    y2[0, 3] = -6 * 448.0
    c2, s2 = NV.quantize_nvfp4(y2, 1.0)
    assert s2.tolist() == [[126]] and c2[0, 3] == 15
    c3, s3 = NV.quantize_nvfp4(y2 * 4, 1.0)
    assert s3.tolist() == [[126]] and c3[0, 3] == 15
    # all-zero group: byte 0, magnitudes 0, sign bits kept
    y4 = np.zeros((1, 16), dtype=np.float32)
    y4[0, 5] = -0.0
    c4, s4 = NV.quantize_nvfp4(y4, 1.0)
    assert s4.tolist() == [[0]] and c4[0].tolist() == [0] * 5 + [8] + [0] * 10


def _exact_reference(y, ts):
    """The definition in exact rational arithmetic, given the scale byte rule."""
    codes = np.zeros(y.shape, dtype=np.uint8)
    sbytes = np.zeros(y.shape[0], dtype=np.uint8)
    grid_s = [Fraction(float(v)) for v in NV.e4m3_value(np.arange(127))]
    grid_e = [Fraction(v) for v in (0, 0.5, 1, 1.5, 2, 3, 4, 6)]
    for g in range(y.shape[0]):
        vals = [Fraction(float(v)) for v in y[g]]
        r = max(abs(v) for v in vals) / (6 * Fraction(float(ts)))
        best = min(range(127), key=lambda b: (abs(grid_s[b] - r), b % 2))      # nearest, ties to even
        sbytes[g] = best
        d = grid_s[best] * Fraction(float(ts))
        for i, v in enumerate(vals):
            if d == 0:
                k = 0
            else:
                k = min(range(8), key=lambda c: (abs(grid_e[c] - abs(v) / d), c % 2))
            codes[g, i] = k | (8 if v < 0 else 0)
    return codes, sbytes


def test_quantizer_against_exact_rational_brute_force():
    rng = np.random.default_rng(7)
    y = (rng.standard_normal((300, 16)) * np.exp(rng.uniform(-6, 6, (300, 1)))).astype(np.float32)
    ts = NV.tensor_scale(y)
    c, s = NV.quantize_nvfp4(y, ts)
    ce, se = _exact_reference(y, ts)
    # FP64 with true divisions: a quotient is off by half an ulp at most, which random inputs never
    # bring within reach of a decision boundary
    assert np.array_equal(s[:, 0], se)
    assert np.array_equal(c, ce)


def test_reconstruction_error_bound():
    rng = np.random.default_rng(3)
    y = (rng.standard_normal((64, 256)) * np.exp(rng.uniform(-3, 3, (64, 1)))).astype(np.float32)
    ts = NV.tensor_scale(y)
    c, s = NV.quantize_nvfp4(y, ts)
    deq = NV.dequantize_nvfp4(c, s, ts)
    d = np.repeat(NV.e4m3_value(s) * float(ts), 16, axis=-1)
    v = np.abs(y.astype(np.float64)) / d
    # half the local E2M1 step (0.25 below 2, 0.5 up to 4, 1 up to 6), or the overshoot past 6
    half = np.where(v <= 2, 0.25, np.where(v <= 4, 0.5, 1.0))
    bound = np.where(v > 6, v - 6, half) * d
    assert np.all(np.abs(y - deq) <= bound * (1 + 1e-6) + 1e-30)
    # the scale is the nearest E4M3 to amax/6 (relative spacing <= 1/8), so no group overshoots
    # 6 by more than one part in 16
    assert v.max() <= 6 * (1 + 1 / 16) * (1 + 1e-6)


def test_power_of_two_invariance():
    rng = np.random.default_rng(5)
    y = rng.standard_normal((8, 64)).astype(np.float32)
    ts = NV.tensor_scale(y)
    c0, s0 = NV.quantize_nvfp4(y, ts)
    c1, s1 = NV.quantize_nvfp4(y * np.float32(2.0 ** 9), ts * np.float32(2.0 ** 9))
    assert np.array_equal(c0, c1) and np.array_equal(s0, s1)
    assert np.array_equal(NV.dequantize_nvfp4(c1, s1, float(ts) * 2.0 ** 9), NV.dequantize_nvfp4(c0, s0, ts) * 2.0 ** 9)


def test_tensor_scale_puts_the_largest_group_on_448():
    rng = np.random.default_rng(11)
    y = rng.standard_normal((32, 128)).astype(np.float32)
    ts = NV.tensor_scale(y)
    _, s = NV.quantize_nvfp4(y, ts)
    assert s.max() == 126


# ---------------------------------------------------------------- transforms of size 16, forward
def test_block16_transform_is_a_block_diagonal_matrix_product():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((5, 48))
    T = rng.standard_normal((3, 16, 16))
    big = np.zeros((48, 48))
    for b in range(3):
        big[16 * b:16 * b + 16, 16 * b:16 * b + 16] = T[b]
    assert np.allclose(NV.transform_act(X, T), X @ big.T, rtol=1e-12, atol=1e-12)
    W = rng.standard_normal((7, 48))
    assert np.allclose(NV.transform_weight(W, T), W @ np.linalg.inv(big), rtol=1e-9, atol=1e-9)
    # the pair leaves the unquantized product unchanged
    assert np.allclose(NV.transform_act(X, T) @ NV.transform_weight(W, T).T, X @ W.T, rtol=1e-9, atol=1e-9)


def _heavy_tailed_layer(seed, M=256, K=256, N=128):
    rng = np.random.default_rng(seed)
    ch = np.exp(rng.standard_normal(K))
    ch[rng.choice(K, 4, replace=False)] *= 30
    X = O.round_to_bf16(rng.standard_normal((M, K)) * ch)
    Xc = O.round_to_bf16(rng.standard_normal((4 * M, K)) * ch)
    W = O.round_to_bf16(rng.standard_normal((N, K)) * 0.02 * np.exp(0.5 * rng.standard_normal((N, 1))))
    return X, Xc, W


def _wush16(W, Xc, lam=1e-2):
    K = W.shape[1]
    T = np.empty((K // 16, 16, 16))
    for b in range(K // 16):
        sl = slice(16 * b, 16 * b + 16)
        T[b] = O.wush_block(O.second_moment(W[:, sl]), O.second_moment(Xc[:, sl]), lam)
    return O.round_to_bf16(T)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_table1_directions_on_synthetic_data(seed):
    """Table 1: with the identity transform NVFP4 loses less than MXFP4 (smaller groups),
    and the 16-block WUSH transform loses less than the identity under NVFP4."""
    X, Xc, W = _heavy_tailed_layer(seed)
    Y = X @ W.T
    K = X.shape[1]
    eye16 = np.broadcast_to(np.eye(16), (K // 16, 16, 16)).copy()
    eye32 = np.broadcast_to(np.eye(32), (K // 32, 32, 32)).copy()
    l_nv_i = O.layer_loss(NV.layer_forward(X, W, eye16), Y)
    l_mx_i = O.layer_loss(O.layer_forward(X, W, eye32), Y)
    l_nv_w = O.layer_loss(NV.layer_forward(X, W, _wush16(W, Xc)), Y)
    assert l_nv_i < l_mx_i
    assert l_nv_w < l_nv_i


def test_forward_reproduces_the_unquantized_product_on_grid_data():
    """Inputs on the NVFP4 grid pass through the layer unchanged, up to the one FP32
    rounding of the weights' tensor scale (1.5 / 2688 is not a binary fraction)."""
    rng = np.random.default_rng(9)
    K = 64
    T = np.broadcast_to(np.eye(16), (K // 16, 16, 16)).copy()
    X = rng.choice([0, .5, 1, 1.5, 2, 3, 4, 6, -1, -6], size=(8, K))
    X[:, ::16] = 6.0                                   # every group's AbsMax is 6
    W = rng.choice([0, 1, -2, 3, 6], size=(4, K)) * 0.25
    W[:, 5::16] = 1.5
    Yq = NV.layer_forward(X, W, T, tsx=np.float32(2.0 ** -4))
    assert np.allclose(Yq, X @ W.T, rtol=2e-7, atol=0)
