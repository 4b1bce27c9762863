"""Pins for the oracle's layer forward on the synthetic workloads.

* with the quantizer removed, the transformed product equals X W^T (the
  weight transform is the inverse transpose of the activation transform);
* on outlier-heavy inputs the WUSH transform gives a lower quantized-output
  loss than the plain blockwise Hadamard (direction of the paper's layerwise
  loss table, MXFP4 rows);
* the seeded generators are reproducible and have the advertised structure.
"""
import os

import numpy as np
import pytest

import wush_inputs as I
from oracle import wush_oracle as O


def _f64(bits):
    return O.bf16_bits_to_f64(bits)


@pytest.fixture(scope="module")
def c1():
    L = I.make_layer(I.CONFIGS["c1"])
    X, Xc, W = _f64(L["X"]), _f64(L["X_cal"]), _f64(L["W"])
    T = O.round_to_bf16(O.build_transforms(W, Xc, 1e-2))
    return L, X, Xc, W, T


def test_generators_are_seeded_and_structured():
    cfg = I.CONFIGS["c1"]
    A, B = I.make_layer(cfg), I.make_layer(cfg)
    for k in ("X", "X_cal", "W"):
        assert A[k].dtype == np.uint16 and np.array_equal(A[k], B[k])
    assert A["X"].shape == (16, 256) and A["X_cal"].shape == (512, 256) and A["W"].shape == (256, 256)
    assert len(A["outlier_idx"]) == 2
    rms = np.sqrt(np.mean(_f64(A["X_cal"]) ** 2, axis=0))
    assert np.allclose(rms, A["chan_scale"], rtol=0.2)
    assert np.all(rms[A["outlier_idx"]] > 5 * np.median(rms))
    assert I.CONFIGS["c2"].n_outlier == 20 and I.CONFIGS["c3"].n_outlier == 143 and I.CONFIGS["c5"].n_outlier == 41
    # BF16 helpers agree with the oracle's independent implementation
    f = I.random_f32((1000,), 3)
    assert np.array_equal(_f64(I.f32_to_bf16_bits(f)), O.round_to_bf16(f.astype(np.float64)))
    assert np.array_equal(I.bf16_bits_to_f32(A["X"]).astype(np.float64), _f64(A["X"]))


def test_unquantized_invariance(c1):
    _, X, _, W, T = c1
    Y = O.transform_act(X, T) @ O.transform_weight(W, T).T
    assert O.rel_fro(Y, X @ W.T) < 1e-10
    # also with the Hadamard baseline and with random invertible blocks
    Th = O.hadamard_transforms(8)
    assert O.rel_fro(O.transform_act(X, Th) @ O.transform_weight(W, Th).T, X @ W.T) < 1e-12
    Tr = O.bf16_bits_to_f64(I.make_transforms_random(8, 1))
    assert O.rel_fro(O.transform_act(X, Tr) @ O.transform_weight(W, Tr).T, X @ W.T) < 1e-10


def test_transform_index_convention(c1):
    """Yt[m, 32b+j] = sum_k X[m,32b+k] T[b][j][k]; Wt uses inv(T[b])[k][j]."""
    _, X, _, W, T = c1
    Yt, Wt = O.transform_act(X, T), O.transform_weight(W, T)
    m, b, j = 3, 5, 17
    assert Yt[m, 32 * b + j] == pytest.approx(sum(X[m, 32 * b + k] * T[b, j, k] for k in range(32)), rel=1e-12)
    Tinv = np.linalg.inv(T[b])
    assert Wt[7, 32 * b + j] == pytest.approx(sum(W[7, 32 * b + k] * Tinv[k, j] for k in range(32)), rel=1e-10)
    # block-diagonal: channels outside block b do not leak into block b
    X2 = X.copy()
    X2[:, :32 * b] = 0
    X2[:, 32 * b + 32:] = 0
    assert np.array_equal(O.transform_act(X2, T)[:, 32 * b:32 * b + 32], Yt[:, 32 * b:32 * b + 32])


def _losses(cfg, lam=1e-2, eval_on="fresh"):
    L = I.make_layer(cfg)
    X, Xc, W = _f64(L["X"]), _f64(L["X_cal"]), _f64(L["W"])
    Xe = X if eval_on == "fresh" else Xc
    Yref = Xe @ W.T
    out = {}
    Tw = O.round_to_bf16(O.build_transforms(W, Xc, lam))
    Th = O.round_to_bf16(O.hadamard_transforms(cfg.C))
    Ti = np.broadcast_to(np.eye(32), (cfg.C, 32, 32)).copy()
    for name, T in (("wush", Tw), ("h", Th), ("i", Ti)):
        out[name] = O.layer_loss(O.layer_forward(Xe, W, T), Yref)
    return out


@pytest.mark.parametrize("lam", [0.0, 1e-4, 1e-2])
def test_wush_beats_hadamard_on_outlier_heavy_inputs_c1(lam):
    cfg = I.scaled(I.CONFIGS["c1"], M=256)      # more evaluation tokens for a stable estimate
    for eval_on in ("fresh", "calib"):
        l = _losses(cfg, lam, eval_on)
        assert l["wush"] < l["h"], (lam, eval_on, l)


def test_wush_beats_hadamard_scaled_c2_and_c3():
    # same laws and seeds as configs 2 and 3, shapes cut down to keep the CPU suite short
    c2 = I.scaled(I.CONFIGS["c2"], M=256, K=1024, N=512, calib_tokens=2048, n_outlier=5)
    c3 = I.scaled(I.CONFIGS["c3"], M=256, K=1024, N=512, calib_tokens=2048, n_outlier=10)
    ratios = []
    for cfg in (c2, c3):
        l = _losses(cfg)
        assert l["wush"] < l["h"], (cfg.name, l)
        ratios.append(l["wush"] / l["h"])
    # context: the paper's MXFP4 WUSH/H ratios on a real model lie in this range
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table1_mxfp4_rtn_loss.txt")) as f:
        for line in f:
            if not line.startswith("#") and line.strip():
                k, *v = line.split()
                rows[k] = np.array([float(t) for t in v])
    paper = rows["WUSH"] / rows["H"]
    assert 0.38 < paper.min() < 0.39 and 0.86 < paper.max() < 0.88
    assert all(r < 1.0 for r in ratios)
