"""The kernel arithmetic models of tests/kernel_models.py (the steps the NVFP4 and INT4 GPU quantizers
take, in their working precision) against the definitions in oracle/ and against exact rational
arithmetic: a model may differ from the definition only where a value sits within rounding of a
decision boundary, and then by one code (or one BF16 step of the scale).  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import wush_int4_oracle as Q4
from oracle import wush_nvfp4_oracle as NV
from oracle import wush_oracle as O
from tests import kernel_models as KM


def _spread(shape, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(shape) * np.exp(rng.uniform(-6, 6, (shape[0], 1)))).astype(np.float32)


@pytest.mark.parametrize("prec,tol,rate_bar", [(np.float32, 2e-6, 1e-3), (np.float64, 1e-14, 1e-9)])
def test_nvfp4_steps_differ_from_the_definition_only_at_boundaries(prec, tol, rate_bar):
    y = _spread((4000, 64), 1)
    ts = NV.tensor_scale(y)
    cm, sm = KM.nvfp4_steps(y, ts, prec)
    cd, sd = NV.quantize_nvfp4(y, ts)
    rate, unexplained = KM.nvfp4_explained(y.astype(np.float64), ts, cm, sm, cd, sd, tol=tol)
    assert rate <= rate_bar and unexplained == 0, (rate, unexplained)
    assert np.all(np.abs((cm & 7).astype(int) - (cd & 7)) <= 1)
    assert np.all(np.abs(sm.astype(int) - sd) <= 1)


@pytest.mark.parametrize("prec,tol,rate_bar", [(np.float32, 2e-6, 2e-3), (np.float64, 1e-14, 1e-9)])
def test_int4_steps_differ_from_the_definition_only_at_boundaries(prec, tol, rate_bar):
    y = _spread((4000, 64), 2)
    qm, sm = KM.int4_steps(y, prec)
    qd, sd = Q4.quantize_int4(y)
    rate, unexplained = KM.int4_explained(y.astype(np.float64), qm, sm, qd, sd, tol=tol)
    assert rate <= rate_bar and unexplained == 0, (rate, unexplained)
    same = sm == sd
    assert np.all(np.abs(qm.reshape(-1, 2, 32)[same].astype(int) - qd.reshape(-1, 2, 32)[same]) <= 1)
    # a scale that differs is the neighbouring BF16 number
    assert np.all(np.abs(sm.astype(int) - sd) <= 1)


def test_models_on_the_exact_boundaries():
    """Values placed ON code midpoints: the definition resolves the tie to the even code; the FP32 steps
    may land on either neighbour (the reciprocal is rounded), never further."""
    s = 0.4375                                        # a BF16 number
    g = np.zeros((1, 32), dtype=np.float32)
    g[0, :15] = (np.arange(-8, 7) + 0.5) * s          # every midpoint between neighbouring codes
    # choose the remaining entries so that STEP * rms lands in the interior of the BF16 cell of s
    rest = np.sqrt(max((s / Q4.STEP) ** 2 * 32 - float(np.sum(g.astype(np.float64) ** 2)), 0.0) / 17)
    g[0, 15:] = rest
    qd, sd = Q4.quantize_int4(g)
    if O.bf16_bits_to_f64(sd)[0, 0] == s:             # the construction hit the intended scale
        exp = np.array([int(np.rint(k + 0.5)) for k in range(-8, 7)])       # half to even
        assert np.array_equal(qd[0, :15], np.clip(exp, -8, 7))
        qm, sm = KM.int4_steps(g, np.float32)
        assert np.array_equal(sm, sd) and np.all(np.abs(qm.astype(int) - qd) <= 1)


def test_fp32_models_against_exact_rational_arithmetic():
    """The FP32 step lists themselves, pinned to exact arithmetic as the definitions are: rare
    differences, never more than one code."""
    y = _spread((200, 16), 7)
    ts = NV.tensor_scale(y)
    c, s = KM.nvfp4_steps(y, ts, np.float32)
    grid_s = [Fraction(float(v)) for v in NV.e4m3_value(np.arange(127))]
    grid_e = [Fraction(v) for v in (0, 0.5, 1, 1.5, 2, 3, 4, 6)]
    n_diff = 0
    for g in range(y.shape[0]):
        vals = [Fraction(float(v)) for v in y[g]]
        r = max(abs(v) for v in vals) / (6 * Fraction(float(ts)))
        best = min(range(127), key=lambda b: (abs(grid_s[b] - r), b % 2))
        if best != s[g, 0]:
            assert abs(best - int(s[g, 0])) == 1
            continue
        d = grid_s[best] * Fraction(float(ts))
        for i, v in enumerate(vals):
            k = 0 if d == 0 else min(range(8), key=lambda cc: (abs(grid_e[cc] - abs(v) / d), cc % 2))
            if k != (c[g, i] & 7):
                n_diff += 1
                assert abs(k - int(c[g, i] & 7)) == 1
    assert n_diff <= 4
