"""Pins for the oracle's MXFP4 quantizer.

The quantizer is checked against definitions, not against itself: the E2M1
grid from the fixture file, a brute-force nearest-point search, a brute-force
search over all E8M0 scales, idempotence, and exact integer arithmetic for the
dequantized GEMM.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import wush_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _grid_from_fixture():
    vals = {}
    with open(os.path.join(GOLDEN, "e2m1_grid.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            code, bits, value = line.split()
            assert int(bits, 2) == int(code)
            vals[int(code)] = float(value)
    return vals


def test_grid_matches_format_definition():
    vals = _grid_from_fixture()
    assert [vals[c] for c in range(8)] == list(O.E2M1_VALUES)
    # E2M1 value formula: exponent field e (bias 1), mantissa bit m
    for c in range(8):
        e, m = c >> 1, c & 1
        expect = (m * 0.5) if e == 0 else 2.0 ** (e - 1) * (1 + 0.5 * m)
        assert vals[c] == expect


def test_dequantized_values_are_exact_grid_times_power_of_two():
    rng = np.random.default_rng(0)
    Y = rng.standard_normal((7, 96)) * np.exp2(rng.integers(-20, 20, (7, 96)))
    c, s = O.quantize_mxfp4(Y)
    dq = O.dequantize(c, s)
    ratio = np.abs(dq.reshape(7, 3, 32)) / np.exp2(s.astype(float) - 127)[..., None]
    assert set(np.unique(ratio)) <= set(O.E2M1_VALUES)
    # idempotent: values already on the grid are reproduced bit for bit
    c2, s2 = O.quantize_mxfp4(dq)
    assert np.array_equal(O.dequantize(c2, s2), dq)


def _nearest_code_bruteforce(a):
    """Definition: minimise |a - grid|; among equidistant points take the even code."""
    dist = np.abs(a - O.E2M1_VALUES)
    best = np.flatnonzero(dist == dist.min())
    if len(best) == 1:
        return int(best[0])
    assert len(best) == 2
    return int(best[0] if best[0] % 2 == 0 else best[1])


def test_rounding_is_nearest_with_ties_to_even_code():
    mids = [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]
    pts = list(np.linspace(0, 8, 3201)) + mids
    for mpt in mids:
        pts += [np.nextafter(mpt, 0), np.nextafter(mpt, 10)]
    pts = np.array(pts)
    got = O.round_e2m1(pts)
    want = np.array([_nearest_code_bruteforce(a) for a in pts])
    assert np.array_equal(got, want)
    # the tie table spelled out
    assert list(O.E2M1_VALUES[O.round_e2m1(np.array(mids))]) == [0, 1, 1, 2, 2, 4, 4]
    assert O.round_e2m1(np.array([6.0, 6.5, 7.9, 100.0])).tolist() == [7, 7, 7, 7]
    # symmetric in sign
    assert np.array_equal(O.round_e2m1(-pts), got)


def _bruteforce_scale(group, rule):
    a = np.max(np.abs(group))
    if rule == "nosat":
        # smallest power of two under which no element exceeds the largest E2M1 value
        for byte in range(255):
            if a <= 6.0 * 2.0 ** (byte - 127):
                return byte
        return 254
    # ocp_floor: the byte with 4 <= a / 2^e < 8 (AbsMax lands in the top binade)
    for byte in range(255):
        if 4.0 <= a / 2.0 ** (byte - 127) < 8.0:
            return byte
    return 0 if a < 1 else 254


@pytest.mark.parametrize("rule", ["nosat", "ocp_floor"])
def test_scale_byte_against_search_over_all_scales(rule):
    rng = np.random.default_rng(1)
    groups = []
    for _ in range(300):
        groups.append(rng.standard_normal(32) * np.exp2(rng.uniform(-30, 30)))
    for e in (-20, -3, 0, 1, 7, 40):                       # adversarial maxima
        for top in (6.0, np.nextafter(6.0, 7), np.nextafter(6.0, 5), 4.0,
                    np.nextafter(4.0, 3), 8.0, np.nextafter(8.0, 7), 3.0, 1.5):
            g = rng.uniform(-1, 1, 32) * 2.0 ** e
            g[rng.integers(32)] = -top * 2.0 ** e
            groups.append(g)
    for g in groups:
        _, s = O.quantize_mxfp4(g[None, :], rule)
        assert int(s[0, 0]) == _bruteforce_scale(g, rule), (g.max(), rule)


def test_absmax_scale_never_clips_and_is_tight():
    rng = np.random.default_rng(2)
    Y = rng.standard_normal((50, 64)) * np.exp2(rng.uniform(-10, 10, (50, 1)))
    c, s = O.quantize_mxfp4(Y, "nosat")
    G = np.abs(Y.reshape(50, 2, 32)) / np.exp2(s.astype(float) - 127)[..., None]
    assert G.max() <= 6.0
    assert np.all(G.max(axis=-1) > 3.0)            # one binade lower would clip
    # error never exceeds half the local grid step (in units of the group scale)
    dq = O.dequantize(c, s)
    err = np.abs(dq - Y).reshape(50, 2, 32) / np.exp2(s.astype(float) - 127)[..., None]
    half_step = np.where(G <= 2.0, 0.25, np.where(G <= 4.0, 0.5, 1.0))
    assert np.all(err <= half_step)


def test_absmax_scale_minimises_group_error_among_nonclipping_scales():
    """On tiny blocks: among all scales that do not clip, the AbsMax scale gives
    the smallest squared error (a coarser grid can only be worse or equal)."""
    rng = np.random.default_rng(3)
    for _ in range(40):
        g = rng.standard_normal(32) * np.exp2(rng.uniform(-5, 5))
        _, s = O.quantize_mxfp4(g[None], "nosat")
        s0 = int(s[0, 0])
        errs = {}
        for byte in range(s0, min(s0 + 6, 255)):
            v = g / 2.0 ** (byte - 127)
            q = O.E2M1_VALUES[O.round_e2m1(v)] * np.sign(v) * 2.0 ** (byte - 127)
            errs[byte] = np.sum((q - g) ** 2)
        assert min(errs, key=errs.get) == s0 or errs[s0] <= min(errs.values()) * (1 + 1e-12)


def test_zero_group_denormals_and_signed_zero():
    Y = np.zeros((1, 64))
    Y[0, 32] = -1e-42                                # below the smallest E8M0 scale's grid
    Y[0, 33] = 3.0e-39
    c, s = O.quantize_mxfp4(Y)
    assert s.tolist() == [[0, 0]]
    assert np.all(c[0, :32] == 0)
    assert c[0, 32] == 8                             # -0: sign kept, magnitude 0
    # 3e-39 / 2^-127 = 0.51 -> 0.5
    assert c[0, 33] == 1
    assert O.dequantize(c, s)[0, 33] == 0.5 * 2.0 ** -127


def test_pack_unpack_nibble_order():
    codes = np.arange(16, dtype=np.uint8)[None, :].repeat(2, 0)
    p = O.pack_codes(codes)
    assert p.shape == (2, 8)
    assert p[0, 0] == 0x10 and p[0, 1] == 0x32 and p[0, 7] == 0xFE
    assert np.array_equal(O.unpack_codes(p), codes)


def test_dequant_gemm_is_exact_against_integer_arithmetic():
    """Dequantized values are (integer/2) * 2^e: the FP64 GEMM must agree with
    exact integer accumulation (Python big ints) on a small case."""
    rng = np.random.default_rng(4)
    X = rng.standard_normal((5, 96)) * np.exp2(rng.integers(-4, 4, (5, 96)))
    W = rng.standard_normal((6, 96)) * 0.02
    xc, xs = O.quantize_mxfp4(X)
    wc, ws = O.quantize_mxfp4(W)
    Y = O.linear_dequant(xc, xs, wc, ws)
    twice = (2 * O.E2M1_VALUES).astype(int)
    for m, n in itertools.product(range(5), range(6)):
        acc, base = 0, -400
        for k in range(96):
            ix = int(twice[xc[m, k] & 7]) * (-1 if xc[m, k] & 8 else 1)
            iw = int(twice[wc[n, k] & 7]) * (-1 if wc[n, k] & 8 else 1)
            e = int(xs[m, k // 32]) - 127 + int(ws[n, k // 32]) - 127
            acc += ix * iw * (1 << (e - base))
        exact = acc / 4.0 * 2.0 ** base
        assert Y[m, n] == pytest.approx(exact, rel=1e-13, abs=0)


def test_bf16_rounding_helper():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -9, -3.14159, 1e-3, 65504.0])
    r = O.round_to_bf16(x)
    assert r[0] == 1.0
    assert r[1] == 1.0                      # tie -> even significand
    assert r[2] == 1.0 + 2 ** -6            # tie -> even (1 + 4*2^-8)
    assert r[3] == 1.0
    # agrees with the widen/narrow definition on random data (float32 inputs: no double rounding)
    rng = np.random.default_rng(5)
    f = (rng.standard_normal(10000) * np.exp2(rng.uniform(-20, 20, 10000))).astype(np.float32)
    u = f.view(np.uint32)
    ref = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16).astype(np.uint32).view(np.float32)
    assert np.array_equal(O.round_to_bf16(f.astype(np.float64)), ref.astype(np.float64))
    assert np.array_equal(O.bf16_bits_to_f64(O.bf16_values_to_bits(r)), r)
