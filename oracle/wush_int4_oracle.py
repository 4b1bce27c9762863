"""CPU oracle for the INT4 variant of the quantized layer -- TEST INFRASTRUCTURE ONLY.

The paper's layerwise experiment (Table 1, "Layerwise Quantization Loss") also
runs the method with a format it calls INT4: "4-bit integers with Gaussian MSE
clipping and BF16 scales of group size 32"; the transform block stays 32.  This
module writes that variant out in plain numpy.  It shares no code with the HIP
library and is imported only by tests and the benchmark's CPU-baseline leg.

Readings of what the paper leaves open (listed in the design notes as well):
  * grid: the 16 two's-complement integers -8 .. 7; a stored element is worth
    q * scale, scale = a BF16 number per group of 32 consecutive channels.
  * "Gaussian MSE clipping": the scale is the step that minimizes the mean
    squared error of this 16-level quantizer on a zero-mean Gaussian of the
    group's standard deviation: scale = STEP * sigma, STEP = the minimizer for a
    unit Gaussian (gaussian_mse below gives the error in closed form; a pin
    recomputes the minimizer), sigma = the group's root mean square (zero mean is
    the method's own assumption, Assumption 1 of the error analysis).  Values
    beyond -8.5 / 7.5 steps are clipped; that is the point of the rule, and it is
    what Table 1 shows: with the identity transform INT4 loses an order of
    magnitude more than MXFP4 (outlier channels are clipped), behind a Hadamard
    or WUSH transform it loses less -- a pattern an AbsMax-based step would not give.
  * elements: q = clip(round-half-even(v / scale), -8, 7); a scale below BF16's
    normal range (an all-zero group) is stored as 0 and gives q = 0.
  * arithmetic: every step is one IEEE operation in ONE working precision `prec`
    (FP32 for activations, the precision of the kernel's accumulators; FP64 for
    the offline weight path), in this order:
        t_i = v_i * v_i,   s_lo = t_0 + ... + t_15,  s_hi = t_16 + ... + t_31
        (each left to right),  ss = s_lo + s_hi,   sigma = sqrt(ss / 32),
        scale = BF16(STEP * sigma)  (STEP rounded to `prec`; round to nearest even),
        rcp = 1 / scale,            q = clip(rint(v * rcp), -8, 7).
    The two half sums are how the GPU holds a group (16 channels per lane).

Conventions: as in wush_oracle.py (row-major, channels last, T[b][j][k]); codes
are int8 values -8 .. 7; packed: two's-complement nibbles, even k in the low
nibble; scales travel as BF16 bit patterns (uint16).
Pins: tests/test_oracle_int4.py.
"""
from __future__ import annotations

import math

import numpy as np

from . import wush_oracle as O

G = 32
QMIN, QMAX = -8, 7
STEP = 0.33860793          # argmin of gaussian_mse over the step, to 8 digits (pinned by a test)


def _phi(x):
    return math.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)


def _Phi(x):
    return 0.5 * (1.0 + math.erf(x / math.sqrt(2.0)))


def gaussian_mse(step: float, levels=None) -> float:
    """E (x - Q(x))^2 for x ~ N(0, 1) and the quantizer that maps x to the nearest
    of `levels` (default: step * {-8..7}), in closed form cell by cell:
    int (x - c)^2 phi = (1 + c^2) Phi - (x - 2c) phi."""
    if levels is None:
        levels = [step * q for q in range(QMIN, QMAX + 1)]
    levels = sorted(levels)
    total = 0.0
    for i, c in enumerate(levels):
        a = -math.inf if i == 0 else 0.5 * (levels[i - 1] + c)
        b = math.inf if i == len(levels) - 1 else 0.5 * (c + levels[i + 1])

        def F(x):
            if math.isinf(x):
                return (1.0 + c * c) if x > 0 else 0.0
            return (1.0 + c * c) * _Phi(x) - (x - 2.0 * c) * _phi(x)
        total += F(b) - F(a)
    return total


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Non-negative finite values (FP32 or FP64) -> BF16 bit patterns, one rounding
    to nearest even."""
    v = O.round_to_bf16(np.asarray(x, dtype=np.float64))
    return O.bf16_values_to_bits(v)


def quantize_int4(Y: np.ndarray, prec=np.float32):
    """INT4 quantizer on values Y [..., K].  Returns (q int8 [..., K] in -8..7,
    scale bits uint16 [..., K/32])."""
    Y = np.asarray(Y, dtype=prec)
    *lead, K = Y.shape
    Gr = Y.reshape(-1, K // G, G)
    with np.errstate(over="ignore"):                           # squares beyond the range of `prec` give an infinite scale
        t = (Gr * Gr).astype(prec)
        s_lo = np.zeros(t.shape[:2], dtype=prec)
        s_hi = np.zeros(t.shape[:2], dtype=prec)
        for i in range(16):                                    # left to right, one rounding per addition
            s_lo = (s_lo + t[..., i]).astype(prec)
            s_hi = (s_hi + t[..., 16 + i]).astype(prec)
        ss = (s_lo + s_hi).astype(prec)
        sigma = np.sqrt((ss / prec(32)).astype(prec)).astype(prec)
        sbits = round_to_bf16_bits((prec(STEP) * sigma).astype(prec))
    sbits = np.where(sbits < 0x80, 0, sbits).astype(np.uint16)      # below BF16's normal range: an empty group
    scale = O.bf16_bits_to_f64(sbits).astype(prec)
    with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
        rcp = (prec(1) / scale).astype(prec)
        v = (Gr * rcp[..., None]).astype(prec)
        q = np.clip(np.rint(v), QMIN, QMAX)
    q = np.where(scale[..., None] == 0, 0, q).astype(np.int8)
    return q.reshape(*lead, K), sbits.reshape(*lead, K // G)


def dequantize_int4(q: np.ndarray, sbits: np.ndarray) -> np.ndarray:
    """FP64 values of stored INT4 data."""
    *lead, K = q.shape
    s = O.bf16_bits_to_f64(sbits)
    return (np.asarray(q, dtype=np.float64).reshape(*lead, K // G, G) * s[..., None]).reshape(*lead, K)


def pack_codes(q: np.ndarray) -> np.ndarray:
    """Two's-complement nibbles, two per byte, element 2i in the low nibble."""
    n = (np.asarray(q, dtype=np.int16) & 0xF).astype(np.uint8)
    return (n[..., 0::2] | (n[..., 1::2] << 4)).astype(np.uint8)


def unpack_codes(packed: np.ndarray) -> np.ndarray:
    p = np.asarray(packed, dtype=np.uint8)
    n = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.int16)
    n[..., 0::2] = p & 0xF
    n[..., 1::2] = p >> 4
    return np.where(n >= 8, n - 16, n).astype(np.int8)


def linear_dequant(Xq, Xs, Wq, Ws) -> np.ndarray:
    """deq(X) . deq(W)^T in FP64."""
    return dequantize_int4(Xq, Xs) @ dequantize_int4(Wq, Ws).T


def layer_forward(X, W, T):
    """Quantized forward with INT4 on both operands; X, W on the BF16 grid, T
    16-bit values [K/32][32][32] (activations decided in FP32, weights in FP64)."""
    Xq, Xs = quantize_int4(O.transform_act(X, T).astype(np.float32), prec=np.float32)
    Wq, Ws = quantize_int4(O.transform_weight(W, T), prec=np.float64)
    return linear_dequant(Xq, Xs, Wq, Ws)
