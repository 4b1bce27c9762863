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
  * elements: q = clip(round-half-even(v / scale), -8, 7).
  * edge cases (each its own reading): a scale whose BF16 rounding falls below
    BF16's normal range (an all-zero group, or one of FP32 denormals) is stored
    as 0 -- sub-normal BF16 numbers are flushed by the FP16/BF16 conversion
    hardware of every current GPU, so a stored sub-normal scale could not be
    used -- and a group whose scale is 0 has q = 0 everywhere (0 / 0 has no value).
  * arithmetic: FP64 throughout, the formulas as written: sigma =
    sqrt(sum(v^2) / 32) with numpy's sum, scale = BF16(STEP * sigma) (one
    rounding to nearest even from the FP64 product), a true division v / scale.
    The GPU decides in FP32 (activations) with a reciprocal; a model of those
    steps lives with the tests (tests/kernel_models.py), not here.

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


def quantize_int4(Y: np.ndarray):
    """INT4 quantizer on values Y [..., K], FP64.  Returns (q int8 [..., K] in -8..7,
    scale bits uint16 [..., K/32])."""
    Y = np.asarray(Y, dtype=np.float64)
    *lead, K = Y.shape
    Gr = Y.reshape(-1, K // G, G)
    sigma = np.sqrt(np.sum(Gr * Gr, axis=-1) / G)
    sbits = round_to_bf16_bits(STEP * sigma)
    sbits = np.where(sbits < 0x80, 0, sbits).astype(np.uint16)      # below BF16's normal range: stored as 0
    scale = O.bf16_bits_to_f64(sbits)
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.clip(np.rint(Gr / scale[..., None]), QMIN, QMAX)
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
    16-bit values [K/32][32][32]."""
    Xq, Xs = quantize_int4(O.transform_act(X, T))
    Wq, Ws = quantize_int4(O.transform_weight(W, T))
    return linear_dequant(Xq, Xs, Wq, Ws)
