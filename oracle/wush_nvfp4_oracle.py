"""CPU oracle for the NVFP4 variant of the quantized layer -- TEST INFRASTRUCTURE ONLY.

The paper's experiments ("Layerwise Quantization Loss", Table 1 and the accuracy
tables) run the same method with the NVFP4 format: E2M1 elements in groups of
16, and -- "the transform block size is matched to the quantization group size" --
16 x 16 transform blocks.  This module writes that variant out in plain numpy:
block transforms of size d = 16, the NVFP4 quantizer, its inverse, and the layer
forward.  It shares no code with the HIP library and is imported only by tests
and the benchmark's CPU-baseline leg.

Format (the public NVFP4 definition, which the paper follows without restating
it): element = E2M1 (as in MXFP4); one FP8 E4M3 scale per group of 16 consecutive
channels; one FP32 scale per tensor.  A stored element is worth
    E2M1(code) * E4M3(scale byte) * tensor_scale.
E4M3 here is the "finite, no infinities" FP8: bias 7, 3 fraction bits, subnormals
m/8 * 2^-6, largest finite value 448 (byte 0x7E); scales are non-negative.

Readings of what the paper leaves open (listed in the design notes as well):
  * tensor scale: AbsMax of the whole (transformed) tensor / (6 * 448), so that
    the largest group scale lands on the largest E4M3 value.  For activations it
    is an INPUT of the quantizer (a calibrated or separately reduced constant).
  * group scale: AbsMax of the group / (6 * tensor_scale), rounded to the nearest
    E4M3 value (ties to the even byte), saturating at 448.  Rounding down can push
    the group maximum past 6; it then saturates (round-to-nearest as in the
    MXFP4 case, no stochastic part).
  * elements: value / (group scale * tensor scale), rounded to the nearest E2M1
    value, ties to even, saturating; the sign bit of the input is kept even when
    the magnitude rounds to zero.
  * edge cases (each its own reading): a group whose scale byte is 0 (its AbsMax
    is below half the smallest E4M3 value times 6 ts) has all magnitudes 0 -- the
    value / 0 of the definition has no nearest grid point, and 0 is what the
    stored data can represent; a tensor scale of 0 (an all-zero tensor) gives
    scale bytes 0 and magnitudes 0 for the same reason.
  * arithmetic: FP64 throughout, the formulas as written, with true divisions:
        r = amax / (6 ts)    byte = E4M3(r)    code = E2M1(v / (value(byte) ts)).
    The GPU decides in FP32 (activations) with reciprocals; a model of those
    steps lives with the tests (tests/kernel_models.py), not here.

Conventions: row-major, channels last; X [M][K], W [N][K]; T[b][j][k] with
b = 0 .. K/16-1; codes hold 4-bit patterns (bit 3 sign, bits 2..0 magnitude).
Pins: tests/test_oracle_nvfp4.py.
"""
from __future__ import annotations

import numpy as np

G = 16                    # NVFP4 group = transform block of this variant
E2M1_VALUES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
_E2M1_MID = (E2M1_VALUES[1:] + E2M1_VALUES[:-1]) / 2.0
E4M3_MAX = 448.0


def e4m3_value(byte: np.ndarray) -> np.ndarray:
    """Value of a non-negative E4M3 byte 0..126 (FP64, exact)."""
    b = np.asarray(byte, dtype=np.int64)
    e, m = b >> 3, b & 7
    return np.where(e == 0, np.ldexp(m / 8.0, -6), np.ldexp(1.0 + m / 8.0, e - 7))


_E4M3_GRID = e4m3_value(np.arange(127))
_E4M3_MID = (_E4M3_GRID[1:] + _E4M3_GRID[:-1]) / 2.0     # exact in FP64


def _nearest_even(mid: np.ndarray, a: np.ndarray) -> np.ndarray:
    """Index of the grid point nearest to a >= 0, ties to the even index,
    saturating at the last index; `mid` = midpoints between neighbours."""
    lo = np.searchsorted(mid, a, side="left")
    hi = np.searchsorted(mid, a, side="right")
    return np.where(lo == hi, lo, np.where(lo % 2 == 0, lo, hi))


def round_e4m3(r: np.ndarray) -> np.ndarray:
    """Byte of the E4M3 value nearest to r >= 0 (ties to even, saturating at 448)."""
    return _nearest_even(_E4M3_MID, np.asarray(r, dtype=np.float64)).astype(np.uint8)


def round_e2m1(v: np.ndarray) -> np.ndarray:
    """Magnitude code 0..7 nearest to |v| (ties to even, saturating at 6)."""
    return _nearest_even(_E2M1_MID, np.abs(np.asarray(v, dtype=np.float64))).astype(np.uint8)


def tensor_scale(Y: np.ndarray) -> np.float32:
    """FP32 per-tensor scale: AbsMax / (6 * 448), computed in FP64, rounded once."""
    return np.float32(np.max(np.abs(np.asarray(Y, dtype=np.float64))) / (6.0 * E4M3_MAX))


def quantize_nvfp4(Y: np.ndarray, ts):
    """NVFP4 quantizer on values Y [..., K] with tensor scale ts, FP64.
    Returns (codes uint8 [..., K], scale bytes uint8 [..., K/16])."""
    Y = np.asarray(Y, dtype=np.float64)
    ts = float(ts)
    *lead, K = Y.shape
    Gr = Y.reshape(*lead, K // G, G)
    amax = np.max(np.abs(Gr), axis=-1)
    if ts == 0.0:                                       # an all-zero tensor
        sb = np.zeros(amax.shape, dtype=np.uint8)
    else:
        sb = round_e4m3(amax / (6.0 * ts))
    d = e4m3_value(sb) * ts
    with np.errstate(divide="ignore", invalid="ignore"):
        v = np.where(d[..., None] == 0, 0.0, Gr / d[..., None])
    code = round_e2m1(v) | (np.signbit(Gr).astype(np.uint8) << 3)
    return code.reshape(*lead, K), sb


def dequantize_nvfp4(codes: np.ndarray, sbytes: np.ndarray, ts) -> np.ndarray:
    """FP64 values of stored NVFP4 data."""
    c = np.asarray(codes, dtype=np.uint8)
    mag = E2M1_VALUES[c & 7]
    val = np.where((c & 8) != 0, -mag, mag)
    *lead, K = c.shape
    s = e4m3_value(sbytes) * float(ts)
    return (val.reshape(*lead, K // G, G) * s[..., None]).reshape(*lead, K)


# --------------------------------------------------------------------------
# Block transforms of size 16 and the layer forward (forward-pass equation with
# d = 16; Alg. 2, RTN case, for the weight side)
# --------------------------------------------------------------------------
def transform_act(X: np.ndarray, T: np.ndarray) -> np.ndarray:
    """Yt[m, d b + j] = sum_k X[m, d b + k] T[b][j][k], d = T.shape[-1]."""
    M, K = X.shape
    d = T.shape[-1]
    Xb = np.asarray(X, dtype=np.float64).reshape(M, K // d, d)
    return np.einsum("mbk,bjk->mbj", Xb, T).reshape(M, K)


def transform_weight(W: np.ndarray, T: np.ndarray) -> np.ndarray:
    """Wt[n, d b + j] = sum_k W[n, d b + k] inv(T[b])[k][j]."""
    N, K = W.shape
    d = T.shape[-1]
    Wb = np.asarray(W, dtype=np.float64).reshape(N, K // d, d)
    return np.einsum("nbk,bkj->nbj", Wb, np.linalg.inv(T)).reshape(N, K)


def prepare_weight(W: np.ndarray, T: np.ndarray):
    """Offline weight side: transformed weights, their tensor scale (FP32) and
    their NVFP4 codes / scale bytes."""
    Wt = transform_weight(W, T)
    ts = tensor_scale(Wt)
    codes, sb = quantize_nvfp4(Wt, ts)
    return codes, sb, ts


def linear_dequant(Xc, Xs, tsx, Wc, Ws, tsw) -> np.ndarray:
    """deq(X) . deq(W)^T in FP64."""
    return dequantize_nvfp4(Xc, Xs, tsx) @ dequantize_nvfp4(Wc, Ws, tsw).T


def layer_forward(X, W, T, tsx=None):
    """Quantized forward with NVFP4 on both operands; X, W on the BF16 grid,
    T 16-bit values [K/16][16][16].  tsx defaults to the tensor scale of T X."""
    Yt = transform_act(X, T)
    if tsx is None:
        tsx = tensor_scale(Yt)
    Xc, Xs = quantize_nvfp4(Yt, tsx)
    Wc, Ws, tsw = prepare_weight(W, T)
    return linear_dequant(Xc, Xs, tsx, Wc, Ws, tsw)
