"""Kernel arithmetic models of the NVFP4 and INT4 quantizers -- test helpers, NOT oracles.

The GPU quantizers take every decision step as one IEEE operation in one working
precision (FP32 on the accumulators of the activation kernels, FP64 in the offline
weight kernels) and put a reciprocal and a multiplication where the definition
divides.  The functions here replay exactly those steps in numpy so that a test
can demand bit-for-bit agreement from the GPU ("the kernel does what it says"),
while the definition itself -- oracle/wush_nvfp4_oracle.py, oracle/wush_int4_oracle.py,
plain FP64 with true divisions -- is what the results are judged against:
tests/test_kernel_models.py bounds model against definition on the CPU (differences
only next to a rounding boundary), the GPU tests do the same for the kernels.
"""
from __future__ import annotations

import numpy as np

from oracle import wush_int4_oracle as Q4
from oracle import wush_nvfp4_oracle as NV
from oracle import wush_oracle as O


def int4_steps(Y: np.ndarray, prec=np.float32):
    """The INT4 kernels' steps in `prec`: t_i = v_i v_i; channels 0..15 summed left to
    right, 16..31 likewise (a lane holds 16 channels of a group), the two sums added;
    sigma = sqrt(ss / 32); scale = BF16(STEP sigma); rcp = 1 / scale;
    q = clip(rint(v rcp), -8, 7).  No fused multiply-add anywhere."""
    Y = np.asarray(Y, dtype=prec)
    *lead, K = Y.shape
    Gr = Y.reshape(-1, K // 32, 32)
    with np.errstate(over="ignore"):
        t = (Gr * Gr).astype(prec)
        s_lo = np.zeros(t.shape[:2], dtype=prec)
        s_hi = np.zeros(t.shape[:2], dtype=prec)
        for i in range(16):
            s_lo = (s_lo + t[..., i]).astype(prec)
            s_hi = (s_hi + t[..., 16 + i]).astype(prec)
        ss = (s_lo + s_hi).astype(prec)
        sigma = np.sqrt((ss / prec(32)).astype(prec)).astype(prec)
        sbits = Q4.round_to_bf16_bits((prec(Q4.STEP) * sigma).astype(prec))
    sbits = np.where(sbits < 0x80, 0, sbits).astype(np.uint16)
    scale = O.bf16_bits_to_f64(sbits).astype(prec)
    with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
        rcp = (prec(1) / scale).astype(prec)
        v = (Gr * rcp[..., None]).astype(prec)
        q = np.clip(np.rint(v), Q4.QMIN, Q4.QMAX)
    q = np.where(scale[..., None] == 0, 0, q).astype(np.int8)
    return q.reshape(*lead, K), sbits.reshape(*lead, K // 32)


def nvfp4_steps(Y: np.ndarray, ts, prec=np.float32):
    """The NVFP4 kernels' steps in `prec`: c = 1 / (6 ts); r = amax c; byte = E4M3(r);
    d = value(byte) ts; rcp = 1 / d; code = E2M1(v rcp)."""
    Y = np.asarray(Y, dtype=prec)
    ts = prec(ts)
    *lead, K = Y.shape
    Gr = Y.reshape(*lead, K // 16, 16)
    with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
        amax = np.max(np.abs(Gr), axis=-1)
        c = prec(0) if ts == 0 else prec(1) / (prec(6) * ts)
        r = (amax * c).astype(prec)
        sb = NV.round_e4m3(r)
        d = (NV.e4m3_value(sb).astype(prec) * ts).astype(prec)
        rcp = np.where(sb == 0, prec(0), prec(1) / d).astype(prec)
        v = (Gr * rcp[..., None]).astype(prec)
    code = NV.round_e2m1(v) | (np.signbit(Gr).astype(np.uint8) << 3)
    return code.reshape(*lead, K), sb


# --------------------------------------------------------------------------
# "Explained mismatch" rules: which differences between a decision taken in
# lower precision and the FP64 definition are legitimate.
# --------------------------------------------------------------------------
def int4_explained(vals64, q_a, s_a, q_ref, s_ref, tol):
    """(mismatch rate, number of differing elements that sit neither within tol (relative to
    the group's largest |v / scale|) of a rounding midpoint nor in a group whose STEP * sigma
    is within tol of a BF16 rounding boundary).  vals64: the exact values both sides quantized;
    q_*: int8 codes; s_*: BF16 scale bits."""
    R, K = vals64.shape
    Gr = vals64.reshape(R, K // 32, 32)
    qg, qr = q_a.reshape(R, K // 32, 32), q_ref.reshape(R, K // 32, 32)
    sdiff = s_a != s_ref
    bad = (qg != qr) | sdiff[..., None]
    if not bad.any():
        return 0.0, 0
    s_real = Q4.STEP * np.sqrt(np.mean(Gr * Gr, axis=-1))
    sref = O.bf16_bits_to_f64(s_ref)
    lo = np.minimum(O.bf16_bits_to_f64(s_a), sref)
    hi = np.maximum(O.bf16_bits_to_f64(s_a), sref)
    near_scale = sdiff & (np.abs(s_real - 0.5 * (lo + hi)) <= tol * s_real)
    with np.errstate(divide="ignore", invalid="ignore"):
        v = Gr / sref[..., None]
    frac = np.abs(v - np.floor(v) - 0.5)
    near_mid = frac <= tol * np.maximum(np.max(np.abs(v), axis=-1, keepdims=True), 1.0)
    unexplained = bad & ~near_mid & ~near_scale[..., None]
    return float(np.mean(bad)), int(unexplained.sum())


def nvfp4_explained(vals64, ts, codes_gpu, sb_gpu, codes_ref, sb_ref, tol):
    """Counts differing elements that do NOT sit within tol (relative to the group
    AbsMax) of an E2M1 midpoint and whose group is NOT within tol of an E4M3 midpoint."""
    R, K = vals64.shape
    Gr = vals64.reshape(R, K // 16, 16)
    amax = np.max(np.abs(Gr), axis=-1)
    cg, cr = codes_gpu.reshape(R, K // 16, 16), codes_ref.reshape(R, K // 16, 16)
    same = (cg == cr) | (((cg & 7) == 0) & ((cr & 7) == 0))
    bad = ~same | (sb_gpu != sb_ref)[..., None]
    if not bad.any():
        return 0.0, 0
    r = amax / (6.0 * float(ts))
    grid = NV.e4m3_value(np.arange(127))
    mids = (grid[1:] + grid[:-1]) / 2
    near_scale = np.min(np.abs(r[..., None] - mids), axis=-1) <= tol * np.maximum(r, 2.0 ** -9)
    d = NV.e4m3_value(sb_ref) * float(ts)
    with np.errstate(divide="ignore", invalid="ignore"):
        v = np.abs(Gr) / d[..., None]
        a = amax / d
    emid = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
    near_mid = np.min(np.abs(v[..., None] - emid), axis=-1) <= tol * a[..., None]
    unexplained = bad & ~near_mid & ~near_scale[..., None]
    return float(np.mean(bad)), int(unexplained.sum())
