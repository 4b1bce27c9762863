"""Helpers for the GPU parity tests (device buffers, comparison rules)."""
from __future__ import annotations

import numpy as np

from oracle import wush_oracle as O

MIDPOINTS = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])


def torch_mod():
    import torch
    return torch


def bf16_dev(bits: np.ndarray):
    """uint16 BF16 bit patterns -> torch.bfloat16 tensor on the GPU."""
    torch = torch_mod()
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def u8_dev(a: np.ndarray):
    torch = torch_mod()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).cuda()


def empty_u8(*shape):
    torch = torch_mod()
    return torch.empty(shape, dtype=torch.uint8, device="cuda")


def host(t) -> np.ndarray:
    torch = torch_mod()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def code_mismatch_report(Yt64, codes_gpu, scales_gpu, codes_ref, scales_ref, tol=1e-5):
    """Compare GPU codes with the oracle's codes computed from exact FP64
    transformed values `Yt64`.

    Returns (mismatch_rate, unexplained): `unexplained` counts differing
    elements that are NOT within tol*AbsMax of a rounding midpoint and whose
    group AbsMax is NOT within tol (relative) of a scale threshold.  +-0 with
    the same magnitude code count as equal here.
    """
    M, K = Yt64.shape
    G = Yt64.reshape(M, K // 32, 32)
    amax = np.max(np.abs(G), axis=-1)
    cg = codes_gpu.reshape(M, K // 32, 32)
    cr = codes_ref.reshape(M, K // 32, 32)
    same = (cg == cr) | (((cg & 7) == 0) & ((cr & 7) == 0))
    scale_diff = scales_gpu != scales_ref
    bad = ~same | scale_diff[..., None]
    rate = float(np.mean(bad))
    if not bad.any():
        return 0.0, 0
    # group-level excuse: AbsMax within tol of a power-of-two threshold (6*2^e or 4*2^e family)
    with np.errstate(divide="ignore"):
        m, _ = np.frexp(amax)
    mant = 2 * m  # in [1,2)
    near_thresh = (np.abs(mant - 1.5) <= 1.5 * tol) | (np.abs(mant - 1.0) <= tol) | (np.abs(mant - 2.0) <= 2 * tol)
    # element-level excuse: scaled value within tol*AbsMax_scaled of a midpoint (under the reference scale)
    v = np.abs(G) / np.exp2(scales_ref.astype(np.float64) - 127)[..., None]
    a_scaled = amax / np.exp2(scales_ref.astype(np.float64) - 127)
    dist = np.min(np.abs(v[..., None] - MIDPOINTS), axis=-1)
    near_mid = dist <= tol * a_scaled[..., None]
    unexplained = bad & ~near_mid & ~near_thresh[..., None]
    return rate, int(unexplained.sum())


def oracle_quant_packed(Y, rule="nosat"):
    c, s = O.quantize_mxfp4(Y, rule)
    return O.pack_codes(c), s
