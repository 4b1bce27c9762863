"""Seeded synthetic inputs for the W4A4 layer-forward path.

This module holds the workload recipes only: shapes, value distributions and
the BF16 storage format of the tensors a layer receives.  It contains none of
the method's arithmetic (no transform construction, no quantizer, no GEMM), so
the CPU oracle, the tests and the benchmark can all draw the same inputs from
it without sharing anything else.

The distributions stand in for the statistics of LLM activations and weights
(per-channel scale spread, a few massive outlier channels, heavy tails); no
model weights or dataset samples are involved.

Every tensor is returned as BF16 bit patterns (numpy uint16, the top half of
the IEEE binary32 word, round-to-nearest-even).  `bf16_bits_to_f32` widens
them exactly.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

BLOCK = 32  # transform block size = quantization group size (MXFP4)


@dataclass(frozen=True)
class LayerConfig:
    name: str
    M: int                 # tokens in the evaluated batch
    K: int                 # input channels (d_in)
    N: int                 # output channels (d_out); 0 = activation path only
    calib_tokens: int      # tokens used for the second moments
    act_law: str           # "normal" | "student_t3"
    n_outlier: int         # number of outlier channels
    outlier_gain: float    # multiplier applied to outlier channels
    seed: int

    @property
    def C(self) -> int:
        return self.K // BLOCK


# One seed per configuration: 95600 + index.
CONFIGS = {
    "c1": LayerConfig("c1", 16, 256, 256, 512, "normal", 2, 50.0, 95601),
    "c2": LayerConfig("c2", 2048, 4096, 6144, 4096, "normal", 20, 50.0, 95602),
    "c3": LayerConfig("c3", 4096, 14336, 4096, 8192, "student_t3", 143, 100.0, 95603),
    "c4": LayerConfig("c4", 16384, 4096, 6144, 4096, "normal", 20, 50.0, 95604),
    "c5": LayerConfig("c5", 8192, 8192, 57344, 16384, "normal", 41, 50.0, 95605),
}


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of `cfg` with some sizes replaced (same seed, same laws)."""
    return replace(cfg, **kw)


# --------------------------------------------------------------------------
# BF16 storage helpers (format plumbing, not method arithmetic)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round binary32 values to BF16 (nearest, ties to even); return uint16."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen BF16 bit patterns to binary32 exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# Draws
# --------------------------------------------------------------------------
_ROW_CHUNK = 1024


def _draw_act(rng: np.random.Generator, rows: int, K: int, law: str,
              chan_scale: np.ndarray) -> np.ndarray:
    out = np.empty((rows, K), dtype=np.uint16)
    for r0 in range(0, rows, _ROW_CHUNK):
        r1 = min(rows, r0 + _ROW_CHUNK)
        if law == "normal":
            z = rng.standard_normal((r1 - r0, K), dtype=np.float32)
        elif law == "student_t3":
            z = rng.standard_t(3.0, size=(r1 - r0, K)).astype(np.float32)
        else:
            raise ValueError(f"unknown activation law {law!r}")
        z *= chan_scale[None, :]
        out[r0:r1] = f32_to_bf16_bits(z)
    return out


def _draw_weight(rng: np.random.Generator, N: int, K: int,
                 row_scale: np.ndarray) -> np.ndarray:
    out = np.empty((N, K), dtype=np.uint16)
    for r0 in range(0, N, _ROW_CHUNK):
        r1 = min(N, r0 + _ROW_CHUNK)
        z = rng.standard_normal((r1 - r0, K), dtype=np.float32)
        z *= np.float32(0.02)
        z *= row_scale[r0:r1, None]
        out[r0:r1] = f32_to_bf16_bits(z)
    return out


def make_layer(cfg: LayerConfig, *, want_weight: bool = True) -> dict:
    """Draw one layer's tensors.

    Draw order is fixed: channel scales, outlier channel indices, calibration
    activations, evaluation activations, weight row scales, weights.

    Returns a dict with BF16 bit patterns:
      X_cal [calib_tokens][K], X [M][K], W [N][K] (absent if N == 0 or
      want_weight is False), plus `chan_scale` (float32 [K]) and
      `outlier_idx` for reporting.
    """
    if cfg.K % BLOCK:
        raise ValueError("K must be a multiple of 32")
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    chan_scale = rng.lognormal(0.0, 1.0, size=cfg.K).astype(np.float32)
    outlier_idx = np.sort(rng.choice(cfg.K, size=cfg.n_outlier, replace=False))
    chan_scale[outlier_idx] *= np.float32(cfg.outlier_gain)
    out = {
        "cfg": cfg,
        "chan_scale": chan_scale,
        "outlier_idx": outlier_idx,
        "X_cal": _draw_act(rng, cfg.calib_tokens, cfg.K, cfg.act_law, chan_scale),
        "X": _draw_act(rng, cfg.M, cfg.K, cfg.act_law, chan_scale),
    }
    if cfg.N and want_weight:
        row_scale = rng.lognormal(0.0, 0.5, size=cfg.N).astype(np.float32)
        out["W"] = _draw_weight(rng, cfg.N, cfg.K, row_scale)
    return out


def make_transforms_random(C: int, seed: int, block: int = BLOCK) -> np.ndarray:
    """Well-conditioned random block x block transforms as BF16 bits, shape [C][block][block]
    (block = 32, or 16 for the NVFP4 variant).

    Timing of the path does not depend on the values of the transforms; the
    benchmark uses these when it only needs a tensor of the right shape whose
    blocks are all different and invertible.  Each block is a random orthogonal
    matrix (QR of a Gaussian) with its rows rescaled by log-normal factors.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    T = np.empty((C, block, block), dtype=np.float32)
    for b in range(C):
        q, _ = np.linalg.qr(rng.standard_normal((block, block)))
        s = rng.lognormal(0.0, 0.5, size=block)
        T[b] = (s[:, None] * q).astype(np.float32)
    return f32_to_bf16_bits(T)


def random_f32(shape, seed: int, spread: float = 4.0) -> np.ndarray:
    """Float32 test values spanning many binades: N(0,1) * 2^U(-spread, spread)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    z = rng.standard_normal(shape, dtype=np.float32)
    e = rng.uniform(-spread, spread, size=shape).astype(np.float32)
    return (z * np.exp2(e)).astype(np.float32)
