"""CPU oracle for the GPTQ case of Alg. 2 -- TEST INFRASTRUCTURE ONLY.

Plain FP64 numpy, written from the paper's Alg. 2 (GPTQ case) and the paragraph
"GPTQ integration": WUSH transforms interleaved with GPTQ's intra-block and
inter-block error propagation, producing the per-block transforms and the
pre-quantized transformed weights of a layer.  It takes the algorithm's steps in
the paper's order and notation (full Hessian, damping, inverse, Cholesky factor
L of the inverse, its d x d blocks, the transformed block Hessian, the GPTQ
subroutine, the error in the original space, the propagation through
L_(j,i) L_(i,i)^-1), with library routines for inverse / Cholesky.  It shares no
code with the HIP library and is imported only by tests.

Conventions: as in wush_oracle.py (row-major, channels last; X_cal [M][K],
W [N][K]; T[b][j][k]).  The paper's W_(i) (d x d_out) is the transpose of
W[:, block i] here.

Readings of what the paper leaves open (all listed in the design notes):
  * T_(i) is rounded to 16 bits (BF16) right after Alg. 1; that rounded matrix
    is the transform for everything that follows in the iteration (weight side,
    transformed Hessian, error in the original space), exactly as in the RTN
    case, because it is what the online kernel applies.
  * "standard GPTQ subroutine" on a transformed block: the d transformed
    channels are processed in index order; for channel r the values of all
    output channels are quantized, the error divided by R[r][r] and propagated to
    channels r' > r with R[r][r'], where R is the upper Cholesky factor of the
    inverse of the transformed Hessian (R^T R = inv(Hbar)).
  * MXFP4 group = the d transformed channels of one output channel = exactly the
    block.  Its E8M0 scale is taken once, from the AbsMax of the transformed
    weights before any intra-block update ("static" scale, as GPTQ implementations
    do for group scales); values pushed past the grid by later updates saturate.
  * The error in the original space uses the dequantized codes.
  * The update of block j = i itself (the loop starts at j = i) is dropped:
    block i is not read again.

Pins: tests/test_oracle_gptq.py.
"""
from __future__ import annotations

import numpy as np

from . import wush_oracle as O

D = O.D


def hessian(X_cal: np.ndarray) -> np.ndarray:
    """GPTQ's Hessian d_batch^-1 X X^T (K x K)."""
    X = np.asarray(X_cal, dtype=np.float64)
    return X.T @ X / X.shape[0]


def inverse_cholesky(H: np.ndarray, lam: float) -> np.ndarray:
    """Lower-triangular L with L L^T = inv(H + lam * tr(H)/d_in * I)."""
    K = H.shape[0]
    Hd = H + lam * np.trace(H) / K * np.eye(K)
    return np.linalg.cholesky(np.linalg.inv(Hd))


def quantize_static(v: np.ndarray, scale_byte: np.ndarray):
    """RTN to E2M1 at a given E8M0 scale (saturating).  Returns (codes, values)."""
    scaled = np.ldexp(v, 127 - scale_byte.astype(np.int64))
    code = O.round_e2m1(scaled) | (np.signbit(v).astype(np.uint8) << 3)
    grid = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
    val = np.where(code & 8, -1.0, 1.0) * np.ldexp(grid[code & 7], scale_byte.astype(np.int64) - 127)
    return code, val


def gptq_block(Wbar: np.ndarray, Hbar: np.ndarray, rule: str = "nosat"):
    """The GPTQ subroutine on one transformed block.

    Wbar [N][d]: transformed weights (one MXFP4 group per row); Hbar [d][d]: the
    transformed Hessian.  Returns (codes [N][d], scale bytes [N], dequantized
    values [N][d]).
    """
    Wbar = np.array(Wbar, dtype=np.float64)
    d = Wbar.shape[1]
    R = np.linalg.cholesky(np.linalg.inv(Hbar)).T            # upper, R^T R = inv(Hbar)
    sb = O.scale_bytes(np.max(np.abs(Wbar), axis=1), rule)   # static group scale
    codes = np.zeros(Wbar.shape, dtype=np.uint8)
    deq = np.zeros(Wbar.shape)
    for r in range(d):
        codes[:, r], deq[:, r] = quantize_static(Wbar[:, r], sb)
        err = (Wbar[:, r] - deq[:, r]) / R[r, r]
        Wbar[:, r + 1:] -= np.outer(err, R[r, r + 1:])
    return codes, sb, deq


def gptq_wush_layer(W: np.ndarray, X_cal: np.ndarray, lam: float = 1e-2, rule: str = "nosat",
                    transform: str = "wush"):
    """Alg. 2, GPTQ case.  W [N][K], X_cal [M][K] (FP64 values).

    transform: "wush" (the algorithm), or "hadamard" / "identity" (the same
    schedule with a fixed transform; used by pins and comparisons).
    Returns (T [C][d][d] BF16-valued FP64, codes [N][K], scale bytes [N][C]).
    """
    W = np.array(W, dtype=np.float64)
    N, K = W.shape
    C = K // D
    Hs = hessian(X_cal)
    L = inverse_cholesky(Hs, lam)
    T = np.empty((C, D, D))
    codes = np.empty((N, K), dtype=np.uint8)
    scales = np.empty((N, C), dtype=np.uint8)
    for i in range(C):
        bi = slice(D * i, D * i + D)
        if transform == "wush":
            M_W = O.second_moment(W[:, bi])                  # updated weight block
            M_X = Hs[bi, bi]                                 # diagonal block of the Hessian
            Ti = O.round_to_bf16(O.wush_block(M_W, M_X, lam))
        elif transform == "hadamard":
            Ti = O.round_to_bf16(O.hadamard(D))
        else:
            Ti = np.eye(D)
        T[i] = Ti
        Tinv = np.linalg.inv(Ti)
        Wbar = W[:, bi] @ Tinv                               # (T_xvsh W_(i))^T
        Lii = L[bi, bi]
        Hbar = Ti @ np.linalg.inv(Lii @ Lii.T) @ Ti.T        # transformed Hessian
        codes[:, bi], scales[:, i], deq = gptq_block(Wbar, Hbar, rule)
        E = deq @ Ti - W[:, bi]                              # (T_xvsh^-1 Wtilde - W_(i))^T
        if i + 1 < C:
            rest = slice(D * (i + 1), K)
            P = L[rest, bi] @ np.linalg.inv(Lii)             # L_(j,i) L_(i,i)^-1, stacked over j > i
            W[:, rest] += E @ P.T
    return T, codes, scales


def proxy_loss(T, codes, scales, W, X) -> float:
    """Output error of the pre-quantized weights under UNquantized activations,
    ||X W^T - (X T^T)(deq)^T||_F^2 / (M N): the objective GPTQ's propagation targets."""
    Wt = O.dequantize(codes, scales)
    Yt = O.transform_act(X, T)
    return float(np.mean((X @ W.T - Yt @ Wt.T) ** 2))
