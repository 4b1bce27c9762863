"""CPU oracle for the W4A4 WUSH layer forward -- TEST INFRASTRUCTURE ONLY.

A plain, slow, FP64 numpy implementation of what the GPU path computes, written
from the paper (Methodology: problem setup, block-independent constraint,
Eq. for W'/X', the SVD equation, the WUSH construction equation, Alg. 1,
Alg. 2 RTN case, the layer forward-pass equation).  It shares no code with the
HIP library and is imported only by tests, the smoke check and the benchmark's
CPU-baseline leg.  The product never routes through it.

Conventions (ours <-> paper).  The paper works with column data,
X in R^{d_in x d_batch}, W in R^{d_in x d_out}.  Here tensors are row-major with
the channel axis last: X [M][K] (M tokens), W [N][K] (N output channels).
Block b owns channels 32b..32b+31.  T[b] is the paper's T_wush for block b:
T[b][j][k] maps input channel k to transformed channel j, so

    Yt[m, 32b+j] = sum_k X[m, 32b+k] * T[b][j][k]              (T_wush X)
    Wt[n, 32b+j] = sum_k W[n, 32b+k] * inv(T[b])[k][j]         (T_wush^{-T} W)
    Y[m, n]      = sum_kappa deq(q(Yt))[m,kappa] * deq(q(Wt))[n,kappa]

Quantizer q: the paper fixes only "RTN with AbsMax scales on each group of d
values" and MXFP4 with d = 32.  The bit-level reading used here:
  * element grid E2M1: codes 0..7 -> 0, 0.5, 1, 1.5, 2, 3, 4, 6; bit 3 = sign;
  * scale E8M0: byte s -> 2^(s-127), s in 0..254;
  * scale rule "nosat" (default): the smallest power of two 2^e with
    AbsMax <= 6*2^e, i.e. no element is clipped (the FP error model in the
    appendix assumes |x/s| <= max representable);
    rule "ocp_floor": e = floor(log2 AbsMax) - 2 (the OCP MX recipe; group
    maxima in (6,8)*2^e saturate to 6);
  * round to nearest grid point, ties to the even code, saturate above 6;
  * the sign bit of the input is kept even when the magnitude rounds to 0.

Pins: see tests/test_oracle_*.py.  One item stays "parity unpinned": the
paper publishes no bit patterns of its own MXFP4 quantizer, so agreement with
the authors' implementation on tie and scale rules cannot be checked.
"""
from __future__ import annotations

import numpy as np

D = 32  # block size d = MXFP4 group size

E2M1_VALUES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
_E2M1_MIDPOINTS = (E2M1_VALUES[1:] + E2M1_VALUES[:-1]) / 2.0


# --------------------------------------------------------------------------
# BF16 grid
# --------------------------------------------------------------------------
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """FP64 values rounded to the BF16 grid (8-bit significand, RNE)."""
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)                       # |x| = m * 2^e, m in [0.5, 1)
    q_exp = np.maximum(e - 8, -133)          # quantum 2^(e-8); BF16 subnormal floor
    return np.ldexp(np.rint(np.ldexp(x, -q_exp)), q_exp)


def bf16_values_to_bits(x: np.ndarray) -> np.ndarray:
    """Bit patterns (uint16) of values that already lie on the BF16 grid."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# WUSH construction (Alg. 1, the WUSH construction equation)
# --------------------------------------------------------------------------
def hadamard(d: int = D) -> np.ndarray:
    """Normalized Sylvester Hadamard matrix, entries +-d^(-1/2)."""
    i = np.arange(d)
    bits = i[:, None] & i[None, :]
    parity = np.zeros((d, d), dtype=np.int64)
    while bits.any():
        parity ^= bits & 1
        bits = bits >> 1
    return (1.0 - 2.0 * parity) / np.sqrt(d)


def second_moment(A: np.ndarray) -> np.ndarray:
    """A holds one sample per row ([n][d]); returns n^-1 A^T A (d x d)."""
    A = np.asarray(A, dtype=np.float64)
    return A.T @ A / A.shape[0]


def damped(Mom: np.ndarray, lam: float) -> np.ndarray:
    d = Mom.shape[0]
    return Mom + lam * np.trace(Mom) / d * np.eye(d)


def wush_factors(M_W: np.ndarray, M_X: np.ndarray, lam: float):
    """Damped Cholesky factors and the SVD of W'^T X' (Alg. 1).

    Returns (Wp, Xp, U, s, V) with Wp Wp^T = damped M_W, Xp Xp^T = damped M_X,
    Wp^T Xp = U diag(s) V^T, s descending.  Sign convention: the entry of
    largest magnitude in each column of U is positive.
    """
    Wp = np.linalg.cholesky(damped(M_W, lam))
    Xp = np.linalg.cholesky(damped(M_X, lam))
    U, s, Vt = np.linalg.svd(Wp.T @ Xp)
    V = Vt.T
    pick = np.argmax(np.abs(U), axis=0)
    sign = np.sign(U[pick, np.arange(U.shape[1])])
    sign[sign == 0] = 1.0
    return Wp, Xp, U * sign[None, :], s, V * sign[None, :]


def wush_block(M_W: np.ndarray, M_X: np.ndarray, lam: float) -> np.ndarray:
    """T_wush = H S^(-1/2) U^T W'^T  (activation-side transform)."""
    Wp, _, U, s, _ = wush_factors(M_W, M_X, lam)
    return hadamard(M_W.shape[0]) @ np.diag(s ** -0.5) @ U.T @ Wp.T


def xvsh_block(M_W: np.ndarray, M_X: np.ndarray, lam: float) -> np.ndarray:
    """T_xvsh = H S^(-1/2) V^T X'^T  (weight-side transform)."""
    _, Xp, _, s, V = wush_factors(M_W, M_X, lam)
    return hadamard(M_W.shape[0]) @ np.diag(s ** -0.5) @ V.T @ Xp.T


def build_transforms(W: np.ndarray, X_cal: np.ndarray, lam: float = 1e-2) -> np.ndarray:
    """Alg. 2 (RTN case), transform part: per block, second moments of the
    original weight block and of the calibration activations, then Alg. 1.

    W [N][K], X_cal [M_cal][K] (FP64).  Returns T [K/32][32][32] in FP64,
    not yet rounded to 16 bits.
    """
    K = W.shape[1]
    assert K % D == 0 and X_cal.shape[1] == K
    T = np.empty((K // D, D, D))
    for b in range(K // D):
        sl = slice(D * b, D * b + D)
        T[b] = wush_block(second_moment(W[:, sl]), second_moment(X_cal[:, sl]), lam)
    return T


def hadamard_transforms(C: int) -> np.ndarray:
    """The data-free baseline: every block equal to the normalized H_32."""
    return np.broadcast_to(hadamard(D), (C, D, D)).copy()


# --------------------------------------------------------------------------
# Applying the transforms (layer forward-pass equation; Alg. 2 weight step)
# --------------------------------------------------------------------------
def transform_act(X: np.ndarray, T: np.ndarray) -> np.ndarray:
    M, K = X.shape
    Xb = np.asarray(X, dtype=np.float64).reshape(M, K // D, D)
    return np.einsum("mbk,bjk->mbj", Xb, T).reshape(M, K)


def transform_weight(W: np.ndarray, T: np.ndarray) -> np.ndarray:
    N, K = W.shape
    Tinv = np.linalg.inv(T)                  # per block, LU with partial pivoting
    Wb = np.asarray(W, dtype=np.float64).reshape(N, K // D, D)
    return np.einsum("nbk,bkj->nbj", Wb, Tinv).reshape(N, K)


# --------------------------------------------------------------------------
# MXFP4 quantizer (RTN, AbsMax scale per group of 32 along the last axis)
# --------------------------------------------------------------------------
def scale_bytes(absmax: np.ndarray, rule: str = "nosat") -> np.ndarray:
    """E8M0 byte for each group AbsMax (real-valued rule, no bit tricks)."""
    a = np.asarray(absmax, dtype=np.float64)
    m, e = np.frexp(a)                       # a = m 2^e, m in [0.5,1)
    mant = 2.0 * m                           # a = mant 2^p, mant in [1,2)
    p = e - 1
    if rule == "nosat":
        # smallest E with a <= 6 * 2^E = 1.5 * 2^(E+2)
        E = np.where(mant <= 1.5, p - 2, p - 1)
    elif rule == "ocp_floor":
        E = p - 2                            # floor(log2 a) - emax(E2M1)
    else:
        raise ValueError(rule)
    byte = np.clip(E + 127, 0, 254)
    byte = np.where(a == 0.0, 0, byte)
    return byte.astype(np.uint8)


def round_e2m1(v: np.ndarray) -> np.ndarray:
    """Magnitude code 0..7 of the grid point nearest to |v|; ties go to the
    even code; anything above 6 saturates to code 7."""
    a = np.abs(np.asarray(v, dtype=np.float64))
    lo = np.searchsorted(_E2M1_MIDPOINTS, a, side="left")    # midpoints strictly below
    hi = np.searchsorted(_E2M1_MIDPOINTS, a, side="right")   # midpoints at or below
    # lo != hi only exactly on a midpoint between codes lo and lo+1
    code = np.where(lo == hi, lo, np.where(lo % 2 == 0, lo, hi))
    return code.astype(np.uint8)


def quantize_mxfp4(Y: np.ndarray, rule: str = "nosat"):
    """Returns (codes, scales): codes uint8 [..., K] holding 4-bit patterns
    (bit 3 sign, bits 2..0 magnitude code), scales uint8 [..., K/32]."""
    Y = np.asarray(Y, dtype=np.float64)
    *lead, K = Y.shape
    G = Y.reshape(*lead, K // D, D)
    s = scale_bytes(np.max(np.abs(G), axis=-1), rule)
    v = np.ldexp(G, (127 - s.astype(np.int64))[..., None])   # exact power-of-two scaling
    code = round_e2m1(v) | (np.signbit(G).astype(np.uint8) << 3)
    return code.reshape(*lead, K), s


def pack_codes(codes: np.ndarray) -> np.ndarray:
    """Two codes per byte, element 2i in the low nibble, 2i+1 in the high."""
    c = np.asarray(codes, dtype=np.uint8)
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def unpack_codes(packed: np.ndarray) -> np.ndarray:
    p = np.asarray(packed, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = p & 0xF
    out[..., 1::2] = p >> 4
    return out


def dequantize(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    c = np.asarray(codes, dtype=np.uint8)
    mag = E2M1_VALUES[c & 7]
    val = np.where((c & 8) != 0, -mag, mag)
    *lead, K = c.shape
    e = scales.astype(np.int64) - 127
    return np.ldexp(val.reshape(*lead, K // D, D), e[..., None]).reshape(*lead, K)


# --------------------------------------------------------------------------
# Layer forward and metrics
# --------------------------------------------------------------------------
def linear_dequant(Xc, Xs, Wc, Ws) -> np.ndarray:
    """deq(Xq) . deq(Wq)^T in FP64 (the sum over blocks of the forward-pass
    equation, written as one product over all K)."""
    return dequantize(Xc, Xs) @ dequantize(Wc, Ws).T


def layer_forward(X, W, T, rule: str = "nosat"):
    """Full quantized forward for BF16-grid inputs X, W and 16-bit T."""
    Xc, Xs = quantize_mxfp4(transform_act(X, T), rule)
    Wc, Ws = quantize_mxfp4(transform_weight(W, T), rule)
    return linear_dequant(Xc, Xs, Wc, Ws)


def layer_loss(Y_hat: np.ndarray, Y_ref: np.ndarray) -> float:
    """Output loss of the problem setup: squared error averaged over the
    d_out * d_batch output entries."""
    return float(np.sum((Y_hat - Y_ref) ** 2) / Y_ref.size)


def rel_fro(A: np.ndarray, B: np.ndarray) -> float:
    return float(np.linalg.norm(A - B) / np.linalg.norm(B))


def fp_model_objective(T_X: np.ndarray, Wp: np.ndarray, Xp: np.ndarray) -> float:
    """Trace term of the FP error model for an activation-side transform T_X:
    sum_k ||W'^T T_X^{-1} e_k||^2 * (T_X X' X'^T T_X^T)_kk."""
    Tinv = np.linalg.inv(T_X)
    left = np.sum((Wp.T @ Tinv) ** 2, axis=0)
    right = np.diag(T_X @ Xp @ Xp.T @ T_X.T)
    return float(np.sum(left * right))
