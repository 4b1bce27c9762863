"""Pins for the oracle's WUSH construction (Alg. 1 and the closed form).

Each test checks the oracle against something the paper or linear algebra
fixes independently of the oracle's own formula: the inverse-transpose
identity, the equalization identity of the appendix, the FP-model optimum
(tr S)^2 / d and its lower-bound property, the trace sandwich, invariance to
the choice of moment factor, and two special cases with a textbook answer.
"""
import numpy as np
import pytest

from oracle import wush_oracle as O

D = 32


def _moments(seed, n_w=200, n_x=300, outlier=True):
    rng = np.random.default_rng(seed)
    sx = rng.lognormal(0, 1, D)
    if outlier:
        sx[rng.integers(D)] *= 50
    A = rng.standard_normal((D, D)) * 0.3 + np.eye(D)      # correlate channels
    X = (rng.standard_normal((n_x, D)) * sx) @ A
    W = rng.standard_normal((n_w, D)) * 0.02 * rng.lognormal(0, 0.5, (n_w, 1))
    return O.second_moment(W), O.second_moment(X)


def test_hadamard_is_normalized_and_orthogonal():
    H = O.hadamard(D)
    assert np.allclose(np.abs(H), 1 / np.sqrt(D), rtol=0, atol=1e-16)
    assert np.max(np.abs(H @ H.T - np.eye(D))) < 1e-14
    # Sylvester recursion H_2n = [[H, H], [H, -H]] / sqrt(2)
    H16 = O.hadamard(16)
    assert np.allclose(H, np.block([[H16, H16], [H16, -H16]]) / np.sqrt(2), atol=1e-15)


@pytest.mark.parametrize("lam", [0.0, 1e-4, 1e-2])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_xvsh_is_inverse_transpose_of_wush(seed, lam):
    M_W, M_X = _moments(seed)
    Tw = O.wush_block(M_W, M_X, lam)
    Tx = O.xvsh_block(M_W, M_X, lam)          # built from V and X', not from Tw
    assert np.max(np.abs(Tx @ Tw.T - np.eye(D))) < 1e-9


@pytest.mark.parametrize("seed", [3, 4])
def test_equalization_identity(seed):
    lam = 1e-3
    M_W, M_X = _moments(seed)
    Wp, Xp, U, s, V = O.wush_factors(M_W, M_X, lam)
    H = O.hadamard(D)
    Tw = O.wush_block(M_W, M_X, lam)
    Tx = O.xvsh_block(M_W, M_X, lam)
    target = H @ np.diag(s) @ H.T
    got_x = Tw @ O.damped(M_X, lam) @ Tw.T
    got_w = Tx @ O.damped(M_W, lam) @ Tx.T
    scale = np.max(np.abs(target))
    assert np.max(np.abs(got_x - target)) < 1e-9 * scale
    assert np.max(np.abs(got_w - target)) < 1e-9 * scale
    # constant diagonal tr(S)/d: per-channel RMS is equalized on both sides
    assert np.allclose(np.diag(got_x), s.sum() / D, rtol=1e-9)
    assert np.allclose(np.diag(got_w), s.sum() / D, rtol=1e-9)


@pytest.mark.parametrize("seed", [5, 6])
def test_fp_model_objective_attains_lower_bound(seed):
    lam = 1e-3
    M_W, M_X = _moments(seed)
    Wp, Xp, U, s, V = O.wush_factors(M_W, M_X, lam)
    Tw = O.wush_block(M_W, M_X, lam)
    opt = s.sum() ** 2 / D
    assert O.fp_model_objective(Tw, Wp, Xp) == pytest.approx(opt, rel=1e-9)
    # any other invertible transform is no better
    rng = np.random.default_rng(seed)
    for _ in range(100):
        R = rng.standard_normal((D, D))
        assert O.fp_model_objective(R, Wp, Xp) >= opt * (1 - 1e-9)
    for eps in (1e-3, 1e-1):
        P = Tw + eps * np.max(np.abs(Tw)) * rng.standard_normal((D, D))
        assert O.fp_model_objective(P, Wp, Xp) >= opt * (1 - 1e-9)
    # orthogonal T = T_X W'^{-T}  (incl. identity and plain Hadamard) gives tr(S^2)
    Q, _ = np.linalg.qr(rng.standard_normal((D, D)))
    for Tm in (np.eye(D), O.hadamard(D), Q):
        assert O.fp_model_objective(Tm @ Wp.T, Wp, Xp) == pytest.approx(np.sum(s ** 2), rel=1e-9)
    # dropping either ingredient falls back to tr(S^2): U' = I  or  S' = I
    no_h = np.diag(s ** -0.5) @ U.T @ Wp.T
    no_s = O.hadamard(D) @ U.T @ Wp.T
    assert O.fp_model_objective(no_h, Wp, Xp) == pytest.approx(np.sum(s ** 2), rel=1e-9)
    assert O.fp_model_objective(no_s, Wp, Xp) == pytest.approx(np.sum(s ** 2), rel=1e-9)
    # trace sandwich
    assert np.sum(s ** 2) >= opt >= np.sum(s ** 2) / D


def test_singular_values_descending_and_factorization():
    M_W, M_X = _moments(7)
    lam = 1e-2
    Wp, Xp, U, s, V = O.wush_factors(M_W, M_X, lam)
    assert np.all(np.diff(s) <= 0) and s[-1] > 0
    assert np.allclose(np.tril(Wp), Wp) and np.allclose(np.tril(Xp), Xp)
    assert np.allclose(Wp @ Wp.T, O.damped(M_W, lam), rtol=1e-12, atol=0)
    assert np.allclose(U @ np.diag(s) @ V.T, Wp.T @ Xp, atol=1e-12 * s[0])
    assert np.allclose(U.T @ U, np.eye(D), atol=1e-12)
    # damping adds lam * tr(M)/d to the diagonal only
    assert np.allclose(O.damped(M_W, lam) - M_W, lam * np.trace(M_W) / D * np.eye(D))


def test_invariance_to_choice_of_moment_factor():
    """Replacing the Cholesky factors by symmetric square roots leaves T_wush
    unchanged up to the signs of singular vectors, i.e. up to H -> H diag(+-1)."""
    lam = 1e-3
    M_W, M_X = _moments(8)
    T_chol = O.wush_block(M_W, M_X, lam)

    def sym_sqrt(Mm):
        w, Q = np.linalg.eigh(Mm)
        return Q @ np.diag(np.sqrt(w)) @ Q.T

    Wp, Xp = sym_sqrt(O.damped(M_W, lam)), sym_sqrt(O.damped(M_X, lam))
    U, s, Vt = np.linalg.svd(Wp.T @ Xp)
    H = O.hadamard(D)
    T_sym = H @ np.diag(s ** -0.5) @ U.T @ Wp.T
    A, B = H.T @ T_chol, H.T @ T_sym          # rows equal up to sign
    sign = np.sign(np.sum(A * B, axis=1))
    assert np.max(np.abs(A - sign[:, None] * B)) < 1e-8 * np.max(np.abs(A))


def test_special_case_identity_moments_gives_orthogonal_transform():
    T = O.wush_block(np.eye(D), np.eye(D), 0.0)
    assert np.max(np.abs(T @ T.T - np.eye(D))) < 1e-12


def test_special_case_diagonal_activation_moment():
    """M_W = I, M_X = diag(sigma^2): W'^T X' = diag(sigma), so T_wush must be a
    per-channel rescale by sigma^(-1/2) followed by (a column-permuted, signed) H."""
    rng = np.random.default_rng(9)
    sigma = rng.lognormal(0, 1, D)
    T = O.wush_block(np.eye(D), np.diag(sigma ** 2), 0.0)
    Z = T @ np.diag(np.sqrt(sigma))                       # should be H P^T
    assert np.max(np.abs(Z @ Z.T - np.eye(D))) < 1e-10
    Pm = np.abs(O.hadamard(D).T @ Z)                      # |signed permutation|
    assert np.allclose(np.sort(Pm, axis=0)[-1], 1.0, atol=1e-10)
    assert np.allclose(Pm.sum(axis=0), 1.0, atol=1e-9) and np.allclose(Pm.sum(axis=1), 1.0, atol=1e-9)
    # the permutation sorts sigma in descending order: column k of Z is row rank(k) of ... H
    order = np.argsort(-sigma)
    assert np.array_equal(np.argmax(Pm, axis=0)[order], np.arange(D))


def test_build_transforms_matches_per_block_call():
    rng = np.random.default_rng(10)
    W = rng.standard_normal((64, 3 * D)) * 0.02
    X = rng.standard_normal((128, 3 * D)) * rng.lognormal(0, 1, 3 * D)
    T = O.build_transforms(W, X, 1e-2)
    assert T.shape == (3, D, D)
    b = 1
    ref = O.wush_block(W[:, 32:64].T @ W[:, 32:64] / 64, X[:, 32:64].T @ X[:, 32:64] / 128, 1e-2)
    assert np.allclose(T[b], ref, rtol=1e-12, atol=0)
