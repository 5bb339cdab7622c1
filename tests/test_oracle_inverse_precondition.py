"""Pins for the oracle's damped inverse and two-sided preconditioning."""
import numpy as np
import pytest

from oracle import kfac_oracle as orc
from workloads import rng, shapes


def _spd(seed, n, R=None):
    R = R or 2 * n
    X = rng.draw_normal(seed, 0, (R, n)).astype(np.float64)
    return X.T @ X / R, X


def test_inverse_small_closed_forms():
    assert np.allclose(orc.inverse(np.array([[4.0]]), 1.0), [[0.2]])
    a, b, d, lam = 3.0, 1.0, 2.0, 0.5
    det = (a + lam) * (d + lam) - b * b
    ref = np.array([[d + lam, -b], [-b, a + lam]]) / det
    for m in ("gj", "chol"):
        assert np.allclose(orc.inverse(np.array([[a, b], [b, d]]), lam, m), ref, rtol=1e-14)
    diag = np.diag([1.0, 2.0, 4.0, 8.0])
    assert np.allclose(orc.inverse(diag, 1.0), np.diag(1.0 / (np.array([1.0, 2.0, 4.0, 8.0]) + 1.0)), rtol=1e-15)


@pytest.mark.parametrize("n", [1, 2, 7, 33, 130])
def test_inverse_times_matrix_is_identity_and_routes_agree(n):
    M, _ = _spd(10 + n, n)
    lam = 0.03
    gj = orc.inverse(M, lam, "gj")
    ch = orc.inverse(M, lam, "chol")
    Md = M + lam * np.eye(n)
    assert np.linalg.norm(Md @ gj - np.eye(n)) / np.sqrt(n) < 1e-11
    assert np.linalg.norm(gj @ Md - np.eye(n)) / np.sqrt(n) < 1e-11
    assert np.linalg.norm(gj - ch) / np.linalg.norm(gj) < 1e-11
    assert np.linalg.norm(gj - np.linalg.inv(Md)) / np.linalg.norm(gj) < 1e-11


def test_inverse_needs_pivoting_case_and_asymmetry_probe():
    # Gauss-Jordan route on a general (non-symmetric, zero leading pivot) matrix
    M = np.array([[0.0, 2.0, 1.0], [1.0, 0.0, 3.0], [4.0, 1.0, 0.0]])
    assert np.allclose(orc.inverse(M, 0.0, "gj"), np.linalg.inv(M), rtol=1e-13)


def test_inverse_woodbury_for_rank_deficient_factor():
    # (lam I + s X^T X)^{-1} = (1/lam) [I - X^T ((lam/s) I_R + X X^T)^{-1} X], R < d
    R, d, s, lam = 4, 11, 0.25, 0.03
    X = rng.draw_normal(21, 0, (R, d)).astype(np.float64)
    F = orc.factor(X, s)
    small = np.linalg.inv((lam / s) * np.eye(R) + X @ X.T)
    ref = (np.eye(d) - X.T @ small @ X) / lam
    for m in ("gj", "chol"):
        got = orc.inverse(F, lam, m)
        assert np.linalg.norm(got - ref) / np.linalg.norm(ref) < 1e-11


def test_inverse_large_damping_limit_and_spd_failure_flag():
    M, _ = _spd(30, 6)
    lam = 1e9
    assert np.allclose(orc.inverse(M, lam) * lam, np.eye(6), atol=1e-8)
    bad = np.diag([1.0, 2.0, -3.0, 4.0])
    assert orc.inverse_info(bad, 0.0) == 3           # first non-positive pivot, 1-based
    assert orc.inverse_info(bad, 3.5) == 0


def test_precondition_plain_product_with_nonsymmetric_operands():
    # catches transposed operands / swapped sides, which symmetric inverses would hide
    gen = np.random.default_rng(5)
    Gi, Ai, g = gen.standard_normal((4, 4)), gen.standard_normal((7, 7)), gen.standard_normal((4, 7))
    assert np.allclose(orc.precondition(Gi, g, Ai), Gi @ g @ Ai, rtol=1e-13, atol=1e-13)


def test_precondition_identity_factors():
    g = rng.draw_normal(8, 2, (5, 9)).astype(np.float64)
    lamA, lamG = 0.03, 0.2
    Ai = orc.inverse(np.eye(9), lamA)
    Gi = orc.inverse(np.eye(5), lamG)
    assert np.allclose(orc.precondition(Gi, g, Ai), g / ((1 + lamA) * (1 + lamG)), rtol=1e-13)


def _kron_solve(A, G, grad):
    """[(A (x) G)]^{-1} vec(grad) with column-major vec of the d_G x d_A matrix."""
    dG, dA = grad.shape
    K = np.kron(A, G)
    v = np.linalg.solve(K, grad.reshape(-1, order="F"))
    return v.reshape((dG, dA), order="F")


def test_precondition_equals_explicit_kronecker_inverse_small():
    dA, dG = 7, 4
    A, _ = _spd(40, dA)
    G, _ = _spd(41, dG)
    grad = rng.draw_normal(42, 2, (dG, dA)).astype(np.float64)
    # undamped, full rank: Eq. 5
    P0 = orc.precondition(orc.inverse(G, 0.0), grad, orc.inverse(A, 0.0))
    assert np.allclose(P0, _kron_solve(A, G, grad), rtol=1e-9, atol=1e-11)
    # damping applied per factor: right-hand side of Eq. 12
    lamA, lamG = 0.05, 0.2
    P = orc.precondition(orc.inverse(G, lamG), grad, orc.inverse(A, lamA))
    ref = _kron_solve(A + lamA * np.eye(dA), G + lamG * np.eye(dG), grad)
    assert np.allclose(P, ref, rtol=1e-10, atol=1e-12)


def test_whole_fc_config_against_explicit_kronecker_system():
    # config 1 end to end: 65x65 (x) 32x32 = 2080 x 2080 dense system
    layer = shapes.config_layers("fc_tiny")[0]
    hp = shapes.config_hparams("fc_tiny")
    act, gout, grad = rng.layer_inputs(layer, hp["batch"], 1000, hp["act"], hp["gout_var"] ** 0.5)
    sA, sG = shapes.layer_scales(layer, hp["batch"])
    A, G = orc.update_factors_layer(layer, act, gout, sA, sG, hp["decay"], np.eye(65), np.eye(32))
    lam = hp["damping"]
    Ai, Gi = orc.invert_layer(A, G, lam, lam)
    P = orc.precondition_layer(Ai, Gi, grad)
    ref = _kron_solve(A + lam * np.eye(65), G + lam * np.eye(32), grad.astype(np.float64))
    assert np.linalg.norm(P - ref) / np.linalg.norm(ref) < 1e-10
    # independent reconstruction of the running factors (numpy route)
    abar = np.concatenate([act, np.ones((32, 1), np.float32)], axis=1).astype(np.float64)
    assert np.allclose(A, 0.95 * np.eye(65) + 0.05 * abar.T @ abar / 32, rtol=1e-12, atol=1e-14)
    assert np.allclose(G, 0.95 * np.eye(32) + 0.05 * gout.astype(np.float64).T @ gout.astype(np.float64) / 32,
                       rtol=1e-12, atol=1e-14)


def test_eigen_form_is_exact_inverse_of_damped_kronecker_product():
    # Eq. 13 reproduces (A (x) G + gamma I)^{-1} vec(grad) exactly; Eq. 12's
    # factored damping is only an approximation of it (the gap is reported, not asserted small).
    dA, dG, gamma = 6, 4, 0.01
    A, _ = _spd(50, dA)
    G, _ = _spd(51, dG)
    grad = rng.draw_normal(52, 2, (dG, dA)).astype(np.float64)
    vA, QA = np.linalg.eigh(A)
    vG, QG = np.linalg.eigh(G)
    P = orc.precondition_eigen(QG, vG, QA, vA, grad, gamma)
    K = np.kron(A, G) + gamma * np.eye(dA * dG)
    ref = np.linalg.solve(K, grad.reshape(-1, order="F")).reshape((dG, dA), order="F")
    assert np.allclose(P, ref, rtol=1e-10, atol=1e-12)
    # pi-scaled per-factor damping of Eq. 12 stays within a loose factor of the exact form
    pi = np.sqrt(np.trace(A) / dA) / np.sqrt(np.trace(G) / dG)
    P12 = orc.precondition(orc.inverse(G, np.sqrt(gamma) / pi), grad, orc.inverse(A, pi * np.sqrt(gamma)))
    gap = np.linalg.norm(P12 - ref) / np.linalg.norm(ref)
    assert gap < 1.0


# ---- eigen-decomposition of the factors (Eq. 13) ----------------------------------------------

def test_eigh_closed_forms():
    # diagonal matrix: eigenvalues are the entries, ascending; eigenvectors are unit vectors
    v, Q = orc.eigh(np.diag([3.0, -1.0, 2.0]))
    assert np.array_equal(v, [-1.0, 2.0, 3.0])
    assert np.array_equal(np.abs(Q), np.eye(3)[:, [1, 2, 0]])
    # 2 x 2: [[a, b], [b, a]] has a -+ b with eigenvectors (1, -+1) / sqrt 2
    v, Q = orc.eigh(np.array([[2.0, 0.5], [0.5, 2.0]]))
    assert np.allclose(v, [1.5, 2.5], rtol=0, atol=1e-15)
    assert np.allclose(np.abs(Q), np.full((2, 2), np.sqrt(0.5)), atol=1e-15) and Q[0, 0] * Q[1, 0] < 0 < Q[0, 1] * Q[1, 1]
    # identity plus rank one: c I + u u^T has one eigenvalue c + |u|^2 (vector u / |u|), the rest c
    u = rng.draw_normal(60, 0, (9,)).astype(np.float64)
    v, Q = orc.eigh(0.7 * np.eye(9) + np.outer(u, u))
    assert np.allclose(v[:-1], 0.7, atol=1e-13) and abs(v[-1] - (0.7 + u @ u)) < 1e-12
    assert abs(abs(Q[:, -1] @ u) - np.linalg.norm(u)) < 1e-12


@pytest.mark.parametrize("n", [1, 2, 5, 33, 80])
def test_eigh_against_lapack_and_invariants(n):
    M, _ = _spd(70 + n, n)
    M[0, n - 1] = M[n - 1, 0] = M[0, n - 1] - 0.3          # not a Gram matrix any more; may be indefinite
    v, Q = orc.eigh(M)
    assert np.allclose(v, np.linalg.eigvalsh(M), rtol=1e-12, atol=1e-13 * np.abs(M).max())
    assert np.all(np.diff(v) >= 0)
    assert np.allclose(Q.T @ Q, np.eye(n), atol=1e-13)
    assert np.allclose(M @ Q, Q * v, atol=1e-12 * np.abs(M).max())
    assert abs(v.sum() - np.trace(M)) < 1e-12 * np.abs(M).max() * n
    # a transposed (row) eigenvector layout would fail this for a non-symmetric Q
    assert np.allclose((Q * v) @ Q.T, M, atol=1e-12 * np.abs(M).max())


def test_eigen_layer_helper_matches_inverse_form_when_damping_factorises():
    # with gamma = 0 both Eq. 13 and the inverse form reduce to G^-1 grad A^-1
    dA, dG = 7, 5
    A, _ = _spd(81, dA)
    G, _ = _spd(82, dG)
    grad = rng.draw_normal(83, 2, (dG, dA)).astype(np.float64)
    P = orc.precondition_eigen_layer(A, G, grad, 0.0)
    ref = np.linalg.solve(G, grad) @ np.linalg.inv(A)
    assert np.allclose(P, ref, rtol=1e-9, atol=1e-11)
    # and with damping it is the exact damped Kronecker solve
    gamma = 0.02
    P = orc.precondition_eigen_layer(A, G, grad, gamma)
    K = np.kron(A, G) + gamma * np.eye(dA * dG)
    ref = np.linalg.solve(K, grad.reshape(-1, order="F")).reshape((dG, dA), order="F")
    assert np.allclose(P, ref, rtol=1e-10, atol=1e-12)


# ---- factored Tikhonov damping (Eq. 12) -------------------------------------------------------

def test_pi_damping_closed_forms():
    # A = a I, G = g I: pi = sqrt(a / g) whatever the orders
    lam_A, lam_G = orc.pi_damping(4.0 * np.eye(7), 0.25 * np.eye(3), 0.01)
    assert abs(lam_A - 4.0 * 0.1) < 1e-15 and abs(lam_G - 0.1 / 4.0) < 1e-15
    # equal mean eigenvalues: the split is symmetric, both terms are sqrt(gamma)
    A = np.diag([1.0, 2.0, 3.0])
    G = np.diag([2.0, 2.0])
    lam_A, lam_G = orc.pi_damping(A, G, 0.04)
    assert abs(lam_A - 0.2) < 1e-15 and abs(lam_G - 0.2) < 1e-15


def test_pi_damping_invariants():
    gen = np.random.default_rng(11)
    X = gen.standard_normal((40, 9)); A = X.T @ X / 40
    Y = gen.standard_normal((40, 5)); G = Y.T @ Y / 40 * 1e-3
    gamma = 0.003
    lam_A, lam_G = orc.pi_damping(A, G, gamma)
    assert abs(lam_A * lam_G - gamma) < 1e-15                      # the product of the two terms is gamma
    assert abs(lam_A / lam_G - (np.trace(A) / 9) / (np.trace(G) / 5)) < 1e-9 * lam_A / lam_G
    # scaling A by c scales pi by sqrt(c); off-diagonal entries do not matter
    lam_A2, lam_G2 = orc.pi_damping(9.0 * A, G, gamma)
    assert abs(lam_A2 - 3.0 * lam_A) < 1e-12 and abs(lam_G2 - lam_G / 3.0) < 1e-12
    A_off = A.copy(); A_off[0, 3] += 5.0
    assert orc.pi_damping(A_off, G, gamma) == (lam_A, lam_G)


def test_pi_is_the_split_that_minimises_the_cross_terms():
    # (A + lA I) (x) (G + lG I) = A (x) G + lA I (x) G + lG A (x) I + gamma I: with lA lG = gamma fixed, the
    # trace of the two cross terms, lA dA tr G + lG dG tr A, is smallest at the pi of Eq. 12
    gen = np.random.default_rng(12)
    X = gen.standard_normal((30, 6)); A = X.T @ X / 30
    Y = gen.standard_normal((30, 4)); G = Y.T @ Y / 30 * 0.05
    gamma = 0.01
    lam_A, lam_G = orc.pi_damping(A, G, gamma)
    cross = lambda lA: lA * 6 * np.trace(G) + (gamma / lA) * 4 * np.trace(A)
    grid = lam_A * np.exp(np.linspace(-2, 2, 4001))
    best = grid[np.argmin([cross(x) for x in grid])]
    assert abs(best - lam_A) < 2e-3 * lam_A
    assert cross(lam_A) <= cross(lam_A * 1.01) and cross(lam_A) <= cross(lam_A / 1.01)


def test_invert_layer_pi_is_the_plain_inverse_at_the_split_dampings():
    gen = np.random.default_rng(13)
    X = gen.standard_normal((50, 8)); A = X.T @ X / 50
    Y = gen.standard_normal((50, 5)); G = Y.T @ Y / 50
    Ai, Gi, lam_A, lam_G = orc.invert_layer_pi(A, G, 0.02)
    assert np.allclose(Ai @ (A + lam_A * np.eye(8)), np.eye(8), atol=1e-10)
    assert np.allclose(Gi @ (G + lam_G * np.eye(5)), np.eye(5), atol=1e-10)
    # non-positive trace: symmetric split
    assert orc.pi_damping(np.zeros((3, 3)), G, 0.04) == (0.2, 0.2)
