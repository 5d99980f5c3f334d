"""Pins for the oracle's extras (CPU only): the per-row ridge (Appendix C: lambda learnable per position)
and the statistics rho_i, delta_i of Eq. (lla) that the paper's forward keeps for the backward pass.
Each pin ties the oracle to something other than itself: library least squares, a library linear solve on
moments built here, the closed form of the first row, and the paper's own output formula."""
import numpy as np
import pytest

import oracle


def _rand(n, d, dv, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n, d)), rng.standard_normal((n, d)), rng.standard_normal((n, dv))


def _weights(q, K, scale):
    s = scale * (K @ q)
    return np.exp(s - s.max())


def test_rho_delta_match_a_library_solve_on_moments_built_here():
    """Eq. (query_specific) + Eq. (lla): omega, mu, Sigma from their definitions in numpy, rho by numpy.linalg.solve."""
    n, d, lam, scale = 37, 6, 0.03, 0.4
    Q, K, V = _rand(n, d, 5, 1)
    _, R, Dl = oracle.forward_head_ex(Q, K, V, lam, scale)
    for i in range(n):
        w = _weights(Q[i], K[: i + 1], scale)
        Z = K[: i + 1] - Q[i]
        omega, mu = w.sum(), (w[:, None] * Z).sum(0)
        Sigma = (Z.T * w) @ Z + lam * np.eye(d)
        rho = np.linalg.solve(Sigma, mu)
        assert np.allclose(R[i], rho, rtol=1e-9, atol=1e-12)
        assert np.isclose(Dl[i], omega - mu @ rho, rtol=1e-8, atol=1e-13)


def test_output_formula_of_eq_lla_with_the_oracles_rho_and_delta():
    """o_i = sum_j w_ij (1 - z_ij . rho_i) / delta_i v_j must reproduce the oracle's own (lstsq-pinned) output."""
    n, d, lam, scale = 40, 8, 0.02, 0.3
    Q, K, V = _rand(n, d, 4, 2)
    O, R, Dl = oracle.forward_head_ex(Q, K, V, lam, scale)
    for i in range(n):
        w = _weights(Q[i], K[: i + 1], scale)
        Z = K[: i + 1] - Q[i]
        s = w * (1.0 - Z @ R[i]) / Dl[i]
        assert np.allclose(s @ V[: i + 1], O[i], rtol=1e-8, atol=1e-10)
        assert np.isclose(s.sum(), 1.0, rtol=1e-9)


def test_first_row_closed_form():
    """One visible key with weight 1: rho = z / (|z|^2 + lambda), delta = lambda / (|z|^2 + lambda)."""
    Q, K, V = _rand(5, 7, 3, 3)
    lam = 0.05
    _, R, Dl = oracle.forward_head_ex(Q, K, V, lam, 0.7, rows=[0])
    z = K[0] - Q[0]
    assert np.allclose(R[0], z / (z @ z + lam), rtol=1e-12)
    assert np.isclose(Dl[0], lam / (z @ z + lam), rtol=1e-11)


def test_delta_is_positive_and_at_most_omega():
    Q, K, V = _rand(60, 5, 2, 4)
    _, _, Dl = oracle.forward_head_ex(Q, K, V, 1e-3, 0.5)
    omega = np.array([_weights(Q[i], K[: i + 1], 0.5).sum() for i in range(60)])
    assert np.all(Dl > 0) and np.all(Dl <= omega * (1 + 1e-12))


def test_per_row_ridge_constant_array_equals_scalar():
    Q, K, V = _rand(30, 6, 4, 5)
    a = oracle.forward_head_ex(Q, K, V, 0.02, 0.4)
    b = oracle.forward_head_ex(Q, K, V, np.full(30, 0.02), 0.4)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_per_row_ridge_row_i_depends_on_lambda_i_only():
    Q, K, V = _rand(30, 6, 4, 6)
    rng = np.random.default_rng(7)
    lam1 = rng.uniform(1e-3, 1.0, 30)
    lam2 = rng.uniform(1e-3, 1.0, 30)
    lam2[[3, 17, 29]] = lam1[[3, 17, 29]]
    O1 = oracle.forward_head_ex(Q, K, V, lam1, 0.4)[0]
    O2 = oracle.forward_head_ex(Q, K, V, lam2, 0.4)[0]
    assert np.array_equal(O1[[3, 17, 29]], O2[[3, 17, 29]])
    assert not np.allclose(O1[10], O2[10])


def test_per_row_ridge_against_library_least_squares():
    """Row i: weighted ridge regression of the objective Eq. (lla_obj) with lambda_i, by numpy.linalg.lstsq."""
    n, d, dv, scale = 24, 5, 3, 0.5
    Q, K, V = _rand(n, d, dv, 8)
    lam = np.random.default_rng(9).uniform(1e-3, 0.5, n)
    O = oracle.forward_head_ex(Q, K, V, lam, scale)[0]
    for i in range(n):
        w = _weights(Q[i], K[: i + 1], scale)
        X = np.concatenate([np.ones((i + 1, 1)), K[: i + 1] - Q[i]], axis=1) * np.sqrt(w)[:, None]
        Y = V[: i + 1] * np.sqrt(w)[:, None]
        reg = np.sqrt(lam[i]) * np.concatenate([np.zeros((d, 1)), np.eye(d)], axis=1)
        theta = np.linalg.lstsq(np.concatenate([X, reg]), np.concatenate([Y, np.zeros((d, dv))]), rcond=None)[0]
        assert np.allclose(theta[0], O[i], rtol=1e-7, atol=1e-9)


def test_batched_wrapper_shapes_and_agreement():
    rng = np.random.default_rng(10)
    Q, K, V = [rng.standard_normal((2, 3, 12, 4)) for _ in range(3)]
    lam = rng.uniform(0.01, 0.1, (2, 3, 12))
    O, R, Dl = oracle.forward_ex(Q, K, V, lam, 0.5)
    assert O.shape == (2, 3, 12, 4) and R.shape == (2, 3, 12, 4) and Dl.shape == (2, 3, 12)
    o11 = oracle.forward_head_ex(Q[1, 1], K[1, 1], V[1, 1], lam[1, 1], 0.5)[0]
    assert np.array_equal(O[1, 1], o11)
