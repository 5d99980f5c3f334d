"""Pins for the oracle's approximate mode (CPU only): rho from T conjugate-gradient steps with the matrix-free
product of Section 3.1 (solver of Appendix C).  Tied to: SciPy's CG on an explicitly built Sigma_i, the exact oracle
in the limit of many steps, the closed form of a single step, and the two degenerate settings of the active mask."""
import numpy as np
import pytest
import scipy.sparse.linalg as spla
import torch

import oracle


def _rand(n, d, dv, seed, spread=0.5):
    rng = np.random.default_rng(seed)
    return spread * rng.standard_normal((n, d)), spread * rng.standard_normal((n, d)), rng.standard_normal((n, dv))


def _moments(Q, K, i, lam, scale):
    s = scale * (K[: i + 1] @ Q[i])
    w = np.exp(s - s.max())
    Z = K[: i + 1] - Q[i]
    return w, w.sum(), (w[:, None] * Z).sum(0), (Z.T * w) @ Z + lam * np.eye(Q.shape[1])


@pytest.mark.parametrize("T", [1, 3, 7])
def test_rho_equals_scipy_cg_on_the_explicit_matrix(T):
    n, d, lam, scale = 30, 8, 0.05, 0.6
    Q, K, V = _rand(n, d, 4, 1)
    _, R, _, used = oracle.forward_head_cg(Q, K, V, lam, scale, T)
    for i in range(n):
        _, _, mu, Sigma = _moments(Q, K, i, lam, scale)
        x, _ = spla.cg(Sigma, mu, x0=np.zeros(d), maxiter=T, rtol=0.0, atol=0.0)
        assert np.allclose(R[i], x, rtol=1e-6, atol=1e-9), i     # two fp64 CG runs drift apart by rounding as they converge
        assert used[i] == T


def test_many_steps_reach_the_exact_oracle():
    n, d, lam, scale = 40, 6, 0.05, 0.5
    Q, K, V = _rand(n, d, 5, 2)
    Oe, Re, De = oracle.forward_head_ex(Q, K, V, lam, scale)
    Oc, Rc, Dc, _ = oracle.forward_head_cg(Q, K, V, lam, scale, T=4 * d)
    assert np.allclose(Rc, Re, rtol=1e-7, atol=1e-9)
    assert np.allclose(Dc, De, rtol=1e-7)
    assert np.allclose(Oc, Oe, rtol=1e-6, atol=1e-9)


def test_single_step_closed_form():
    """x1 = (mu.mu / mu.Sigma mu) mu, delta = omega - mu.x1, output by Eq. (lla)."""
    n, d, lam, scale = 20, 5, 0.1, 0.7
    Q, K, V = _rand(n, d, 3, 3)
    O, R, Dl, _ = oracle.forward_head_cg(Q, K, V, lam, scale, T=1)
    for i in range(n):
        w, omega, mu, Sigma = _moments(Q, K, i, lam, scale)
        x1 = (mu @ mu) / (mu @ Sigma @ mu) * mu if mu @ mu > 0 else np.zeros(d)
        delta = omega - mu @ x1
        s = w * (1.0 - (K[: i + 1] - Q[i]) @ x1) / delta
        assert np.allclose(R[i], x1, rtol=1e-9, atol=1e-12)
        assert np.isclose(Dl[i], delta, rtol=1e-10)
        assert np.allclose(O[i], s @ V[: i + 1], rtol=1e-9, atol=1e-12)


def test_zero_steps_or_a_huge_tolerance_give_softmax_attention():
    """rho = 0: delta = omega and the weights of Eq. (lla) are w_ij / omega_i."""
    n, d, scale = 25, 8, 0.4
    Q, K, V = _rand(n, d, 6, 4)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.tensor(Q)[None, None], torch.tensor(K)[None, None], torch.tensor(V)[None, None], is_causal=True,
        scale=scale)[0, 0].numpy()
    for kwargs in (dict(T=0), dict(T=10, eps=1e30)):
        O, R, _, used = oracle.forward_head_cg(Q, K, V, 0.05, scale, **kwargs)
        assert np.allclose(O, ref, rtol=1e-10, atol=1e-12)
        assert np.all(R == 0) and np.all(used == 0)


def test_active_mask_freezes_converged_rows():
    """With a tolerance, a row stops at the first iteration whose starting residual is below it; its rho is then the
    iterate of a run limited to that many steps, and its residual is indeed below the tolerance."""
    n, d, lam, scale, eps = 30, 6, 0.2, 0.5, 1e-3
    Q, K, V = _rand(n, d, 4, 5)
    _, R, _, used = oracle.forward_head_cg(Q, K, V, lam, scale, T=50, eps=eps)
    assert used.max() < 50 and used.min() >= 0
    for i in (0, 7, 29):
        _, Ri, _, _ = oracle.forward_head_cg(Q, K, V, lam, scale, T=int(used[i]), rows=[i])
        assert np.array_equal(Ri[0], R[i])
        _, _, mu, Sigma = _moments(Q, K, i, lam, scale)
        assert np.linalg.norm(mu - Sigma @ R[i]) < eps
