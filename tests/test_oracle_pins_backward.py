"""Pins for the backward oracle (CPU only).  The oracle differentiates a PyTorch fp64 forward typed from the
objective; the pins tie it to things it does not contain: the C oracle's forward (a separate implementation) through
central finite differences, the paper's own expression for the value gradient, the constant-shift property of the
output weights, and the softmax-attention limit differentiated by the library's fused attention."""
import numpy as np
import pytest
import torch

import oracle
from oracle import backward as ob


def _rand(n, d, dv, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n, d)), rng.standard_normal((n, d)), rng.standard_normal((n, dv)),
            rng.standard_normal((n, dv)))


def _loss_c(Q, K, V, G, lam, scale):
    """L = sum_i g_i . o_i with the C oracle's forward (normal equations + Cholesky in C, no PyTorch)."""
    O, _, _ = oracle.forward_head_ex(Q, K, V, lam, scale)
    return float(np.sum(O * G))


def test_the_differentiated_forward_is_the_c_oracles_forward():
    Q, K, V, _ = _rand(45, 6, 4, 1)
    lam = np.random.default_rng(2).uniform(0.01, 0.5, 45)
    assert np.allclose(ob.forward_head(Q, K, V, 0.07, 0.6), oracle.forward_head(Q, K, V, 0.07, 0.6), rtol=1e-9, atol=1e-11)
    assert np.allclose(ob.forward_head(Q, K, V, lam, 0.6), oracle.forward_head_ex(Q, K, V, lam, 0.6)[0], rtol=1e-9,
                       atol=1e-11)


@pytest.mark.parametrize("lam,scale,seed", [(0.3, 0.5, 3), (0.01, 0.35, 4), (2.0, 1.0, 5)])
def test_gradients_match_central_differences_of_the_c_oracle(lam, scale, seed):
    """Directional derivatives along random directions for each argument, and single coordinates (the key holding a
    row's maximum among them, where the derivative of the row maximum enters)."""
    n, d, dv = 24, 5, 3
    Q, K, V, G = _rand(n, d, dv, seed)
    lam_rows = np.full(n, lam) * np.random.default_rng(seed + 50).uniform(0.5, 2.0, n)
    dQ, dK, dV, dlam = ob.backward_head(Q, K, V, G, lam_rows, scale)
    rng = np.random.default_rng(seed + 100)
    h = 1e-6

    def fd(dq=0, dk=0, dv_=0, dl=0):
        return (_loss_c(Q + h * dq, K + h * dk, V + h * dv_, G, lam_rows + h * dl, scale)
                - _loss_c(Q - h * dq, K - h * dk, V - h * dv_, G, lam_rows - h * dl, scale)) / (2 * h)

    for _ in range(3):
        eq, ek, ev = rng.standard_normal(Q.shape), rng.standard_normal(K.shape), rng.standard_normal(V.shape)
        el = rng.standard_normal(n) * lam_rows
        for got, ref in ((np.sum(dQ * eq), fd(dq=eq)), (np.sum(dK * ek), fd(dk=ek)), (np.sum(dV * ev), fd(dv_=ev)),
                         (np.sum(dlam * el), fd(dl=el))):
            assert np.isclose(got, ref, rtol=2e-6, atol=1e-8), (got, ref)
    # single coordinates: the key with the largest logit of the last row, and a few others
    jstar = int(np.argmax(K @ Q[n - 1]))
    for (j, c) in ((jstar, 0), (jstar, d - 1), (0, 1), (n - 1, 2)):
        e = np.zeros_like(K)
        e[j, c] = 1.0
        assert np.isclose(dK[j, c], fd(dk=e), rtol=2e-6, atol=1e-8)
    for (i, c) in ((0, 0), (7, 3), (n - 1, 4)):
        e = np.zeros_like(Q)
        e[i, c] = 1.0
        assert np.isclose(dQ[i, c], fd(dq=e), rtol=2e-6, atol=1e-8)
    for i in (0, 5, n - 1):
        e = np.zeros(n)
        e[i] = 1.0
        assert np.isclose(dlam[i], fd(dl=e), rtol=2e-6, atol=1e-8)


def test_the_row_maximum_matters_for_the_gradient():
    """Under the reading that the ridge acts on max-normalised weights, treating the maximum as a constant gives a
    different (wrong) gradient: the finite-difference pin above would catch that omission."""
    n, d = 16, 4
    Q, K, V, G = _rand(n, d, 3, 6)
    lam, scale = 0.5, 0.8
    dQ, dK, _, _ = ob.backward_head(Q, K, V, G, lam, scale)
    Qt, Kt, Vt, Gt = (torch.tensor(x, requires_grad=True) for x in (Q, K, V, G))
    loss = 0.0
    for i in range(n):
        logits = scale * (Kt[: i + 1] @ Qt[i])
        w = torch.exp(logits - logits.max().detach())
        X = torch.cat([torch.ones(i + 1, 1, dtype=torch.float64), Kt[: i + 1] - Qt[i]], dim=1)
        pen = torch.ones(d + 1, dtype=torch.float64)
        pen[0] = 0
        A = X.T @ (w[:, None] * X) + torch.diag(pen * lam)
        loss = loss + (torch.linalg.solve(A, X.T @ (w[:, None] * Vt[: i + 1]))[0] * Gt[i]).sum()
    loss.backward()
    assert np.linalg.norm(Kt.grad.numpy() - dK) > 1e-3 * np.linalg.norm(dK)
    assert np.linalg.norm(Qt.grad.numpy() - dQ) > 1e-3 * np.linalg.norm(dQ)


def test_value_gradient_is_s_transposed_g():
    """Appendix D, first result: dL/dv_j = sum_{i >= j} s_ij g_i with s_ij = w_ij (1 - z_ij . rho_i) / delta_i, the
    weights of Eq. (lla) built here from the C oracle's rho and delta."""
    n, d, lam, scale = 30, 6, 0.05, 0.4
    Q, K, V, G = _rand(n, d, 4, 7)
    _, R, Dl = oracle.forward_head_ex(Q, K, V, lam, scale)
    S = np.zeros((n, n))
    for i in range(n):
        lg = scale * (K[: i + 1] @ Q[i])
        w = np.exp(lg - lg.max())
        S[i, : i + 1] = w * (1.0 - (K[: i + 1] - Q[i]) @ R[i]) / Dl[i]
    _, _, dV, _ = ob.backward_head(Q, K, V, G, lam, scale)
    assert np.allclose(dV, S.T @ G, rtol=1e-8, atol=1e-10)


def test_value_gradients_sum_to_the_output_gradients():
    """The output weights of a row sum to one (the intercept is not penalised), so sum_j dV_j = sum_i g_i."""
    Q, K, V, G = _rand(33, 5, 4, 8)
    _, _, dV, _ = ob.backward_head(Q, K, V, G, 0.02, 0.7)
    assert np.allclose(dV.sum(0), G.sum(0), rtol=1e-8, atol=1e-10)


def test_huge_ridge_gives_the_gradients_of_softmax_attention():
    n, d, scale = 28, 6, 0.45
    Q, K, V, G = _rand(n, d, 6, 9)
    dQ, dK, dV, dlam = ob.backward_head(Q, K, V, G, 1e12, scale)
    Qt, Kt, Vt = (torch.tensor(x[None, None], requires_grad=True) for x in (Q, K, V))
    out = torch.nn.functional.scaled_dot_product_attention(Qt, Kt, Vt, is_causal=True, scale=scale)
    (out * torch.tensor(G[None, None])).sum().backward()
    for got, ref in ((dQ, Qt.grad), (dK, Kt.grad), (dV, Vt.grad)):
        assert np.allclose(got, ref[0, 0].numpy(), rtol=1e-6, atol=1e-8)
    assert np.all(np.abs(dlam) < 1e-12)


def test_rows_are_additive_and_see_only_their_prefix():
    Q, K, V, G = _rand(20, 4, 3, 10)
    full = ob.backward_head(Q, K, V, G, 0.1, 0.5)
    a = ob.backward_head(Q, K, V, G, 0.1, 0.5, rows=range(0, 20, 2))
    b = ob.backward_head(Q, K, V, G, 0.1, 0.5, rows=range(1, 20, 2))
    for f, x, y in zip(full, a, b):
        assert np.allclose(f, x + y, rtol=1e-10, atol=1e-12)
    only7 = ob.backward_head(Q, K, V, G, 0.1, 0.5, rows=[7])
    assert np.all(only7[1][8:] == 0) and np.all(only7[2][8:] == 0)
    assert np.all(np.delete(only7[0], 7, axis=0) == 0) and np.all(np.delete(only7[3], 7) == 0)
