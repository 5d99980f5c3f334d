"""fp64 CPU oracle of the LLA backward pass -- TEST INFRASTRUCTURE ONLY.

The backward pass has a plain definition: the gradient of L = sum_i g_i . o_i with respect to Q, K, V (and the ridge
of every row), where o_i is the forward output.  It is written out as exactly that: the forward of one row is typed
from the objective of Section 2.3 (Eq. (lla_obj): exp-kernel weights on the causal prefix, intercept plus a linear
term in k - q, ridge on the linear term only, ridge applied to the max-normalised weights) with plain PyTorch CPU ops
in fp64, and PyTorch's reverse-mode differentiation does the rest.  No formula of Appendix D is used here.  The row
maximum is part of the function (it sets the scale on which the ridge acts), so its derivative is part of the
gradient.

Row i touches q_i, the keys and values j <= i and its own ridge only, so gradients can be taken for any subset of
rows: ``rows`` restricts the sum over i (equivalently: g_i = 0 for the other rows).

Nothing in the GPU package imports this module, and this module imports nothing from it.
"""
from __future__ import annotations

import numpy as np
import torch


def _t(x) -> torch.Tensor:
    if isinstance(x, torch.Tensor):
        return x.detach().cpu().double()
    return torch.as_tensor(np.asarray(x, dtype=np.float64))


def row_output(q, Kp, Vp, lam, scale: float) -> torch.Tensor:
    """The forward of one query: q [d], its visible keys Kp [m, d] and values Vp [m, dv], ridge lam (0-dim tensor or
    float).  Weighted ridge least squares of v on [1, k - q]; the fitted intercept is the output."""
    logits = scale * (Kp @ q)
    w = torch.exp(logits - logits.max())
    X = torch.cat([torch.ones_like(logits)[:, None], Kp - q], dim=1)          # [m, d+1]
    pen = torch.ones(X.shape[1], dtype=X.dtype)
    pen[0] = 0.0
    A = X.T @ (w[:, None] * X) + torch.diag(pen * lam)
    Bv = X.T @ (w[:, None] * Vp)
    return torch.linalg.solve(A, Bv)[0]


def forward_head(Q, K, V, lam, scale: float, rows=None) -> np.ndarray:
    """Causal forward of one head through ``row_output`` (for cross-checks with the C oracle)."""
    Q, K, V = _t(Q), _t(K), _t(V)
    n = Q.shape[0]
    lam_rows = _t(lam) if np.ndim(lam) else torch.full((n,), float(lam), dtype=torch.float64)
    rows = range(n) if rows is None else rows
    return np.stack([row_output(Q[i], K[: i + 1], V[: i + 1], lam_rows[i], scale).numpy() for i in rows])


def backward_head(Q, K, V, G, lam, scale: float, rows=None):
    """Gradients of L = sum_{i in rows} G[i] . o_i for one head.  Q, K: [n, d]; V, G: [n, dv]; ``lam`` a float or
    an [n] array.  Returns (dQ [n, d], dK [n, d], dV [n, dv], dlam [n]) in fp64; dlam[i] is dL / d lambda_i."""
    Q, K, V, G = _t(Q), _t(K), _t(V), _t(G)
    n = Q.shape[0]
    lam_rows = _t(lam).clone() if np.ndim(lam) else torch.full((n,), float(lam), dtype=torch.float64)
    Q.requires_grad_(True)
    K.requires_grad_(True)
    V.requires_grad_(True)
    lam_rows.requires_grad_(True)
    rows = range(n) if rows is None else [int(r) for r in rows]
    for i in rows:
        # one row at a time keeps the graph small; gradients accumulate in .grad
        o = row_output(Q[i], K[: i + 1], V[: i + 1], lam_rows[i], scale)
        (o * G[i]).sum().backward()
    z = lambda t: np.zeros(tuple(t.shape)) if t.grad is None else t.grad.numpy().copy()
    return z(Q), z(K), z(V), z(lam_rows)


def backward(Q, K, V, G, lam, scale: float, rows=None):
    """[B, H, n, d] inputs; ``lam`` a float or [B, H, n].  Returns (dQ, dK, dV, dlam) stacked over B, H."""
    Q, K, V, G = _t(Q), _t(K), _t(V), _t(G)
    B, H = Q.shape[:2]
    lam_a = _t(lam) if np.ndim(lam) else None
    res = [[backward_head(Q[b, h], K[b, h], V[b, h], G[b, h], lam if lam_a is None else lam_a[b, h], scale, rows)
            for h in range(H)] for b in range(B)]
    return tuple(np.asarray([[r[k] for r in row] for row in res]) for k in range(4))
