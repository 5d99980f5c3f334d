"""fp64 CPU formulas of the mechanisms the paper compares LLA with -- TEST INFRASTRUCTURE ONLY.

Plain numpy, one head at a time, written straight from the definitions in Section 2.2 (the regression view of
attention): the local-constant (Nadaraya-Watson) estimator that is softmax attention, the recurrent least-squares
solution that is MesaNet, its H ~ I shortcut that is vanilla linear attention, and the position-wise squared error
of Section 4.  Nothing in the GPU package imports this module.
"""
from __future__ import annotations

import numpy as np


def _f64(x) -> np.ndarray:
    if hasattr(x, "detach"):
        x = x.detach().cpu().double().numpy()
    return np.asarray(x, dtype=np.float64)


def softmax_attention(Q, K, V, scale: float) -> np.ndarray:
    """Eq. (local_constant) with w_ij = exp(scale q_i.k_j), causal j <= i.  Q, K: [n, d]; V: [n, dv]."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    n = Q.shape[0]
    out = np.empty((n, V.shape[1]))
    for i in range(n):
        logit = scale * (K[: i + 1] @ Q[i])
        w = np.exp(logit - logit.max())
        out[i] = (w / w.sum()) @ V[: i + 1]
    return out


def mesanet(Q, K, V, lam: float) -> np.ndarray:
    """Eq. (mesanet): S_i = sum_{j<=i} v_j k_j^T, H_i = sum_{j<=i} k_j k_j^T + lam I, prediction S_i H_i^{-1} q_i."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    n, d = Q.shape
    S = np.zeros((V.shape[1], d))
    H = lam * np.eye(d)
    out = np.empty((n, V.shape[1]))
    for i in range(n):
        S += np.outer(V[i], K[i])
        H += np.outer(K[i], K[i])
        out[i] = S @ np.linalg.solve(H, Q[i])
    return out


def linear_attention(Q, K, V) -> np.ndarray:
    """Vanilla linear attention: Eq. (mesanet) with H_i replaced by the identity (Section 2.2)."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    n, d = Q.shape
    S = np.zeros((V.shape[1], d))
    out = np.empty((n, V.shape[1]))
    for i in range(n):
        S += np.outer(V[i], K[i])
        out[i] = S @ Q[i]
    return out


def positionwise_mse(pred, target) -> np.ndarray:
    """l_i = || pred_i - v_i ||_2^2 (Section 4, test-time regression).  pred, target: [..., n, dv] -> [..., n]."""
    diff = _f64(pred) - _f64(target)
    return np.sum(diff * diff, axis=-1)
