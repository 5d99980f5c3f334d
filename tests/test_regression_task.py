"""The paper's test-time regression task (Section 4; Appendix "Piecewise Linear Data Generation") on the CPU:
the generator's stated properties, pins for the plain formulas of the compared mechanisms (library softmax, library
ridge regression, the large-ridge limit), and the qualitative findings the paper reports for this task, computed with
the fp64 oracle.  The paper does not state the noise level, the ridge or the bandwidth it used, so only orderings are
checked, never the printed curves."""
import math

import numpy as np
import pytest
import scipy.special
import torch
from sklearn.linear_model import Ridge

import oracle
import workloads
from oracle import baselines


def _rand(n, d, dv, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n, d)), rng.standard_normal((n, d)), rng.standard_normal((n, dv))


# ---- generator ----------------------------------------------------------------------------------

def test_cone_signs_are_the_low_bits_of_the_segment_index():
    s = workloads.cone_signs(8).numpy()
    assert s.shape == (8, 3)
    for c in range(8):
        assert [int(x) for x in s[c]] == [1 if (c >> j) & 1 else -1 for j in range(3)]
    assert len({tuple(r) for r in s}) == 8                 # distinct patterns: the cones are disjoint
    assert workloads.cone_signs(1).shape == (1, 0)
    with pytest.raises(ValueError):
        workloads.cone_signs(6)


def test_keys_lie_in_their_segments_cone_and_values_follow_the_segments_map():
    w = workloads.E2S
    Q, K, V, A, seg = workloads.piecewise_linear(w)
    assert torch.equal(Q, K)
    signs = workloads.cone_signs(w.n // w.segment)
    m = signs.shape[1]
    assert m == 3
    assert torch.all(K[..., :m] * signs[seg] >= 0)
    # beyond the first m coordinates both signs occur
    assert (K[..., m:] < 0).float().mean() > 0.4
    # v - A_c k is the noise: mean 0, standard deviation `noise`
    Kseg = K.double().reshape(w.B, w.H, -1, w.segment, w.d)
    resid = V.double().reshape(Kseg.shape) - Kseg @ A.double().transpose(-1, -2)
    assert abs(float(resid.mean())) < 0.01
    assert abs(float(resid.std()) - w.noise) < 0.01
    # a different segment's map does not explain the values
    wrong = V.double().reshape(Kseg.shape) - Kseg @ A.double().roll(1, dims=2).transpose(-1, -2)
    assert float(wrong.std()) > 10 * w.noise


def test_generator_is_seeded():
    a = workloads.make_inputs(workloads.E2S)
    b = workloads.make_inputs(workloads.E2S)
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    c = workloads.make_inputs(workloads.E2S.with_shape(index=99))
    assert not torch.equal(a[1], c[1])


# ---- formulas of the compared mechanisms ----------------------------------------------------------

def test_softmax_attention_matches_library_softmax():
    Q, K, V = _rand(33, 5, 4, 11)
    scale = 0.37
    got = baselines.softmax_attention(Q, K, V, scale)
    logits = scale * (Q @ K.T)
    logits[np.triu_indices(33, 1)] = -np.inf
    assert np.allclose(got, scipy.special.softmax(logits, axis=1) @ V, rtol=1e-12, atol=1e-13)


def test_lla_with_a_huge_ridge_is_softmax_attention():
    """Section 2.3: with W forced to zero the local linear fit is the local constant fit."""
    Q, K, V = _rand(40, 6, 3, 12)
    lla = oracle.forward_head(Q, K, V, 1e13, 0.5)
    assert np.allclose(lla, baselines.softmax_attention(Q, K, V, 0.5), rtol=1e-8, atol=1e-9)


def test_mesanet_matches_library_ridge_regression():
    """Eq. (mesanet) is ridge regression of v on k without intercept over the causal prefix."""
    Q, K, V = _rand(30, 4, 3, 13)
    lam = 0.3
    got = baselines.mesanet(Q, K, V, lam)
    for i in (0, 3, 4, 17, 29):
        fit = Ridge(alpha=lam, fit_intercept=False, solver="cholesky").fit(K[: i + 1], V[: i + 1])
        assert np.allclose(got[i], fit.predict(Q[i][None])[0], rtol=1e-9, atol=1e-11)


def test_linear_attention_is_the_large_ridge_limit_of_mesanet_and_a_plain_masked_product():
    Q, K, V = _rand(25, 4, 3, 14)
    la = baselines.linear_attention(Q, K, V)
    assert np.allclose(la, np.tril(Q @ K.T) @ V, rtol=1e-12, atol=1e-12)
    lam = 1e9
    assert np.allclose(lam * baselines.mesanet(Q, K, V, lam), la, rtol=1e-6, atol=1e-8)


def test_positionwise_mse():
    a = np.arange(12.0).reshape(2, 3, 2)
    b = a + np.array([3.0, 4.0])
    assert np.allclose(baselines.positionwise_mse(a, b), 25.0)


# ---- what the paper reports for the task ----------------------------------------------------------

def _task_mse(w, n_seq):
    Q, K, V = workloads.make_inputs(w.with_shape(B=n_seq))
    acc = {k: np.zeros(w.n) for k in ("lla", "softmax", "mesa", "la", "random")}
    rng = np.random.default_rng(5)
    for b in range(n_seq):
        q, k, v = Q[b, 0], K[b, 0], V[b, 0]
        acc["lla"] += baselines.positionwise_mse(oracle.forward_head(q, k, v, w.lam, w.scale), v)
        acc["softmax"] += baselines.positionwise_mse(baselines.softmax_attention(q, k, v, w.scale), v)
        acc["mesa"] += baselines.positionwise_mse(baselines.mesanet(q, k, v, w.lam), v)
        acc["la"] += baselines.positionwise_mse(baselines.linear_attention(q, k, v), v)
        acc["random"] += baselines.positionwise_mse(rng.standard_normal((w.n, w.d)) * math.sqrt(w.d), v)
    return {k: a / n_seq for k, a in acc.items()}


def test_reported_orderings_on_the_piecewise_linear_task():
    """Section 4, Figures regression_fit / scaling: LLA has the lowest error; MesaNet is good only before the first
    distribution shift; the advantage of LLA over softmax attention grows with the dimension."""
    ratio = {}
    for d, S, n_seq in ((16, 64, 4), (64, 256, 2)):
        w = workloads.E2.with_shape(d=d, segment=S, dtype="f32", scale=1.0 / math.sqrt(d))
        mse = _task_mse(w, n_seq)
        total = {k: v.sum() for k, v in mse.items()}
        assert total["lla"] < total["softmax"] < total["mesa"] < total["random"], total
        assert total["mesa"] < total["la"], total
        first, later = mse["mesa"][d:S].mean(), mse["mesa"][S:].mean()
        assert first < 1e-2 * later, (first, later)
        assert mse["lla"][S:].mean() < 0.5 * mse["mesa"][S:].mean()
        ratio[d] = total["softmax"] / total["lla"]
    assert ratio[64] > 5 * ratio[16], ratio
