"""The fact the d = 16 / 32 matrix-core calls rest on, checked on the fp64 oracle (CPU): appending zero features to
every query and key, and zero columns to the values, changes nothing -- the padded block of the system of
Eq. (query_specific) is lambda * y = 0 -- and the gradients with respect to the appended entries vanish."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from oracle import backward as ob


def _inputs(n, d, seed):
    w = workloads.C2.with_shape(name="padinv", B=1, H=2, n=n, d=d, values="normal", index=seed, scale=d ** -0.5)
    return w, workloads.make_inputs(w)


def _pad(x, width):
    out = torch.zeros(x.shape[:-1] + (width,), dtype=x.dtype)
    out[..., :x.shape[-1]] = x
    return out


@pytest.mark.parametrize("d", [16, 32])
@pytest.mark.parametrize("causal", [True, False])
def test_forward_and_statistics_do_not_see_zero_features(d, causal):
    w, (Q, K, V) = _inputs(90, d, 2100 + d)
    O, R, D = oracle.forward_ex(Q, K, V, w.lam, w.scale, causal=causal)
    Op, Rp, Dp = oracle.forward_ex(_pad(Q, 64), _pad(K, 64), _pad(V, 64), w.lam, w.scale, causal=causal)
    np.testing.assert_allclose(Op[..., :d], O, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(Rp[..., :d], R, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(Dp, D, rtol=1e-9, atol=1e-12)
    assert np.abs(Op[..., d:]).max() == 0.0 and np.abs(Rp[..., d:]).max() <= 1e-13


@pytest.mark.parametrize("d", [16, 32])
def test_gradients_of_zero_features_vanish(d):
    w, (Q, K, V) = _inputs(60, d, 2200 + d)
    g = torch.Generator().manual_seed(2300 + d)
    G = torch.randn(Q.shape, generator=g, dtype=torch.float32)
    dQ, dK, dV, dlam = ob.backward(Q, K, V, G, w.lam, w.scale)
    pQ, pK, pV, plam = ob.backward(_pad(Q, 64), _pad(K, 64), _pad(V, 64), _pad(G, 64), w.lam, w.scale)
    for a, b in ((pQ, dQ), (pK, dK), (pV, dV)):
        np.testing.assert_allclose(a[..., :d], b, rtol=1e-8, atol=1e-10)
        assert np.abs(a[..., d:]).max() <= 1e-10 * max(1.0, np.abs(b).max())
    np.testing.assert_allclose(plam, dlam, rtol=1e-8, atol=1e-10)
