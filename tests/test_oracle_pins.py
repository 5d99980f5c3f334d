"""Pins of the fp64 oracle to things other than itself (CPU only).

Each test checks oracle/llla_oracle.c against something the paper or the mathematics fixes:
a library least-squares solve of the defining objective, the paper's closed form evaluated
naively, invariants, limits, and a second algebraic route.  A dropped term, a wrong sign, a
transposed operand or a mis-indexed mask fails at least one of them.
"""
import math

import numpy as np
import pytest
import torch

import oracle

LAM = 1e-2


def _rand(n, d, dv=None, seed=0, spread=1.0):
    rng = np.random.default_rng(seed)
    dv = d if dv is None else dv
    return (spread * rng.standard_normal((n, d)), spread * rng.standard_normal((n, d)),
            rng.standard_normal((n, dv)))


def _weights(q, Kv, scale):
    s = scale * (Kv @ q)
    return np.exp(s - s.max())


def brute_force_row(Q, K, V, i, lam, scale, causal=True):
    """Eq. (lla_obj) handed to a library least-squares routine: rows sqrt(w_j) [1, k_j - q_i]
    against sqrt(w_j) v_j, plus sqrt(lam) rows on W only (the penalty that yields '+ lam I' in
    Eq. (query_specific)).  The prediction at q_i is the fitted intercept."""
    nk = i + 1 if causal else len(K)
    d = Q.shape[1]
    w = _weights(Q[i], K[:nk], scale)
    X = np.concatenate([np.ones((nk, 1)), K[:nk] - Q[i]], axis=1) * np.sqrt(w)[:, None]
    Y = V[:nk] * np.sqrt(w)[:, None]
    R = np.concatenate([np.zeros((d, 1)), math.sqrt(lam) * np.eye(d)], axis=1)
    Xa = np.concatenate([X, R], axis=0)
    Ya = np.concatenate([Y, np.zeros((d, V.shape[1]))], axis=0)
    theta = np.linalg.lstsq(Xa, Ya, rcond=None)[0]
    return theta[0]


def closed_form_row(Q, K, V, i, lam, scale):
    """Eq. (query_specific) and Eq. (lla) evaluated as printed, with numpy's solver."""
    nk = i + 1
    w = _weights(Q[i], K[:nk], scale)
    z = K[:nk] - Q[i]
    omega = w.sum()
    mu = (w[:, None] * z).sum(0)
    Sigma = (w[:, None, None] * z[:, :, None] * z[:, None, :]).sum(0) + lam * np.eye(Q.shape[1])
    rho = np.linalg.solve(Sigma, mu)
    s = w * (1.0 - z @ rho) / (omega - mu @ rho)
    return s @ V[:nk], rho, omega - mu @ rho


@pytest.mark.parametrize("n,d,dv,seed", [(24, 4, 4, 1), (48, 8, 8, 2), (40, 6, 3, 3)])
def test_P1_brute_force_lstsq(n, d, dv, seed):
    Q, K, V = _rand(n, d, dv, seed)
    scale = 1.0 / math.sqrt(d)
    O = oracle.forward_head(Q, K, V, LAM, scale)
    ref = np.stack([brute_force_row(Q, K, V, i, LAM, scale) for i in range(n)])
    assert np.abs(O - ref).max() <= 1e-9 * max(1.0, np.abs(ref).max())


def test_P1_brute_force_noncausal():
    Q, K, V = _rand(20, 5, 5, 4)
    O = oracle.forward_head(Q, K, V, LAM, 0.5, causal=False)
    ref = np.stack([brute_force_row(Q, K, V, i, LAM, 0.5, causal=False) for i in range(20)])
    assert np.abs(O - ref).max() <= 1e-9


@pytest.mark.parametrize("n,d,seed", [(48, 8, 5), (96, 16, 6)])
def test_P2_closed_form_eq_lla(n, d, seed):
    Q, K, V = _rand(n, d, d, seed)
    scale = 1.0 / math.sqrt(d)
    O = oracle.forward_head(Q, K, V, LAM, scale)
    ref = np.stack([closed_form_row(Q, K, V, i, LAM, scale)[0] for i in range(n)])
    assert np.abs(O - ref).max() <= 1e-8 * max(1.0, np.abs(ref).max())


def test_lambda_is_plus_lambda_I_not_two_lambda():
    """The ridge reading: a 2*lambda (literal derivative of the printed objective) would differ
    from Eq. (query_specific) at O(1e-2) here; the oracle must follow the latter."""
    Q, K, V = _rand(32, 8, 8, 7)
    scale = 1.0 / math.sqrt(8)
    O = oracle.forward_head(Q, K, V, LAM, scale)
    ref1 = np.stack([closed_form_row(Q, K, V, i, LAM, scale)[0] for i in range(32)])
    ref2 = np.stack([closed_form_row(Q, K, V, i, 2 * LAM, scale)[0] for i in range(32)])
    assert np.abs(O - ref1).max() < 1e-9
    assert np.abs(O - ref2).max() > 1e-4


def test_P3_constant_values_are_reproduced():
    Q, K, _ = _rand(64, 8, 8, 8)
    c = np.array([1.5, -2.0, 0.25, 3.0, 0.0, -1.0, 7.0, 1e-3])
    V = np.tile(c, (64, 1))
    for lam in (1e-4, 1e-2, 10.0):
        O = oracle.forward_head(Q, K, V, lam, 0.3)
        assert np.abs(O - c).max() <= 1e-8          # cond(A) reaches ~1e6 at lambda = 1e-4


def test_P4_first_row_is_first_value():
    Q, K, V = _rand(16, 8, 8, 9)
    for lam in (1e-3, 1e-2, 5.0):
        O = oracle.forward_head(Q, K, V, lam, 0.35, rows=[0])
        assert np.abs(O[0] - V[0]).max() <= 1e-12


def test_P5_affine_values_exact_identity_and_limit():
    """V = a + K B^T.  For any lambda: o_i = a + B (q_i + lambda rho_i / delta_i) (because
    sum_j s_ij z_ij = lambda rho_i / delta_i); hence o_i -> a + B q_i as lambda -> 0 on rows that
    determine the fit (i >= d + 1)."""
    n, d = 64, 6
    Q, K, _ = _rand(n, d, d, 10)
    rng = np.random.default_rng(11)
    a = rng.standard_normal(d)
    Bm = rng.standard_normal((d, d))
    V = a + K @ Bm.T
    scale = 0.4
    for lam in (1e-2, 1e-5):
        O = oracle.forward_head(Q, K, V, lam, scale)
        for i in range(n):
            _, rho, delta = closed_form_row(Q, K, V, i, lam, scale)
            ident = a + Bm @ (Q[i] + lam * rho / delta)
            assert np.abs(O[i] - ident).max() <= 1e-8
    errs = []
    for lam in (1e-4, 1e-6, 1e-8):
        O = oracle.forward_head(Q, K, V, lam, scale)
        errs.append(np.abs(O[d + 2:] - (a + Q[d + 2:] @ Bm.T)).max())
    assert errs[0] > errs[1] > errs[2]
    assert errs[2] < 1e-4
    assert errs[1] / errs[0] < 0.05 and errs[2] / errs[1] < 0.05     # error proportional to lambda


def test_P6_softmax_limit_matches_library_attention():
    """lambda -> infinity switches the slope off: Eq. (lla) tends to Eq. (local_constant), i.e.
    causal softmax attention, here computed by torch's scaled_dot_product_attention."""
    n, d = 96, 16
    Q, K, V = _rand(n, d, d, 12)
    scale = 1.0 / math.sqrt(d)
    O = oracle.forward_head(Q, K, V, 1e10, scale)
    t = lambda x: torch.from_numpy(x)[None, None]
    ref = torch.nn.functional.scaled_dot_product_attention(t(Q), t(K), t(V), is_causal=True,
                                                           scale=scale)[0, 0].numpy()
    assert np.abs(O - ref).max() <= 1e-7


def test_P7_logit_shift_invariance_via_constant_feature():
    """Appending a constant feature c to every key and t to every query shifts all logits of a
    row by scale*c*t and adds a regressor that is collinear with the intercept, whose ridge-
    optimal coefficient is 0: the output must not change (weights are max-normalised per row
    before lambda is applied, as in Algorithm 1)."""
    n, d = 40, 6
    Q, K, V = _rand(n, d, d, 13)
    O = oracle.forward_head(Q, K, V, LAM, 0.5)
    Qe = np.concatenate([Q, np.full((n, 1), 3.0)], axis=1)
    Ke = np.concatenate([K, np.full((n, 1), -2.0)], axis=1)
    Oe = oracle.forward_head(Qe, Ke, V, LAM, 0.5)
    assert np.abs(O - Oe).max() <= 1e-9


def test_P8_weights_are_max_normalised_before_ridge():
    """Raw weights exp(s) and max-shifted weights exp(s - m) give different outputs for the same
    lambda (Eq. (lla) is homogeneous in w only together with lambda).  The oracle must equal the
    brute force built on max-shifted weights and equal the raw-weight closed form only when
    lambda is rescaled by exp(-m_i)."""
    n, d = 24, 4
    Q, K, V = _rand(n, d, d, 14, spread=2.0)
    scale = 1.0
    O = oracle.forward_head(Q, K, V, LAM, scale)
    for i in (5, 17, 23):
        s = scale * (K[: i + 1] @ Q[i])
        m = s.max()
        z = K[: i + 1] - Q[i]

        def closed(w, lam):
            omega = w.sum()
            mu = (w[:, None] * z).sum(0)
            Sig = (z.T * w) @ z + lam * np.eye(d)
            rho = np.linalg.solve(Sig, mu)
            return (w * (1 - z @ rho) / (omega - mu @ rho)) @ V[: i + 1]

        raw_same_lambda = closed(np.exp(s), LAM)
        raw_scaled_lambda = closed(np.exp(s), LAM * math.exp(m))
        assert np.abs(O[i] - raw_scaled_lambda).max() <= 1e-8
        assert np.abs(O[i] - raw_same_lambda).max() > 1e-6


def test_P9_decode_equals_last_row_and_prefix_property():
    n, d = 50, 8
    Q, K, V = _rand(n, d, d, 15)
    scale = 1.0 / math.sqrt(d)
    O = oracle.forward_head(Q, K, V, LAM, scale)
    o = oracle.decode(Q[None, None, -1], K[None, None], V[None, None], LAM, scale)[0, 0]
    assert np.abs(o - O[-1]).max() <= 1e-12
    i = 30                       # row i of a long forward == last row of a length-(i+1) forward
    Oi = oracle.forward_head(Q[: i + 1], K[: i + 1], V[: i + 1], LAM, scale, rows=[i])[0]
    assert np.abs(Oi - O[i]).max() <= 1e-12
    # per-sequence lengths in a padded cache
    Kc = np.stack([K, K])[:, None]
    Vc = np.stack([V, V])[:, None]
    qq = np.stack([Q[19], Q[-1]])[:, None]
    od = oracle.decode(qq, Kc, Vc, LAM, scale, seqlens=[20, n])
    assert np.abs(od[0, 0] - O[19]).max() <= 1e-12 and np.abs(od[1, 0] - O[-1]).max() <= 1e-12


def test_decode_is_invariant_under_a_permutation_of_the_cache():
    """A decode step is a weighted least-squares fit over a SET of (key, value) pairs (Eq. (lla_obj): a sum over j
    with weights that depend on q and k_j only), so reordering the cache rows, keys and values together, cannot
    change it.  (A forward row sees a prefix and is not invariant; this pins that the decode oracle uses nothing
    positional.)"""
    n, d = 40, 8
    Q, K, V = _rand(n, d, d, 21)
    scale = 1.0 / math.sqrt(d)
    o = oracle.decode(Q[None, None, -1], K[None, None], V[None, None], LAM, scale)[0, 0]
    perm = np.random.default_rng(5).permutation(n)
    op = oracle.decode(Q[None, None, -1], K[None, None, perm], V[None, None, perm], LAM, scale)[0, 0]
    assert np.abs(o - op).max() <= 1e-12
    # and it is NOT invariant when only the keys are permuted (a mistake that pairs k_j with the wrong v_j shows)
    ow = oracle.decode(Q[None, None, -1], K[None, None, perm], V[None, None], LAM, scale)[0, 0]
    assert np.abs(o - ow).max() > 1e-3


def test_P10_uncentred_augmented_identity():
    """Second algebraic route: with phi_j = [1; k_j], At = sum w phi phi^T + lam diag(0, I) and
    y = At^{-1} [1; q_i], the output is sum_j w_j (phi_j . y) v_j (the fit c + W x evaluated at q_i
    is translation invariant because only W is penalised)."""
    n, d = 48, 8
    Q, K, V = _rand(n, d, d, 16)
    scale = 0.3
    O = oracle.forward_head(Q, K, V, LAM, scale)
    for i in range(n):
        w = _weights(Q[i], K[: i + 1], scale)
        phi = np.concatenate([np.ones((i + 1, 1)), K[: i + 1]], axis=1)
        At = (phi.T * w) @ phi + LAM * np.diag([0.0] + [1.0] * d)
        y = np.linalg.solve(At, np.concatenate([[1.0], Q[i]]))
        o = (w * (phi @ y)) @ V[: i + 1]
        assert np.abs(o - O[i]).max() <= 1e-8


def test_causal_mask_is_inclusive_and_strict():
    """Row i must depend on (k_i, v_i) and on nothing after it."""
    n, d = 20, 4
    Q, K, V = _rand(n, d, d, 17)
    O = oracle.forward_head(Q, K, V, LAM, 0.5)
    K2, V2 = K.copy(), V.copy()
    K2[11:] += 5.0
    V2[11:] -= 3.0
    O2 = oracle.forward_head(Q, K2, V2, LAM, 0.5)
    assert np.abs(O2[:11] - O[:11]).max() == 0.0          # future keys invisible
    assert np.abs(O2[11] - O[11]).max() > 1e-3            # own key/value visible


def test_row_weights_sum_to_one():
    """Only W is penalised, so the effective weights s_ij of Eq. (lla) sum to one: shifting all
    values by a constant shifts every output by that constant."""
    Q, K, V = _rand(32, 8, 8, 18)
    O = oracle.forward_head(Q, K, V, LAM, 0.4)
    O2 = oracle.forward_head(Q, K, V + 2.5, LAM, 0.4)
    assert np.abs(O2 - O - 2.5).max() <= 1e-9
