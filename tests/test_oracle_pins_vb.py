"""Pins of the variational E-step oracle (CPU only): closed forms, an invariant, and the definition evaluated by
brute force with a digamma of its own (a central difference of math.lgamma), so that a transposed operand, a
normalisation over the wrong axis, a dropped prior or a wrong sign fails at least one of them."""
import math

import numpy as np
import pytest

import oracle
from oracle import vb_estep
from helpers import csc_from_dense

EULER = 0.5772156649015329


def psi(x: float) -> float:
    h = 1e-5 * max(1.0, x)
    return (math.lgamma(x + h) - math.lgamma(x - h)) / (2 * h)


def toy(seed=0, D=7, V=11, cmax=5, density=0.6):
    rng = np.random.default_rng(seed)
    counts = rng.integers(1, cmax + 1, size=(D, V)) * (rng.uniform(size=(D, V)) < density)
    counts[3, :] = 0                                     # an empty document
    return csc_from_dense(counts), counts


def test_exp_elog_known_values():
    """psi(1) = -Euler's constant, psi(1/2) = -Euler - 2 ln 2, psi(2) = 1 - Euler."""
    a = vb_estep.exp_elog_theta(np.array([[1.0, 0.5]]))
    np.testing.assert_allclose(a[0, 0], math.exp(-EULER - psi(1.5)), rtol=1e-7)
    np.testing.assert_allclose(a[0, 1], math.exp(-EULER - 2 * math.log(2) - psi(1.5)), rtol=1e-7)
    np.testing.assert_allclose(psi(1.5), 2 - EULER - 2 * math.log(2), rtol=1e-8)          # psi(x+1) = psi(x) + 1/x


def test_exp_elog_beta_normalises_over_words_not_topics():
    """lambda constant over words within a topic, different between topics: b_wk = exp(psi(l_k) - psi(V l_k))."""
    V, K = 6, 3
    l = np.array([0.3, 1.0, 7.5])
    lam = np.tile(l, (V, 1))
    b = vb_estep.exp_elog_beta(lam)
    want = np.array([math.exp(psi(x) - psi(V * x)) for x in l])
    np.testing.assert_allclose(b, np.tile(want, (V, 1)), rtol=1e-7)
    # and a matrix that is not constant: column k depends on column k alone
    rng = np.random.default_rng(1)
    lam2 = rng.gamma(2.0, 1.0, size=(V, K))
    b2 = vb_estep.exp_elog_beta(lam2)
    lam3 = lam2.copy(); lam3[:, 1] *= 3.0
    b3 = vb_estep.exp_elog_beta(lam3)
    np.testing.assert_array_equal(b2[:, [0, 2]], b3[:, [0, 2]])
    assert not np.allclose(b2[:, 1], b3[:, 1])


def test_one_topic_closed_form():
    """K = 1: a = 1, mu_i = b_w, gamma' = alpha + N_d whatever lambda is."""
    X, counts = toy(seed=2)
    lam = np.random.default_rng(3).gamma(1.0, 1.0, size=(X.V, 1)) + 0.01
    b = vb_estep.exp_elog_beta(lam)
    g, mu = vb_estep.estep(X, b, 0.3, 3, np.full((X.D, 1), 5.0))
    np.testing.assert_allclose(g[:, 0], 0.3 + counts.sum(axis=1), rtol=1e-12)
    np.testing.assert_allclose(mu, b[X.rowidx, 0], rtol=1e-12)


@pytest.mark.parametrize("iters", [1, 4])
def test_row_sums_are_prior_plus_tokens(iters):
    """sum_k gamma'_dk = K alpha + N_d: the responsibilities of a token sum to one."""
    X, counts = toy(seed=4, D=9, V=13)
    K = 5
    rng = np.random.default_rng(5)
    b = vb_estep.exp_elog_beta(rng.gamma(0.7, 1.0, size=(X.V, K)) + 1e-3)
    g0 = rng.gamma(3.0, 1.0, size=(X.D, K))
    g, _ = vb_estep.estep(X, b, 0.2, iters, g0)
    np.testing.assert_allclose(g.sum(axis=1), K * 0.2 + counts.sum(axis=1), rtol=1e-12)
    np.testing.assert_allclose(g[3], 0.2, rtol=0)          # the empty document keeps the prior


def test_against_the_definition_by_brute_force():
    """Two iterations written out token by token: responsibilities phi_dwk proportional to
    exp(E log theta_dk) exp(E log beta_kw), gamma_dk = alpha + sum_w n_dw phi_dwk; digamma by central differences."""
    X, counts = toy(seed=6, D=5, V=6, cmax=3)
    D, V = counts.shape
    K, alpha = 3, 0.4
    rng = np.random.default_rng(7)
    lam = rng.gamma(1.5, 1.0, size=(V, K)) + 0.05
    g0 = rng.gamma(2.0, 1.0, size=(D, K)) + 0.1
    g, mu = vb_estep.estep(X, vb_estep.exp_elog_beta(lam), alpha, 2, g0)
    colsum = [sum(lam[w][k] for w in range(V)) for k in range(K)]
    elb = [[math.exp(psi(lam[w][k]) - psi(colsum[k])) for k in range(K)] for w in range(V)]
    want = np.zeros((D, K))
    for d in range(D):
        gd = list(g0[d])
        for _ in range(2):
            s = sum(gd)
            elt = [math.exp(psi(gd[k]) - psi(s)) for k in range(K)]
            new = [alpha] * K
            for w in range(V):
                if counts[d][w] == 0:
                    continue
                norm = sum(elt[k] * elb[w][k] for k in range(K))
                for k in range(K):
                    new[k] += counts[d][w] * elt[k] * elb[w][k] / norm
            gd = new
        want[d] = gd
    np.testing.assert_allclose(g, want, rtol=2e-6)
    # mu of the last iteration, for one nonzero, from the state before that iteration
    g1, _ = vb_estep.estep(X, vb_estep.exp_elog_beta(lam), alpha, 1, g0)
    i = int(X.colptr[1])
    w = int(X.rowidx[i])
    a1 = vb_estep.exp_elog_theta(g1)[1]
    np.testing.assert_allclose(mu[i], sum(a1[k] * elb[w][k] for k in range(K)), rtol=2e-6)


def test_zero_iterations_return_the_input():
    X, _ = toy(seed=8)
    g0 = np.random.default_rng(9).gamma(2.0, 1.0, size=(X.D, 4))
    g, _ = vb_estep.estep(X, np.ones((X.V, 4)), 0.1, 0, g0)
    np.testing.assert_array_equal(g, g0)
