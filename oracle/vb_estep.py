"""CPU oracle for the E-step of online variational Bayes LDA: test infrastructure, not product code.

Section 5.3 of the paper names the normaliser of Algorithm 3 (SDDMM: a product of two dense matrices
evaluated at the nonzeros of a sparse one) as the bottleneck that the sampler shares with the authors' online
variational Bayes LDA.  The paper does not print that method; what is written out here is the published
E-step of online variational Bayes for LDA (Hoffman, Blei and Bach, 2010), restated, with the normaliser in
the same place: "parity unpinned" by the paper, pinned below by closed forms, an invariant and a brute-force
evaluation of the definition.

Definitions (all in double; ``digamma`` is the library routine):

    a_dk = exp(psi(gamma_dk) - psi(sum_k gamma_dk))           exp E[log theta_dk]
    b_wk = exp(psi(lambda_wk) - psi(sum_w lambda_wk))         exp E[log beta_kw], lambda stored word-major [V][K]
    mu_i = sum_k a_dk b_wk  for nonzero i = (d, w, c)         the normaliser (SDDMM)
    gamma'_dk = alpha + a_dk * sum_{i in d} (c_i / mu_i) b_wk

One iteration maps gamma to gamma'; the E-step repeats it a fixed number of times for every document.
Nothing here imports the GPU package, and the GPU package never imports this.
"""
from __future__ import annotations

import numpy as np
from scipy.special import digamma


def exp_elog_theta(gamma: np.ndarray) -> np.ndarray:
    """a = exp(E[log theta]) for rows of Dirichlet parameters gamma [D][K]."""
    g = np.asarray(gamma, np.float64)
    return np.exp(digamma(g) - digamma(g.sum(axis=1, keepdims=True)))


def exp_elog_beta(lam: np.ndarray) -> np.ndarray:
    """b = exp(E[log beta]) for topic-word Dirichlet parameters stored word-major, lam [V][K]: a topic is a
    column, normalised over the words."""
    l = np.asarray(lam, np.float64)
    return np.exp(digamma(l) - digamma(l.sum(axis=0, keepdims=True)))


def estep(X, b: np.ndarray, alpha: float, iters: int, gamma0: np.ndarray):
    """``iters`` iterations of the update for every document of the CSC matrix X (columns are documents).
    Returns (gamma [D][K], mu [nnz]); mu holds the normalisers of the last iteration (those the returned gamma
    was computed from)."""
    b = np.asarray(b, np.float64)
    gamma = np.array(gamma0, np.float64, copy=True)
    mu_out = np.zeros(X.rowidx.shape[0], np.float64)
    for d in range(X.D):
        lo, hi = int(X.colptr[d]), int(X.colptr[d + 1])
        words = X.rowidx[lo:hi]
        c = X.val[lo:hi].astype(np.float64)
        B = b[words]                                      # [n][K]
        g = gamma[d]
        for _ in range(iters):
            a = np.exp(digamma(g) - digamma(g.sum()))
            mu = B @ a
            g = alpha + a * ((c / mu) @ B) if hi > lo else np.full_like(g, alpha)
            mu_out[lo:hi] = mu
        gamma[d] = g
    return gamma, mu_out
