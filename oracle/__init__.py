"""CPU oracle for the SAME Gibbs LDA sweep: test infrastructure, not product code.

Thin ctypes access to ``same_lda_oracle.c`` plus :class:`OracleLDA`, which strings
the C steps together in the order of Algorithm 3 of the paper (zero, draw and
accumulate, add priors, normalise over words, blend).  Nothing here imports the
GPU package, and the GPU package never imports this.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from ctypes import POINTER, c_double, c_float, c_int32, c_int64, c_uint32, c_uint64, c_void_p

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "same_lda_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_same_lda.so")

DOMAIN_TRAIN = 0
DOMAIN_HELDOUT = 1
DOMAIN_THETA = 2      # Gamma variables of the sampled theta step
DOMAIN_PHI = 3        # Gamma variables of the sampled phi step


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (one rounding per operation: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        u32p, f32p, i32p, i64p = POINTER(c_uint32), POINTER(c_float), POINTER(c_int32), POINTER(c_int64)
        L.oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.oracle_philox4x32_10.restype = None
        L.oracle_uniform_from_word.argtypes = [c_uint32]
        L.oracle_uniform_from_word.restype = c_float
        L.oracle_stream_uniform.argtypes = [c_uint64, c_uint64, c_uint32, c_uint32, c_uint32]
        L.oracle_stream_uniform.restype = c_float
        L.oracle_chain_uniform.argtypes = [c_uint64, c_uint64, c_uint32, c_uint32, c_uint32]
        L.oracle_chain_uniform.restype = c_float
        L.oracle_block_len.argtypes = [c_int32]
        L.oracle_block_len.restype = c_int32
        L.oracle_prefix.argtypes = [c_int32, f32p, f32p]
        L.oracle_prefix.restype = c_float
        L.oracle_top_position.argtypes = [c_float, c_uint32, c_float]
        L.oracle_top_position.restype = c_float
        L.oracle_log1m.argtypes = [c_float]
        L.oracle_log1m.restype = c_float
        L.oracle_binom_walk.argtypes = [c_uint32, c_float, c_float, c_float]
        L.oracle_binom_walk.restype = c_uint32
        L.oracle_binom.argtypes = [c_uint32, c_float, c_uint64, c_uint64, c_uint32, c_uint32]
        L.oracle_binom.restype = c_uint32
        L.oracle_draw.argtypes = [c_int32, f32p, c_uint32, c_uint64, c_uint64, c_uint32, u32p, f32p]
        L.oracle_draw.restype = c_float
        L.oracle_task_count.argtypes = [c_int64, f32p, c_int32]
        L.oracle_task_count.restype = c_int64
        L.oracle_task_base.argtypes = [c_int64, f32p, c_int32, i64p]
        L.oracle_task_base.restype = None
        L.oracle_pass.argtypes = [c_int32, c_int32, i32p, i32p, f32p, c_int32, c_int32, c_uint32,
                                  c_uint64, c_uint32, c_void_p, c_void_p, u32p, c_void_p, c_void_p]
        L.oracle_pass.restype = None
        L.oracle_draw_tasks.argtypes = [c_int32, i32p, i32p, f32p, c_int32, c_int32, c_uint32, c_uint64,
                                        c_uint32, c_void_p, c_void_p, c_int64, i64p, u32p]
        L.oracle_draw_tasks.restype = None
        L.oracle_theta_update.argtypes = [c_int32, c_int32, u32p, c_uint32, c_float, f32p]
        L.oracle_theta_update.restype = None
        L.oracle_phi_update.argtypes = [c_int32, c_int32, u32p, c_uint32, c_float, c_float, f32p]
        L.oracle_phi_update.restype = None
        L.oracle_expneg.argtypes = [c_float]
        L.oracle_expneg.restype = c_float
        L.oracle_poisson_walk.argtypes = [c_float, c_float, c_float]
        L.oracle_poisson_walk.restype = c_uint32
        L.oracle_poisson.argtypes = [c_float, c_uint64, c_uint64, c_uint32, c_uint32]
        L.oracle_poisson.restype = c_uint32
        L.oracle_draw_poisson.argtypes = [c_int32, f32p, c_float, c_uint64, c_uint64, c_uint32, u32p]
        L.oracle_draw_poisson.restype = c_float
        L.oracle_pass_poisson.argtypes = [c_int32, c_int32, i32p, i32p, f32p, c_int32, c_int32, c_float,
                                          c_uint64, c_uint32, c_void_p, c_void_p, u32p, c_void_p]
        L.oracle_pass_poisson.restype = None
        L.oracle_draw_tasks_poisson.argtypes = [c_int32, i32p, i32p, f32p, c_int32, c_int32, c_float, c_uint64,
                                                c_uint32, c_void_p, c_void_p, c_int64, i64p, u32p]
        L.oracle_draw_tasks_poisson.restype = None
        L.oracle_theta_update_real.argtypes = [c_int32, c_int32, u32p, c_float, c_float, f32p]
        L.oracle_theta_update_real.restype = None
        L.oracle_phi_update_real.argtypes = [c_int32, c_int32, u32p, c_float, c_float, c_float, f32p]
        L.oracle_phi_update_real.restype = None
        L.oracle_flog.argtypes = [c_float]
        L.oracle_flog.restype = c_float
        L.oracle_cos2pi.argtypes = [c_float]
        L.oracle_cos2pi.restype = c_float
        L.oracle_normal.argtypes = [c_float, c_float]
        L.oracle_normal.restype = c_float
        L.oracle_gamma.argtypes = [c_float, c_uint64, c_uint32, c_uint32, c_uint32]
        L.oracle_gamma.restype = c_float
        L.oracle_theta_sample.argtypes = [c_int32, c_int32, u32p, c_float, c_float, c_uint64, c_uint32, f32p]
        L.oracle_theta_sample.restype = None
        L.oracle_phi_sample.argtypes = [c_int32, c_int32, u32p, c_float, c_float, c_uint64, c_uint32, f32p]
        L.oracle_phi_sample.restype = None
        L.oracle_sddmm.argtypes = [c_int32, i32p, i32p, c_int32, f32p, f32p, ctypes.POINTER(c_double)]
        L.oracle_sddmm.restype = None
        L.oracle_loglik_eval.argtypes = [c_int32, i32p, i32p, f32p, c_int32, f32p, f32p]
        L.oracle_loglik_eval.restype = c_double
        _lib = L
    return _lib


def _p(a: np.ndarray, ty):
    return a.ctypes.data_as(POINTER(ty))


def _vp(a):
    return None if a is None else a.ctypes.data_as(c_void_p)


def pass_word(pass_index: int, domain: int = DOMAIN_TRAIN) -> int:
    """Fourth counter word of the stream: pass index (28 bits) and stream domain above."""
    assert 0 <= pass_index < (1 << 28)
    return (domain << 28) | pass_index


# --------------------------------------------------------------------------- #
# single-function access (used by the pins in tests/)
def philox(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_p(c, c_uint32), _p(k, c_uint32), _p(out, c_uint32))
    return out


def uniform_from_word(x: int) -> float:
    return float(lib().oracle_uniform_from_word(c_uint32(x)))


def stream_uniform(seed: int, tau: int, k: int, piece: int, pword: int) -> float:
    """Uniform of piece `piece` of topic k (stream layout of the Poisson form)."""
    return float(lib().oracle_stream_uniform(seed, tau, k, piece, pword))


def chain_uniform(seed: int, tau: int, step: int, slot: int, pword: int) -> float:
    """Uniform of step `step` of the multinomial draw: slot 0 places the highest copy, slot 1 + j decides
    piece j of the step's binomial."""
    return float(lib().oracle_chain_uniform(seed, tau, step, slot, pword))


def block_len(K: int) -> int:
    return int(lib().oracle_block_len(K))


def prefix(w):
    """Two-level running sums of the weights: returns (P[K], mu)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    P = np.zeros(w.shape[0], dtype=np.float32)
    mu = lib().oracle_prefix(w.shape[0], _p(w, c_float), _p(P, c_float))
    return P, float(mu)


def top_position(U: float, R: int, u: float) -> float:
    """Position of the highest of R copies uniform on (0, U), from one uniform u."""
    return float(lib().oracle_top_position(c_float(U), R, c_float(u)))


def log1m(x: float) -> float:
    """-log(1 - x) for 0 < x <= 1/2."""
    return float(lib().oracle_log1m(c_float(x)))


def binom_walk(n: int, pm0: float, r: float, u: float) -> int:
    return int(lib().oracle_binom_walk(n, c_float(pm0), c_float(r), c_float(u)))


def binom(R: int, q: float, seed: int, tau: int, step: int, pword: int) -> int:
    return int(lib().oracle_binom(R, c_float(q), seed, tau, step, pword))


def draw(w, N: int, seed: int, tau: int, pword: int):
    """One factored draw from weights w: returns (counts[K], normaliser)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    K = w.shape[0]
    counts = np.zeros(K, dtype=np.uint32)
    scratch = np.zeros(K, dtype=np.float32)
    S = lib().oracle_draw(K, _p(w, c_float), N, seed, tau, pword, _p(counts, c_uint32), _p(scratch, c_float))
    return counts, float(S)


class CSC:
    """Sparse words x documents count matrix, one column per document."""

    def __init__(self, D, V, colptr, rowidx, val):
        self.D, self.V = int(D), int(V)
        self.colptr = np.ascontiguousarray(colptr, dtype=np.int32)
        self.rowidx = np.ascontiguousarray(rowidx, dtype=np.int32)
        self.val = np.ascontiguousarray(val, dtype=np.float32)
        assert self.colptr.shape == (self.D + 1,)
        self.nnz = int(self.colptr[-1])
        assert self.rowidx.shape == (self.nnz,) and self.val.shape == (self.nnz,)

    @property
    def tokens(self) -> float:
        return float(self.val.astype(np.float64).sum())

    def slice_docs(self, lo: int, hi: int) -> "CSC":
        a, b = int(self.colptr[lo]), int(self.colptr[hi])
        return CSC(hi - lo, self.V, self.colptr[lo:hi + 1] - a, self.rowidx[a:b], self.val[a:b])


def task_base(X: CSC, G: int) -> np.ndarray:
    base = np.zeros(X.nnz + 1, dtype=np.int64)
    lib().oracle_task_base(X.nnz, _p(X.val, c_float), G, _p(base, c_int64))
    return base


def run_pass(X: CSC, K, G, m, seed, pword, theta, phi, want_nwk=True, want_mu=False):
    """One pass of draws over X.  Returns (ndk, nwk or None, mu or None)."""
    ndk = np.zeros((X.D, K), dtype=np.uint32)
    nwk = np.zeros((X.V, K), dtype=np.uint32) if want_nwk else None
    mu = np.zeros(X.nnz, dtype=np.float32) if want_mu else None
    lib().oracle_pass(X.D, X.V, _p(X.colptr, c_int32), _p(X.rowidx, c_int32), _p(X.val, c_float),
                      K, G, m, seed, pword, _vp(theta), _vp(phi), _p(ndk, c_uint32), _vp(nwk), _vp(mu))
    return ndk, nwk, mu


def draw_tasks(X: CSC, K, G, m, seed, pword, theta, phi, task_ids) -> np.ndarray:
    ids = np.ascontiguousarray(task_ids, dtype=np.int64)
    out = np.zeros((ids.shape[0], K), dtype=np.uint32)
    lib().oracle_draw_tasks(X.D, _p(X.colptr, c_int32), _p(X.rowidx, c_int32), _p(X.val, c_float),
                            K, G, m, seed, pword, _vp(theta), _vp(phi), ids.shape[0],
                            _p(ids, c_int64), _p(out, c_uint32))
    return out


def theta_update(ndk, m, alpha) -> np.ndarray:
    D, K = ndk.shape
    theta = np.empty((D, K), dtype=np.float32)
    lib().oracle_theta_update(D, K, _p(ndk, c_uint32), m, c_float(alpha), _p(theta, c_float))
    return theta


def phi_update(nwk, m, beta, rho, phi) -> np.ndarray:
    V, K = nwk.shape
    out = np.zeros((V, K), dtype=np.float32) if phi is None else np.ascontiguousarray(phi, dtype=np.float32).copy()
    lib().oracle_phi_update(V, K, _p(nwk, c_uint32), m, c_float(beta), c_float(rho), _p(out, c_float))
    return out


# --------------------------------------------------------------------------- #
# Poisson form of the factored draw (the number of copies m is a positive real)
def expneg(y: float) -> float:
    return float(lib().oracle_expneg(c_float(y)))


def poisson_walk(rate: float, pm0: float, u: float) -> int:
    return int(lib().oracle_poisson_walk(c_float(rate), c_float(pm0), c_float(u)))


def poisson(lam: float, seed: int, tau: int, k: int, pword: int) -> int:
    return int(lib().oracle_poisson(c_float(lam), seed, tau, k, pword))


def draw_poisson(w, Nf: float, seed: int, tau: int, pword: int):
    """Independent Poisson counts of one task; returns (counts uint32[K], mu)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    counts = np.zeros(w.shape[0], dtype=np.uint32)
    mu = lib().oracle_draw_poisson(w.shape[0], _p(w, c_float), c_float(Nf), seed, tau, pword, _p(counts, c_uint32))
    return counts, float(mu)


def run_pass_poisson(X: CSC, K, G, m: float, seed, pword, theta, phi, want_nwk=True):
    ndk = np.zeros((X.D, K), dtype=np.uint32)
    nwk = np.zeros((X.V, K), dtype=np.uint32) if want_nwk else None
    lib().oracle_pass_poisson(X.D, X.V, _p(X.colptr, c_int32), _p(X.rowidx, c_int32), _p(X.val, c_float),
                              K, G, c_float(m), seed, pword, _vp(theta), _vp(phi), _p(ndk, c_uint32), _vp(nwk))
    return ndk, nwk


def draw_tasks_poisson(X: CSC, K, G, m: float, seed, pword, theta, phi, task_ids) -> np.ndarray:
    ids = np.ascontiguousarray(task_ids, dtype=np.int64)
    out = np.zeros((ids.shape[0], K), dtype=np.uint32)
    lib().oracle_draw_tasks_poisson(X.D, _p(X.colptr, c_int32), _p(X.rowidx, c_int32), _p(X.val, c_float),
                                    K, G, c_float(m), seed, pword, _vp(theta), _vp(phi), ids.shape[0],
                                    _p(ids, c_int64), _p(out, c_uint32))
    return out


def theta_update_real(ndk, m: float, alpha) -> np.ndarray:
    D, K = ndk.shape
    theta = np.empty((D, K), dtype=np.float32)
    lib().oracle_theta_update_real(D, K, _p(ndk, c_uint32), c_float(m), c_float(alpha), _p(theta, c_float))
    return theta


def phi_update_real(nwk, m: float, beta, rho, phi) -> np.ndarray:
    V, K = nwk.shape
    out = np.zeros((V, K), dtype=np.float32) if phi is None else np.ascontiguousarray(phi, dtype=np.float32).copy()
    lib().oracle_phi_update_real(V, K, _p(nwk, c_uint32), c_float(m), c_float(beta), c_float(rho), _p(out, c_float))
    return out


def flog(x: float) -> float:
    return float(lib().oracle_flog(c_float(x)))


def cos2pi(u: float) -> float:
    return float(lib().oracle_cos2pi(c_float(u)))


def normal(u1: float, u2: float) -> float:
    return float(lib().oracle_normal(c_float(u1), c_float(u2)))


def gamma(a: float, seed: int, row: int, k: int, pword: int) -> float:
    """One Gamma(a, 1) variable of the sampled parameter step (element (row, k) of its stream)."""
    return float(lib().oracle_gamma(c_float(a), seed, row, k, pword))


def theta_sample(ndk, m: float, alpha, seed: int, pword: int) -> np.ndarray:
    """theta_d ~ Dirichlet(n_dk + m*alpha), left unnormalised with mean n_dk/m + alpha."""
    D, K = ndk.shape
    theta = np.empty((D, K), dtype=np.float32)
    lib().oracle_theta_sample(D, K, _p(ndk, c_uint32), c_float(m), c_float(alpha), seed, pword, _p(theta, c_float))
    return theta


def phi_sample(nwk, m: float, beta, seed: int, pword: int) -> np.ndarray:
    """phi_k ~ Dirichlet over words (n_wk + m*beta), normalised over words."""
    V, K = nwk.shape
    phi = np.empty((V, K), dtype=np.float32)
    lib().oracle_phi_sample(V, K, _p(nwk, c_uint32), c_float(m), c_float(beta), seed, pword, _p(phi, c_float))
    return phi


def sddmm(X: CSC, theta, phi) -> np.ndarray:
    """mu[i] = sum_k theta[d][k] * phi[w][k] for every nonzero (the normaliser of Algorithm 3), in double."""
    theta = np.ascontiguousarray(theta, dtype=np.float32)
    phi = np.ascontiguousarray(phi, dtype=np.float32)
    mu = np.zeros(X.nnz, dtype=np.float64)
    lib().oracle_sddmm(X.D, _p(X.colptr, c_int32), _p(X.rowidx, c_int32), theta.shape[1],
                       _p(theta, c_float), _p(phi, c_float), _p(mu, c_double))
    return mu


def loglik_eval(X: CSC, theta, phi) -> float:
    K = theta.shape[1]
    return float(lib().oracle_loglik_eval(X.D, _p(X.colptr, c_int32), _p(X.rowidx, c_int32),
                                          _p(X.val, c_float), K, _p(theta, c_float), _p(phi, c_float)))


class OracleLDA:
    """SAME Gibbs LDA state advanced by the oracle, one pass at a time.

    ``t`` counts passes of the training stream: pass 0 is the random
    initialisation (uniform weights), every sweep or new minibatch takes the
    next index.  The held-out fold-in of :meth:`loglik` uses its own stream
    domain and restarts at pass 0 on every call.
    """

    def __init__(self, X: CSC, K: int, alpha: float, beta: float, seed: int, m0: int, G: int = 8):
        self.X, self.K, self.G = X, int(K), int(G)
        self.alpha, self.beta, self.seed = float(np.float32(alpha)), float(np.float32(beta)), int(seed)
        self.t = 0
        self.ndk, self.nwk, _ = run_pass(X, self.K, self.G, m0, self.seed, pass_word(self.t), None, None)
        self.theta = theta_update(self.ndk, m0, self.alpha)
        self.phi = phi_update(self.nwk, m0, self.beta, 1.0, None)
        self.t += 1

    def sweep(self, m: int, rho: float = 1.0):
        self.ndk, self.nwk, _ = run_pass(self.X, self.K, self.G, m, self.seed, pass_word(self.t),
                                         self.theta, self.phi)
        self.theta = theta_update(self.ndk, m, self.alpha)
        self.phi = phi_update(self.nwk, m, self.beta, rho, self.phi)
        self.t += 1

    def sweep_sampled(self, m: int):
        """One sweep whose parameter step draws theta and phi from their Dirichlet conditionals
        (Algorithm 2, third step) instead of taking their means."""
        self.ndk, self.nwk, _ = run_pass(self.X, self.K, self.G, m, self.seed, pass_word(self.t),
                                         self.theta, self.phi)
        self.theta = theta_sample(self.ndk, float(m), self.alpha, self.seed, pass_word(self.t, DOMAIN_THETA))
        self.phi = phi_sample(self.nwk, float(m), self.beta, self.seed, pass_word(self.t, DOMAIN_PHI))
        self.t += 1

    def sweep_poisson(self, m: float, rho: float = 1.0):
        """One sweep in the Poisson form (Algorithm 3 as printed): m may be any positive real."""
        m = float(np.float32(m))
        self.ndk, self.nwk = run_pass_poisson(self.X, self.K, self.G, m, self.seed, pass_word(self.t),
                                              self.theta, self.phi)
        self.theta = theta_update_real(self.ndk, m, self.alpha)
        self.phi = phi_update_real(self.nwk, m, self.beta, rho, self.phi)
        self.t += 1

    def set_batch(self, X: CSC, m_init: int):
        """New minibatch: phi is kept, theta of the new documents starts from a uniform-weight pass."""
        assert X.V == self.X.V
        self.X = X
        self.ndk, _, _ = run_pass(X, self.K, self.G, m_init, self.seed, pass_word(self.t), None, None,
                                  want_nwk=False)
        self.theta = theta_update(self.ndk, m_init, self.alpha)      # phi and n_wk stay as the last sweep left them
        self.t += 1

    def loglik(self, Xtest: CSC, foldin_sweeps: int, m_eval: int) -> float:
        p = 0
        ndk, _, _ = run_pass(Xtest, self.K, self.G, m_eval, self.seed, pass_word(p, DOMAIN_HELDOUT),
                             None, None, want_nwk=False)
        theta = theta_update(ndk, m_eval, self.alpha)
        for _ in range(foldin_sweeps):
            p += 1
            ndk, _, _ = run_pass(Xtest, self.K, self.G, m_eval, self.seed, pass_word(p, DOMAIN_HELDOUT),
                                 theta, self.phi, want_nwk=False)
            theta = theta_update(ndk, m_eval, self.alpha)
        return loglik_eval(Xtest, theta, self.phi)
