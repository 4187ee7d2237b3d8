"""Mutation check of the oracle's pins (CPU only, about ten minutes: marked `slow` and skipped unless
SAME_LDA_SLOW=1 is set; `python tests/test_oracle_mutants.py` runs it by hand and prints every mutant).

One plausible mistake at a time (a dropped term, a wrong sign, index or operand) is planted in a COPY of
the oracle (oracle/same_lda_oracle.c or oracle/__init__.py) under a temporary directory; the pins of
tests/test_oracle_pins.py are run against the copy, and the mutants that no pin notices are listed.  The
mutant named in EXPECTED_SURVIVORS changes only which integers come out, not their distribution (the length
of a binomial piece): a build decision that no mathematical pin can see, expected to survive; every other
one must be caught.
"""
import os
import re
import shutil
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXPECTED_SURVIVORS = {"binom: piece length wrong"}

C_FILE, PY_FILE = "same_lda_oracle.c", "__init__.py"

# mistakes in the Python class that strings the steps together: (name, text in oracle/__init__.py, replacement)
PY_MUTS = [
 ("set_batch: phi recomputed from the uniform pass",
  "        self.ndk, _, _ = run_pass(X, self.K, self.G, m_init, self.seed, pass_word(self.t), None, None,\n                                  want_nwk=False)\n        self.theta = theta_update(self.ndk, m_init, self.alpha)",
  "        self.ndk, self.nwk, _ = run_pass(X, self.K, self.G, m_init, self.seed, pass_word(self.t), None, None)\n        self.phi = phi_update(self.nwk, m_init, self.beta, 1.0, None)\n        self.theta = theta_update(self.ndk, m_init, self.alpha)"),
 ("set_batch: pass index not advanced",
  "        self.theta = theta_update(self.ndk, m_init, self.alpha)      # phi and n_wk stay as the last sweep left them\n        self.t += 1",
  "        self.theta = theta_update(self.ndk, m_init, self.alpha)      # phi and n_wk stay as the last sweep left them"),
 ("set_batch: theta divided by the wrong m",
  "        self.theta = theta_update(self.ndk, m_init, self.alpha)      # phi",
  "        self.theta = theta_update(self.ndk, 1, self.alpha)      # phi"),
 ("set_batch: initial pass weighted by the old model",
  "pass_word(self.t), None, None,\n                                  want_nwk=False)\n        self.theta = theta_update(self.ndk, m_init",
  "pass_word(self.t), np.ones((X.D, self.K), np.float32), self.phi,\n                                  want_nwk=False)\n        self.theta = theta_update(self.ndk, m_init"),
 ("set_batch: the old minibatch stays resident", "        self.X = X\n        self.ndk, _, _ = run_pass(X,", "        self.ndk, _, _ = run_pass(X,"),
 ("sweep: blend ignored", "self.phi = phi_update(self.nwk, m, self.beta, rho, self.phi)\n        self.t += 1\n\n    def sweep_sampled",
  "self.phi = phi_update(self.nwk, m, self.beta, 1.0, self.phi)\n        self.t += 1\n\n    def sweep_sampled"),
 ("sweep: pass index not advanced", "self.phi = phi_update(self.nwk, m, self.beta, rho, self.phi)\n        self.t += 1\n\n    def sweep_sampled",
  "self.phi = phi_update(self.nwk, m, self.beta, rho, self.phi)\n\n    def sweep_sampled"),
 ("loglik: fold-in never updates theta", "                                 theta, self.phi, want_nwk=False)\n            theta = theta_update(ndk, m_eval, self.alpha)",
  "                                 theta, self.phi, want_nwk=False)"),
]

# (name, text in the oracle's C source, its replacement); the first occurrence is replaced
MUTS = [
 ("chain: the step's topic keeps only the top copy", "n += oracle_binom(R - 1u, q, seed, tau, step, pass);", "n += 0u * oracle_binom(R - 1u, q, seed, tau, step, pass);"),
 ("chain: binomial over all R copies", "n += oracle_binom(R - 1u, q, seed, tau, step, pass);", "n += oracle_binom(R, q, seed, tau, step, pass); if (n > R) n = R;"),
 ("chain: width over the whole range", "float q = width / y;", "float q = width / U;"),
 ("chain: width from the topic's upper end", "float width = y - prev;", "float width = P[k] - prev;"),
 ("chain: next range keeps the topic", "        U = prev;\n        top = k;", "        U = P[k];\n        top = k + 1;"),
 ("chain: R not reduced", "        counts[k] += n;\n        R -= n;", "        counts[k] += n;\n        R -= 1;"),
 ("chain: topic above the position", "while (k < top - 1 && !(P[k] >= y)) ++k;", "while (k < top - 1 && !(P[k] >= y)) ++k;\n        if (k < top - 1) ++k;"),
 ("chain: every step reuses step 0's uniforms", "float u = chain_uniform(seed, tau, step, 0, pass);", "float u = chain_uniform(seed, tau, 0, 0, pass);"),
 ("top: root of order R+1", "float z = a / (float)R;", "float z = a / (float)(R + 1u);"),
 ("top: no root taken", "float e = oracle_expneg(z);\n        if (e > 1.0f) e = 1.0f;", "float e = oracle_expneg(a);\n        if (e > 1.0f) e = 1.0f;"),
 ("top: single copy at the top end", "        y = U * u;\n    } else {", "        y = U;\n    } else {"),
 ("prefix: block sums restart", "        S = S + r;\n    }\n    return S;", "        S = r;\n    }\n    return S;"),
 ("prefix: running sum skips the block's first weight", "            r = r + w[k];\n            P[k] = S + r;", "            P[k] = S + r;\n            r = r + w[k];"),
 ("prefix: block length off", "return 4 * ((K + 127) / 128);", "return 4 * ((K + 127) / 128) + 4;"),
 ("binom: complement not undone", "return flip ? R - total : total;", "return total;"),
 ("binom: r = qq instead of qq/s", "float r = qq / s;", "float r = qq;"),
 ("binom: piece length wrong", "uint32_t L = single ? R : (uint32_t)(32.0f / qq);", "uint32_t L = single ? R : (uint32_t)(16.0f / qq) + 7u;"),
 ("binom: pieces share one uniform", "float u = chain_uniform(seed, tau, step, 1u + piece, pass);", "float u = chain_uniform(seed, tau, step, 1u, pass);"),
 ("binom: binomial reuses the position's uniform", "float u = chain_uniform(seed, tau, step, 1u + piece, pass);", "float u = chain_uniform(seed, tau, step, piece == 0 ? 0u : 1u + piece, pass);"),
 ("binom: zero-success probability from the rounded 1-qq", "float pm0 = oracle_expneg((float)n * lq);", "float pm0 = oracle_expneg((float)n * -oracle_flog(s));"),
 ("binom: zero-success probability ignores n", "float pm0 = oracle_expneg((float)n * lq);", "float pm0 = oracle_expneg(lq);"),
 ("log1m: denominator 1 - x", "float den = 2.0f - x;", "float den = 1.0f - x;"),
 ("log1m: series cut after t^3", "    p = p * z; p = p + 0.2f;\n", "    p = 0.2f;\n"),
 ("walk: n-x instead of n-x+1", "pm = pm * (float)(n - x + 1u);", "pm = pm * (float)(n - x);"),
 ("walk: starts cdf at 0", "float pm = pm0, cdf = pm0;\n    while (u > cdf && x < n) {", "float pm = pm0, cdf = 0.0f;\n    while (u > cdf && x < n) {"),
 ("chain stream: slot ignored", "return oracle_uniform_from_word(out[2u * (step & 1u) + slot]);", "return oracle_uniform_from_word(out[2u * (step & 1u)]);"),
 ("uniform: can be 0", "(2u * (x >> 9) + 1u)", "(2u * (x >> 9))"),
 ("stream: topic word index ignores k", "return oracle_uniform_from_word(out[k & 3u]);", "return oracle_uniform_from_word(out[0]);"),
 ("weights: phi row of wrong word", "phi ? phi + (size_t)word * K : NULL, w);\n                uint32_t ntask", "phi ? phi + (size_t)((word + 1) % V) * K : NULL, w);\n                uint32_t ntask"),
 ("weights: sum instead of product", "w[k] = theta_d[k] * phi_w[k];", "w[k] = theta_d[k] + phi_w[k];"),
 ("pass: counts go to wrong topic", "ndk[(size_t)d * K + k] += cnt[k];", "ndk[(size_t)d * K + (K - 1 - k)] += cnt[k];"),
 ("pass: N ignores group size", "oracle_draw(K, w, m * g, seed, (uint64_t)(base[i] + j), pass, cnt, scratch);\n                    if (mu", "oracle_draw(K, w, m, seed, (uint64_t)(base[i] + j), pass, cnt, scratch);\n                    if (mu"),
 ("update: theta multiplied by m", "float avg = (float)ndk[e] / mf;", "float avg = (float)ndk[e] * mf;"),
 ("update: alpha dropped", "theta[e] = avg + alpha;", "theta[e] = avg;"),
 ("update: V*beta -> beta", "float vbeta = (float)V * beta;", "float vbeta = beta;"),
 ("update: blend weights swapped", "float keep = one_minus_rho * phi[(size_t)w * K + k];\n                float add = rho * hat;", "float keep = rho * phi[(size_t)w * K + k];\n                float add = one_minus_rho * hat;"),
 ("update: nk over wrong axis", "for (int32_t w = 0; w < V; ++w) nk += nwk[(size_t)w * K + k];", "for (int32_t w = 0; w < V; ++w) nk += nwk[(size_t)w * K + (k + 1) % K];"),
 ("loglik: theta total not removed", "total += (double)val[i] * (log((double)S) - log_tsum);", "total += (double)val[i] * (log((double)S));"),
 ("loglik: unweighted by count", "total += (double)val[i] * (log((double)S) - log_tsum);\n            tokens += (double)val[i];", "total += (log((double)S) - log_tsum);\n            tokens += 1.0;"),
 ("poisson: rate ignores Nf", "float scaled = Nf * w[k];", "float scaled = w[k];"),
 ("poisson: one piece too few", "J = (uint32_t)(lambda / 32.0f) + 1u;\n        rate = lambda / (float)J;", "J = (uint32_t)(lambda / 32.0f) + 1u;\n        rate = lambda / (float)(J + 1u);"),
 ("poisson walk: divides by x+1", "float inv_x = 1.0f / (float)x;\n        pm = pm * rate;", "float inv_x = 1.0f / (float)(x + 1u);\n        pm = pm * rate;"),
 ("expneg: wrong log2e", "1.4426950408889634f", "1.4326950408889634f"),
 ("gamma: d = a", "float d = a1 - 0.333333343f;", "float d = a1;"),
 ("gamma: c from 3d", "float nine_d = 9.0f * d;", "float nine_d = 3.0f * d;"),
 ("gamma: accept test sign", "accept = lhs < rhs;", "accept = lhs > rhs;"),
 ("gamma: small shape boost uses 1/(a+1)", "y = y / a;", "y = y / a1;"),
 ("gamma: v squared not cubed", "float v = t * t;\n        v = v * t;", "float v = t * t;"),
 ("normal: sine instead of cosine quadrant 0", "case 0:  return cs;", "case 0:  return sn;"),
 ("flog: ln2 wrong", "0.693147182f", "0.683147182f"),
 ("theta_sample: not divided by m", "theta[(size_t)d * K + k] = g / mf;", "theta[(size_t)d * K + k] = g;"),
 ("theta_sample: prior alpha not m*alpha", "float prior = mf * alpha;", "float prior = alpha;"),
 ("phi_sample: normalised over topics of a word", "float den = (float)total;", "float den = 1.0f;"),
 ("tasks: one task too many per nonzero", "return (ci + (uint32_t)G - 1u) / (uint32_t)G;", "return ci / (uint32_t)G + 1u;"),
 ("sddmm: theta row of the wrong document", "const float* t = theta + (size_t)d * K;\n            const float* p = phi + (size_t)rowidx[i] * K;\n            double acc", "const float* t = theta + (size_t)((d + 1) % D) * K;\n            const float* p = phi + (size_t)rowidx[i] * K;\n            double acc"),
 ("sddmm: sum of squares of theta", "acc += (double)t[k] * (double)p[k];", "acc += (double)t[k] * (double)t[k];"),
 ("poisson: rate not normalised", "float lambda = scaled / mu;", "float lambda = scaled;"),
 ("poisson pass: copies ignore the group size", "float Nf = m * (float)g;", "float Nf = m;"),
 ("update: beta dropped from the numerator", "float num = avg + beta;", "float num = avg;"),
 ("loglik: inner product with phi of the wrong word", "const float* ph = phi + (size_t)rowidx[i] * K;\n            const float* th = theta + (size_t)d * K;", "const float* ph = phi + (size_t)rowidx[colptr[d]] * K;\n            const float* th = theta + (size_t)d * K;"),
 ("phi_sample: prior beta not m*beta", "float prior = mf * beta;", "float prior = beta;"),
 ("gamma: fallback boost uses the acceptance uniform", "float l = oracle_flog(oracle_uniform_from_word(out[3]));", "float l = oracle_flog(oracle_uniform_from_word(out[2]));"),
 ("normal: radius without the factor two", "float r2 = -2.0f * l;", "float r2 = -1.0f * l;"),
]


VB_FILE = "vb_estep.py"
VB_MUTS = [
 ("vb: beta normalised over the topics of a word", "digamma(l.sum(axis=0, keepdims=True))", "digamma(l.sum(axis=1, keepdims=True))"),
 ("vb: theta normalised over documents", "digamma(g.sum(axis=1, keepdims=True))", "digamma(g.sum(axis=0, keepdims=True))"),
 ("vb: counts multiplied by the normaliser", "((c / mu) @ B)", "((c * mu) @ B)"),
 ("vb: prior dropped", "g = alpha + a * ((c / mu) @ B) if hi > lo", "g = a * ((c / mu) @ B) if hi > lo"),
 ("vb: expectation of theta instead of exp E log", "a = np.exp(digamma(g) - digamma(g.sum()))", "a = g / g.sum()"),
 ("vb: counts ignored", "c = X.val[lo:hi].astype(np.float64)", "c = np.ones(hi - lo)"),
 ("vb: rows of beta of the wrong words", "B = b[words]", "B = b[(words + 1) % b.shape[0]]"),
]
PINS_OF = {VB_FILE: "tests/test_oracle_pins_vb.py"}


def run_mutant(fname: str, src: str, work: str, old: str, new: str):
    """Builds a tree with the mutated oracle under work/ and runs the pins there; returns (caught, first failure)."""
    shutil.rmtree(work, ignore_errors=True)
    os.makedirs(work)
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(work, "oracle"),
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    shutil.copytree(os.path.join(ROOT, "tests"), os.path.join(work, "tests"), ignore=shutil.ignore_patterns("__pycache__"))
    os.symlink(os.path.join(ROOT, "paper_1409_5402_amd"), os.path.join(work, "paper_1409_5402_amd"))
    with open(os.path.join(work, "oracle", fname), "w") as f:
        f.write(src.replace(old, new, 1))
    pins = PINS_OF.get(fname, "tests/test_oracle_pins.py")
    r = subprocess.run([sys.executable, "-m", "pytest", pins, "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=work, capture_output=True, text=True)
    m = re.search(r"FAILED " + re.escape(pins) + r"::(\S+)", r.stdout)
    return r.returncode != 0, (m.group(1) if m else "")


def check(verbose: bool):
    """Returns (survivors, stale): mutants no pin notices, and mutants whose text is no longer in the oracle."""
    base = tempfile.mkdtemp(prefix="oracle_mutants_")
    survivors, stale = [], []
    for fname, muts in ((C_FILE, MUTS), (PY_FILE, PY_MUTS), (VB_FILE, VB_MUTS)):
        src = open(os.path.join(ROOT, "oracle", fname)).read()
        for name, old, new in muts:
            if old not in src:
                stale.append(name)
                continue
            caught, first = run_mutant(fname, src, os.path.join(base, "w"), old, new)
            if verbose:
                print(("caught   " if caught else "SURVIVED ") + name + (f"  [{first}]" if first else ""), flush=True)
            if not caught:
                survivors.append(name)
    shutil.rmtree(base, ignore_errors=True)
    return survivors, stale


@pytest.mark.slow
@pytest.mark.skipif(os.environ.get("SAME_LDA_SLOW") != "1", reason="about ten minutes: set SAME_LDA_SLOW=1 to run")
def test_every_planted_mistake_is_noticed_by_a_pin():
    survivors, stale = check(verbose=False)
    assert not stale, f"the text of these mutants is no longer in the oracle: {stale}"
    assert sorted(set(survivors) - EXPECTED_SURVIVORS) == []


def test_mutant_texts_are_current():
    """Cheap guard, always run: every mutant still names text that is in the oracle's sources."""
    for fname, muts in ((C_FILE, MUTS), (PY_FILE, PY_MUTS), (VB_FILE, VB_MUTS)):
        src = open(os.path.join(ROOT, "oracle", fname)).read()
        missing = [name for name, old, _ in muts if old not in src]
        assert not missing, (fname, missing)


if __name__ == "__main__":
    survivors, stale = check(verbose=True)
    print("survivors:", survivors, "stale:", stale)
    unexpected = sorted(set(survivors) - EXPECTED_SURVIVORS)
    if unexpected or stale:
        sys.exit(f"no pin notices: {unexpected}; stale: {stale}")
