"""GPU parity of the variational E-step (same_lda_vb_exp_elog_beta, same_lda_vb_estep) against its oracle in
double, element by element.  Tolerance 1e-5 relative: psi and exp are evaluated in double on both sides; the
kernel's products and sums over topics and nonzeros are binary32 (a few hundred terms of one sign: relative
error of some 1e-7 per iteration).  The library stores a row of b divided by its largest entry and returns the
logarithm of the normaliser; the oracle keeps the plain definitions, so b and mu are compared through their
logarithms (absolute 1e-5 relative to magnitudes of 2 to 200)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import vb_estep
from helpers import corpus_to_csc, csc_from_dense
from paper_1409_5402_amd import binding, synth

pytestmark = pytest.mark.gpu
RTOL = 1e-5
DEV = torch.device("cuda:0")


def toy(seed, D=37, V=53, density=0.35, cmax=12):
    rng = np.random.default_rng(seed)
    counts = rng.integers(1, cmax + 1, size=(D, V)) * (rng.uniform(size=(D, V)) < density)
    counts[2, :] = 0
    counts[D - 1, :] = 0
    return csc_from_dense(counts)


def check_b(b, shift, b_o):
    """log(b) + shift against log of the oracle's b where b is a binary32 number; where it underflowed the oracle's
    entry lies at least e^-87 below its row's largest."""
    with np.errstate(divide="ignore"):
        log_o = np.log(b_o)                                   # -inf where even the double underflowed
    top = log_o.max(axis=1)
    np.testing.assert_allclose(shift, top, rtol=RTOL, atol=1e-6)
    assert np.all(b.max(axis=1) == 1.0)
    pos = b > 1e-30
    np.testing.assert_allclose(np.log(b[pos].astype(np.float64)) + np.broadcast_to(shift[:, None], b.shape)[pos],
                               log_o[pos], rtol=RTOL, atol=2e-5)
    assert np.all((log_o - top[:, None])[~pos] < -69.0)


def run_both(X, K, alpha, iters, lam, g0):
    g = binding.SameLDA(X.D, X.V, X.colptr, X.rowidx, X.val, K, 0.1, 0.01, seed=1, m0=1)
    lam_t = torch.from_numpy(lam.astype(np.float32)).to(DEV)
    b_t = torch.empty_like(lam_t)
    sh_t = torch.empty(X.V, dtype=torch.float32, device=DEV)
    g.vb_exp_elog_beta(lam_t, b_t, sh_t)
    gam_t = torch.from_numpy(g0.astype(np.float32)).to(DEV)
    lmu_t = torch.full((X.rowidx.shape[0],), 7.0, dtype=torch.float32, device=DEV)
    g.vb_estep(b_t, sh_t, alpha, iters, gam_t, lmu_t)
    g.synchronize()
    b_o = vb_estep.exp_elog_beta(lam.astype(np.float32))
    g_o, mu_o = vb_estep.estep(X, b_o, alpha, iters, g0.astype(np.float32))
    check_b(b_t.cpu().numpy(), sh_t.cpu().numpy(), b_o)
    out = (gam_t.cpu().numpy(), lmu_t.cpu().numpy(), g_o, np.log(mu_o))
    g.close()
    return out


@pytest.mark.parametrize("K", [1, 3, 40, 64, 256, 300, 511, 1000, 1028, 2048])
@pytest.mark.parametrize("iters", [1, 4])
def test_estep_matches_the_oracle(K, iters):
    """K = 1, K not a multiple of 4 (the LDS path), one to eight 256-topic chunks per lane with a ragged last one;
    documents with an odd and an even number of nonzeros and without any."""
    X = toy(seed=K)
    rng = np.random.default_rng(100 + K)
    lam = rng.gamma(0.5, 1.0, size=(X.V, K)) + 1e-3          # exp E[log beta] of the small ones is far below binary32
    g0 = rng.gamma(2.0, 1.0, size=(X.D, K)) + 0.05
    gam, lmu, g_o, lmu_o = run_both(X, K, 0.3, iters, lam, g0)
    np.testing.assert_allclose(gam, g_o, rtol=RTOL)
    np.testing.assert_allclose(lmu, lmu_o, rtol=RTOL, atol=1e-5)
    np.testing.assert_allclose(gam[2], 0.3, rtol=1e-6)              # an empty document keeps the prior


def test_estep_medium_shape_slice_converges_like_the_oracle():
    """2,000 documents of the medium shape (V = 20k, K = 64), a concentrated lambda, ten iterations from gamma = 1."""
    p = synth.PRESETS["medium"]
    c = synth.preset("medium")
    X = corpus_to_csc(c.slice_docs(0, 2000))
    _, phi = synth.state(c.slice_docs(0, 2000), p["K"], p["alpha"], p["beta"], seed=5, zipf_s=1.1)
    lam = 0.01 + np.asarray(phi.cpu() if hasattr(phi, "cpu") else phi, np.float64) * 5000.0
    g0 = np.ones((X.D, p["K"]))
    gam, lmu, g_o, lmu_o = run_both(X, p["K"], 0.1, 10, lam, g0)
    np.testing.assert_allclose(gam, g_o, rtol=RTOL)
    np.testing.assert_allclose(lmu, lmu_o, rtol=RTOL, atol=1e-5)


def test_estep_errors_and_no_ops():
    X = toy(seed=3)
    g = binding.SameLDA(X.D, X.V, X.colptr, X.rowidx, X.val, 8, 0.1, 0.01, seed=1, m0=1)
    b = torch.ones((X.V, 8), dtype=torch.float32, device=DEV)
    gam = torch.full((X.D, 8), 2.0, dtype=torch.float32, device=DEV)
    g.vb_estep(b, None, 0.5, 0, gam)                                 # zero iterations: untouched
    g.synchronize()
    assert torch.all(gam == 2.0)
    with pytest.raises(binding.SameLdaError):
        g.vb_estep(b, None, 0.0, 1, gam)
    with pytest.raises(binding.SameLdaError):
        g.vb_estep(b, None, 0.5, -1, gam)
    g.close()


@pytest.mark.timeout(900)
def test_estep_news_full_size_sampled_documents_and_row_sums():
    """The news-shaped matrix at full size (270k documents, K = 256), five iterations: every document's gamma sums to
    K alpha + its tokens; 1,500 documents from the start, the middle and the end of the matrix against the oracle."""
    p = synth.PRESETS["news"]
    K = p["K"]
    c = synth.preset("news", device=DEV)
    train = c.slice_docs(0, c.D - c.D // 10)
    _, phi = synth.state(train, K, p["alpha"], p["beta"], seed=123, zipf_s=1.1)
    lam_t = (0.01 + phi.to(DEV).float() * (float(train.val.sum()) / K)).contiguous()
    g = binding.SameLDA(train.D, train.V, train.colptr, train.rowidx, train.val, K, p["alpha"], p["beta"], seed=2, m0=1)
    b_t = torch.empty_like(lam_t)
    sh_t = torch.empty(train.V, dtype=torch.float32, device=DEV)
    g.vb_exp_elog_beta(lam_t, b_t, sh_t)
    gam_t = torch.ones((train.D, K), dtype=torch.float32, device=DEV)
    lmu_t = torch.empty(train.nnz, dtype=torch.float32, device=DEV)
    alpha, iters = 0.1, 5
    g.vb_estep(b_t, sh_t, alpha, iters, gam_t, lmu_t)
    g.synchronize()
    colptr = train.colptr.cpu().numpy().astype(np.int64)
    val = train.val.cpu().numpy()
    tokens = np.add.reduceat(np.concatenate([val, [0.0]]).astype(np.float64), colptr[:-1])
    tokens[colptr[:-1] == colptr[1:]] = 0.0
    gam = gam_t.cpu().numpy()
    np.testing.assert_allclose(gam.sum(axis=1, dtype=np.float64), K * alpha + tokens, rtol=2e-5)
    lam = lam_t.cpu().numpy()
    b_o = vb_estep.exp_elog_beta(lam)
    check_b(b_t.cpu().numpy()[::97], sh_t.cpu().numpy()[::97], b_o[::97])
    lmu = lmu_t.cpu().numpy()
    for lo in (0, train.D // 2, train.D - 500):
        sl = train.slice_docs(lo, lo + 500)
        Xs = corpus_to_csc(sl)
        g_o, mu_o = vb_estep.estep(Xs, b_o, alpha, iters, np.ones((500, K)))
        np.testing.assert_allclose(gam[lo:lo + 500], g_o, rtol=RTOL)
        np.testing.assert_allclose(lmu[colptr[lo]:colptr[lo + 500]], np.log(mu_o), rtol=RTOL, atol=1e-5)
    g.close()
