"""GPU checks at the benchmark's full size (news-shaped workload, K=256, m=100, the launch
configuration bench.py times): properties that hold at any size over the whole result, and
sampled outputs recomputed one by one by the CPU oracle.  The parameter state is a seeded
synthetic one (nothing computed by the GPU is fed to the oracle)."""
import numpy as np
import pytest
import torch

import oracle
from paper_1409_5402_amd import binding, synth

pytestmark = pytest.mark.gpu


def test_device_selftest():
    """Philox known answers on the device and the integer reciprocal against 1/x for all x < 2^24."""
    assert binding.selftest() == 0


def test_news_full_size_properties_and_sampled_parity():
    dev = torch.device("cuda:0")
    p = synth.PRESETS["news"]
    K, m, alpha, beta, G = p["K"], p["m"], p["alpha"], p["beta"], binding.DEFAULT_TOKENS_PER_DRAW
    corpus = synth.preset("news", device=dev)
    train = corpus.slice_docs(0, corpus.D - corpus.D // 10)
    theta_t, phi_t = synth.state(train, K, alpha, beta, seed=123, zipf_s=1.1)
    g = binding.SameLDA(train.D, train.V, train.colptr, train.rowidx, train.val, K, alpha, beta,
                        seed=5, m0=1, tokens_per_draw=G)
    g.set(binding.THETA, theta_t)
    g.set(binding.PHI, phi_t)
    X = oracle.CSC(train.D, train.V, train.colptr.cpu().numpy(), train.rowidx.cpu().numpy(), train.val.cpu().numpy())
    theta, phi = theta_t.cpu().numpy(), phi_t.cpu().numpy()
    pword = oracle.pass_word(g.pass_index)
    n_tasks = g.task_count
    base = oracle.task_base(X, G)
    assert n_tasks == int(base[-1])

    # sampled tasks, recomputed one by one by the oracle (including the most frequent words' large groups)
    rng = np.random.default_rng(0)
    ids = np.unique(np.concatenate([rng.choice(n_tasks, 3000, replace=False), np.arange(0, 200), np.arange(n_tasks - 200, n_tasks)]))
    got = g.debug_draw(m, ids)
    ref = oracle.draw_tasks(X, K, G, m, 5, pword, theta, phi, ids)
    assert np.array_equal(got, ref)

    # the same sampled tasks in the Poisson form (a non-integer m)
    got_p = g.debug_draw_poisson(37.5, ids[::4])
    ref_p = oracle.draw_tasks_poisson(X, K, G, 37.5, 5, pword, theta, phi, ids[::4])
    assert np.array_equal(got_p, ref_p)

    g.sweep(m)                                        # the full-size launch that bench.py times
    ndk, nwk, nk = g.get(binding.NDK), g.get(binding.NWK), g.get(binding.NK)
    # properties at full size: every document and every word keeps m times its tokens
    doc_tokens = np.add.reduceat(X.val.astype(np.int64), X.colptr[:-1].astype(np.int64)) * (np.diff(X.colptr) > 0)
    assert np.array_equal(ndk.sum(axis=1, dtype=np.int64), m * doc_tokens)
    word_tokens = np.bincount(X.rowidx, weights=X.val.astype(np.float64), minlength=X.V).astype(np.int64)
    assert np.array_equal(nwk.sum(axis=1, dtype=np.int64), m * word_tokens)
    assert np.array_equal(nk.astype(np.int64), nwk.sum(axis=0, dtype=np.int64))
    # sampled whole documents: n_dk rows from the oracle's task-by-task draws
    for d in [0, 1, 777, X.D // 2, X.D - 1]:
        t0, t1 = int(base[X.colptr[d]]), int(base[X.colptr[d + 1]])
        vec = oracle.draw_tasks(X, K, G, m, 5, pword, theta, phi, np.arange(t0, t1))
        assert np.array_equal(vec.sum(axis=0, dtype=np.int64), ndk[d].astype(np.int64)), d
    # the update at full size against its formula in double (sampled rows)
    th = g.get(binding.THETA)
    rows = rng.choice(X.D, 200, replace=False)
    np.testing.assert_allclose(th[rows], ndk[rows] / m + alpha, rtol=1e-6)
    ph = g.get(binding.PHI)
    wrows = rng.choice(X.V, 200, replace=False)
    np.testing.assert_allclose(ph[wrows], (nwk[wrows] / m + beta) / (nk.astype(np.float64) / m + X.V * beta), rtol=1e-5)

    # one full-size sweep in the Poisson form, from a second seeded state: both count matrices hold the same
    # copies, document totals are Poisson around m * tokens (checked in units of their standard deviation),
    # sampled documents match the oracle
    theta2_t, phi2_t = synth.state(train, K, alpha, beta, seed=124, zipf_s=1.1)
    g.set(binding.THETA, theta2_t)
    g.set(binding.PHI, phi2_t)
    theta2, phi2 = theta2_t.cpu().numpy(), phi2_t.cpu().numpy()
    pword2 = oracle.pass_word(g.pass_index)
    g.sweep_poisson(float(m))
    ndk, nwk, nk = g.get(binding.NDK), g.get(binding.NWK), g.get(binding.NK)
    assert ndk.sum(dtype=np.int64) == nwk.sum(dtype=np.int64) == int(nk.sum())
    tot = ndk.sum(axis=1, dtype=np.int64).astype(np.float64)
    z = (tot - m * doc_tokens) / np.sqrt(np.maximum(m * doc_tokens, 1.0))
    assert np.abs(z).max() < 6.5 and abs(z.mean()) < 0.02 and abs(z.std() - 1.0) < 0.02
    for d in [0, 777, X.D - 1]:
        t0, t1 = int(base[X.colptr[d]]), int(base[X.colptr[d + 1]])
        vec = oracle.draw_tasks_poisson(X, K, G, float(m), 5, pword2, theta2, phi2, np.arange(t0, t1))
        assert np.array_equal(vec.sum(axis=0, dtype=np.int64), ndk[d].astype(np.int64)), d

    # one full-size sweep with the sampled parameter step, from a third seeded state: sampled documents'
    # counts from the oracle's draws, their theta rows from the oracle's Gamma variables one by one;
    # phi is a probability vector over words for every topic
    theta3_t, phi3_t = synth.state(train, K, alpha, beta, seed=125, zipf_s=1.1)
    g.set(binding.THETA, theta3_t)
    g.set(binding.PHI, phi3_t)
    theta3, phi3 = theta3_t.cpu().numpy(), phi3_t.cpu().numpy()
    t3 = g.pass_index
    g.sweep_sampled(m)
    ndk, th, ph = g.get(binding.NDK), g.get(binding.THETA), g.get(binding.PHI)
    prior = np.float32(np.float32(m) * np.float32(alpha))
    for d in [0, 777, X.D - 1]:
        t0, t1 = int(base[X.colptr[d]]), int(base[X.colptr[d + 1]])
        vec = oracle.draw_tasks(X, K, G, m, 5, oracle.pass_word(t3), theta3, phi3, np.arange(t0, t1))
        n_d = vec.sum(axis=0, dtype=np.int64)
        assert np.array_equal(n_d, ndk[d].astype(np.int64)), d
        want = np.array([oracle.gamma(float(np.float32(n_d[k]) + prior), 5, d, k, oracle.pass_word(t3, oracle.DOMAIN_THETA))
                         for k in range(K)], np.float32) / np.float32(m)
        np.testing.assert_allclose(th[d], want, rtol=1e-5)
    assert np.all(np.isfinite(ph)) and ph.min() > 0
    np.testing.assert_allclose(ph.astype(np.float64).sum(axis=0), 1.0, atol=1e-4)
    g.close()
