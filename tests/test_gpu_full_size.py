"""GPU checks at the benchmark's full size (news-shaped workload, K=256, m=100, the launch
configuration bench.py times): properties that hold at any size over the whole result, and
sampled outputs recomputed one by one by the CPU oracle.  The parameter state is a seeded
synthetic one (nothing computed by the GPU is fed to the oracle)."""
import numpy as np
import pytest
import torch

import oracle
from paper_1409_5402_amd import binding, schedule, synth

pytestmark = pytest.mark.gpu


def test_device_selftest():
    """Philox known answers on the device and the integer reciprocal against 1/x for all x < 2^24."""
    assert binding.selftest() == 0


@pytest.mark.timeout(900)
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


def _csc(c):
    return oracle.CSC(c.D, c.V, c.colptr.cpu().numpy(), c.rowidx.cpu().numpy(), c.val.cpu().numpy())


def _assert_counts_equal(g, o, what):
    ndk = g.get(binding.NDK)
    bad = np.flatnonzero((ndk != o.ndk).any(axis=1))
    assert bad.size == 0, f"{what}: n_dk differs in {bad.size} of {ndk.shape[0]} documents, first {bad[:5]}"
    nwk = g.get(binding.NWK)
    badw = np.flatnonzero((nwk != o.nwk).any(axis=1))
    assert badw.size == 0, f"{what}: n_wk differs in {badw.size} words, first {badw[:5]}"
    assert np.array_equal(g.get(binding.NK), o.nwk.sum(axis=0, dtype=np.uint64)), f"{what}: n_k differs"


@pytest.mark.timeout(900)
def test_news_full_size_one_sweep_every_element():
    """One sweep at m = 100 over the whole news-shaped matrix (60.6M nonzeros, K = 256) from a seeded concentrated
    state, then one from the flat state right after the initialisation (every task overflows its pair-list slot and
    goes on in chunks of the pool): both count matrices equal the oracle's in every element, theta and phi follow.
    The oracle needs some ten seconds per sweep on the machine's host cores."""
    dev = torch.device("cuda:0")
    p = synth.PRESETS["news"]
    K, m, alpha, beta, G = p["K"], p["m"], p["alpha"], p["beta"], binding.DEFAULT_TOKENS_PER_DRAW
    corpus = synth.preset("news", device=dev)
    train = corpus.slice_docs(0, corpus.D - corpus.D // 10)
    X = oracle.CSC(train.D, train.V, train.colptr.cpu().numpy(), train.rowidx.cpu().numpy(), train.val.cpu().numpy())
    g = binding.SameLDA(train.D, train.V, train.colptr, train.rowidx, train.val, K, alpha, beta,
                        seed=9, m0=1, tokens_per_draw=G)

    def check(theta, phi, what):
        pword = oracle.pass_word(g.pass_index)
        g.sweep(m)
        ndk_o, nwk_o, _ = oracle.run_pass(X, K, G, m, 9, pword, theta, phi)
        ndk = g.get(binding.NDK)
        bad = np.flatnonzero((ndk != ndk_o).any(axis=1))
        assert bad.size == 0, f"{what}: n_dk differs in {bad.size} documents, first {bad[:5]}"
        del ndk
        nwk = g.get(binding.NWK)
        bad = np.flatnonzero((nwk != nwk_o).any(axis=1))
        assert bad.size == 0, f"{what}: n_wk differs in {bad.size} words, first {bad[:5]}"
        np.testing.assert_allclose(g.get(binding.THETA), oracle.theta_update(ndk_o, m, alpha), rtol=1e-5, err_msg=what)
        np.testing.assert_allclose(g.get(binding.PHI), oracle.phi_update(nwk_o, m, beta, 1.0, None), rtol=1e-5, err_msg=what)

    # the flat state the library's own initialisation leaves (the oracle repeats the initial pass)
    ndk0, nwk0, _ = oracle.run_pass(X, K, G, 1, 9, oracle.pass_word(0), None, None)
    theta0, phi0 = oracle.theta_update(ndk0, 1, alpha), oracle.phi_update(nwk0, 1, beta, 1.0, None)
    assert np.array_equal(g.get(binding.NDK), ndk0) and np.array_equal(g.get(binding.NWK), nwk0)
    del ndk0, nwk0
    check(theta0, phi0, "first sweep after the initialisation")
    del theta0, phi0
    theta_t, phi_t = synth.state(train, K, alpha, beta, seed=126, zipf_s=1.1)
    g.set(binding.THETA, theta_t)
    g.set(binding.PHI, phi_t)
    check(theta_t.cpu().numpy(), phi_t.cpu().numpy(), "sweep from the seeded concentrated state")
    g.close()


@pytest.mark.timeout(900)
def test_medium_full_size_all_twenty_annealed_sweeps():
    """The medium workload at its real size (D=50,000, V=20,000, K=64; Zipf-skewed words) through all twenty
    sweeps of the linear schedule m = 1..20 (Section 6.1.3): the whole state against the oracle after every
    sweep, counts bit for bit, theta and phi to 1e-5."""
    p = synth.PRESETS["medium"]
    X = _csc(synth.preset("medium"))
    ms = schedule.linear(10.5, p["sweeps"])
    assert ms == list(range(1, 21)) and X.D == 50_000
    G = 32
    o = oracle.OracleLDA(X, p["K"], p["alpha"], p["beta"], seed=1, m0=ms[0], G=G)
    g = binding.SameLDA(X.D, X.V, X.colptr, X.rowidx, X.val, p["K"], p["alpha"], p["beta"], seed=1, m0=ms[0],
                        tokens_per_draw=G)
    _assert_counts_equal(g, o, "init")
    for s, m in enumerate(ms):
        o.sweep(m)
        g.sweep(m)
        print(f"medium sweep {s + 1} m={m}", flush=True)
        _assert_counts_equal(g, o, f"sweep {s + 1} m={m}")
    np.testing.assert_allclose(g.get(binding.THETA), o.theta, rtol=1e-5, atol=0)
    np.testing.assert_allclose(g.get(binding.PHI), o.phi, rtol=1e-5, atol=0)
    assert g.pass_index == o.t == 21
    g.close()


@pytest.mark.timeout(900)
def test_news_k1024_full_size_sampled_parity_and_conservation():
    """The many-topics workload at its real size (the news-shaped corpus, K=1024, m=100): sampled tasks
    recomputed one by one by the oracle, among them tasks of the most frequent words and the largest groups;
    one full-size sweep with per-document and per-word conservation and whole sampled documents and words."""
    dev = torch.device("cuda:0")
    p = synth.PRESETS["news_k1024"]
    K, m, alpha, beta, G = p["K"], p["m"], p["alpha"], p["beta"], binding.DEFAULT_TOKENS_PER_DRAW
    corpus = synth.preset("news_k1024", device=dev)
    train = corpus.slice_docs(0, corpus.D - corpus.D // 10)
    theta_t, phi_t = synth.state(train, K, alpha, beta, seed=223, zipf_s=1.1)
    g = binding.SameLDA(train.D, train.V, train.colptr, train.rowidx, train.val, K, alpha, beta,
                        seed=6, m0=1, tokens_per_draw=G)
    g.set(binding.THETA, theta_t)
    g.set(binding.PHI, phi_t)
    X = _csc(train)
    theta, phi = theta_t.cpu().numpy(), phi_t.cpu().numpy()
    del theta_t, phi_t
    pword = oracle.pass_word(g.pass_index)
    base = oracle.task_base(X, G)
    n_tasks = g.task_count
    assert n_tasks == int(base[-1])

    rng = np.random.default_rng(4)
    word_tokens = np.bincount(X.rowidx, weights=X.val.astype(np.float64), minlength=X.V).astype(np.int64)
    top_words = np.argsort(-word_tokens)[:3]
    nz_top = np.concatenate([np.flatnonzero(X.rowidx == w)[:150] for w in top_words])     # tasks of the most frequent words
    nz_big = np.argsort(-X.val)[:100]                                                     # the largest groups
    ids = np.unique(np.concatenate([rng.choice(n_tasks, 1500, replace=False), base[nz_top], base[nz_big],
                                    np.arange(0, 100), np.arange(n_tasks - 100, n_tasks)]))
    got = g.debug_draw(m, ids)
    ref = oracle.draw_tasks(X, K, G, m, 6, pword, theta, phi, ids)
    bad = np.flatnonzero((got != ref).any(axis=1))
    assert bad.size == 0, f"{bad.size} of {ids.size} sampled tasks differ, first task ids {ids[bad[:5]]}"

    g.sweep(m)
    print("news_k1024 sweep done", flush=True)
    ndk, nwk, nk = g.get(binding.NDK), g.get(binding.NWK), g.get(binding.NK)
    doc_tokens = np.add.reduceat(X.val.astype(np.int64), X.colptr[:-1].astype(np.int64)) * (np.diff(X.colptr) > 0)
    assert np.array_equal(ndk.sum(axis=1, dtype=np.int64), m * doc_tokens)
    assert np.array_equal(nwk.sum(axis=1, dtype=np.int64), m * word_tokens)
    assert np.array_equal(nk.astype(np.int64), nwk.sum(axis=0, dtype=np.int64))
    for d in [0, 5, 1234, X.D // 3, X.D - 1]:                    # whole documents
        t0, t1 = int(base[X.colptr[d]]), int(base[X.colptr[d + 1]])
        vec = oracle.draw_tasks(X, K, G, m, 6, pword, theta, phi, np.arange(t0, t1))
        assert np.array_equal(vec.sum(axis=0, dtype=np.int64), ndk[d].astype(np.int64)), d
    # whole words (rows of n_wk, which reach the matrix through the pair list and the reduce kernel): a frequent
    # word would need millions of draws, so words with a few hundred nonzeros are taken
    per_word = np.bincount(X.rowidx, minlength=X.V)
    for w in np.flatnonzero((per_word > 100) & (per_word < 400))[[0, 7, -1]]:
        nz = np.flatnonzero(X.rowidx == w)
        tids = np.concatenate([np.arange(base[i], base[i + 1]) for i in nz])
        vec = oracle.draw_tasks(X, K, G, m, 6, pword, theta, phi, tids)
        assert np.array_equal(vec.sum(axis=0, dtype=np.int64), nwk[w].astype(np.int64)), int(w)
    th = g.get(binding.THETA)
    rows = rng.choice(X.D, 100, replace=False)
    np.testing.assert_allclose(th[rows], ndk[rows] / m + alpha, rtol=1e-6)
    g.close()


@pytest.mark.timeout(900)
def test_abstract_stream_two_full_size_minibatches():
    """The streamed workload at its real minibatch size (100,000 documents, V=140,000, K=256): two minibatches,
    the second one staged on the library's second stream while the first is swept and then committed
    (Section 5.2), m from the geometric schedule and rho_t blending; the whole state against the oracle's
    set_batch / sweep sequence, counts bit for bit."""
    p = synth.PRESETS["abstracts_batch"]
    K, alpha, beta, G = p["K"], p["alpha"], p["beta"], 64
    batches = []
    for i in range(2):
        gen = dict(p["gen"]); gen["seed"] = 50 + i
        batches.append(_csc(synth.generate(**gen)))
    assert batches[0].D == 100_000 and batches[0].V == 140_000
    sched = schedule.geometric(1, 100, 80)
    steps = [(30, sched[30]), (70, sched[70])]                   # (minibatch number, m): m = 6 and m = 59
    o = oracle.OracleLDA(batches[0], K, alpha, beta, seed=17, m0=1, G=G)
    g = binding.SameLDA(batches[0].D, batches[0].V, batches[0].colptr, batches[0].rowidx, batches[0].val, K, alpha,
                        beta, seed=17, m0=1, tokens_per_draw=G)
    _assert_counts_equal(g, o, "init")
    t, m = steps[0]
    rho = float(np.float32(schedule.rho(t)))
    o.sweep(m, rho)
    g.sweep(m, rho)                                              # asynchronous: runs while the next minibatch is staged
    B = batches[1]
    pinned = [torch.from_numpy(a).pin_memory() for a in (B.colptr, B.rowidx, B.val)]
    g.stage_batch(B.D, *pinned, 1, 0)
    _assert_counts_equal(g, o, f"minibatch 0 m={m}")
    print("stream minibatch 0 done", flush=True)
    g.commit_batch()
    o.set_batch(B, 1)
    assert np.array_equal(g.get(binding.NDK), o.ndk)
    np.testing.assert_allclose(g.get(binding.PHI), o.phi, rtol=1e-5, atol=0)
    t, m = steps[1]
    rho = float(np.float32(schedule.rho(t)))
    o.sweep(m, rho)
    g.sweep(m, rho)
    _assert_counts_equal(g, o, f"minibatch 1 m={m}")
    np.testing.assert_allclose(g.get(binding.THETA), o.theta, rtol=1e-5, atol=0)
    np.testing.assert_allclose(g.get(binding.PHI), o.phi, rtol=1e-5, atol=0)
    assert g.pass_index == o.t
    g.close()


@pytest.mark.timeout(900)
def test_news_heldout_loglik_full_size():
    """Held-out per-word log-likelihood (Section 6.1.1) on the news workload's held-out tenth (30,000 documents,
    K=256, m=100, three fold-in sweeps) under a seeded topic-word matrix: within 1e-4 of the oracle's."""
    p = synth.PRESETS["news"]
    K, m, alpha, beta, G = p["K"], p["m"], p["alpha"], p["beta"], binding.DEFAULT_TOKENS_PER_DRAW
    corpus = synth.preset("news")
    test = _csc(corpus.slice_docs(corpus.D - corpus.D // 10, corpus.D))
    seedX = _csc(corpus.slice_docs(0, 50))                       # a handle needs a resident matrix: fifty documents
    _, phi_t = synth.state(corpus.slice_docs(0, 50), K, alpha, beta, seed=323, zipf_s=1.1)
    phi = phi_t.numpy()
    o = oracle.OracleLDA(seedX, K, alpha, beta, seed=8, m0=1, G=G)
    g = binding.SameLDA(seedX.D, seedX.V, seedX.colptr, seedX.rowidx, seedX.val, K, alpha, beta, seed=8, m0=1,
                        tokens_per_draw=G)
    o.phi = phi
    g.set(binding.PHI, phi)
    ll_g = g.loglik(test.D, test.colptr, test.rowidx, test.val, 3, m)
    ll_o = o.loglik(test, 3, m)
    print(f"held-out ll gpu {ll_g:.6f} oracle {ll_o:.6f}", flush=True)
    assert abs(ll_g - ll_o) <= 1e-4
    assert -12.0 < ll_o < -5.0
    g.close()
