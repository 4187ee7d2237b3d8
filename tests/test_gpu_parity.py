"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Integer count matrices must be bit-exact; theta/phi within 1e-5 relative (they are in fact
expected to be identical, both sides rounding every step once); held-out log-likelihood within
1e-4 absolute.  Inputs are seeded and synthetic; nothing here feeds GPU results to the oracle.
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import corpus_to_csc, csc_from_dense
from paper_1409_5402_amd import binding, schedule, synth

pytestmark = pytest.mark.gpu

RTOL = 1e-5          # accumulated fp32 theta / phi
LL_ATOL = 1e-4       # held-out per-word log-likelihood


def make_gpu(X: oracle.CSC, K, alpha, beta, seed, m0, G, on_device=False):
    if on_device:
        dev = torch.device("cuda:0")
        return binding.SameLDA(X.D, X.V, torch.from_numpy(X.colptr).to(dev), torch.from_numpy(X.rowidx).to(dev),
                               torch.from_numpy(X.val).to(dev), K, alpha, beta, seed, m0, G)
    return binding.SameLDA(X.D, X.V, X.colptr, X.rowidx, X.val, K, alpha, beta, seed, m0, G)


def assert_state_equal(g: binding.SameLDA, o: oracle.OracleLDA, what=""):
    ndk, nwk = g.get(binding.NDK), g.get(binding.NWK)
    bad_d = np.flatnonzero((ndk != o.ndk).any(axis=1))
    assert bad_d.size == 0, f"{what}: n_dk differs in {bad_d.size} documents, first {bad_d[:5]}"
    if o.nwk is not None:
        assert np.array_equal(nwk, o.nwk), f"{what}: n_wk differs"
        assert np.array_equal(g.get(binding.NK), o.nwk.sum(axis=0, dtype=np.uint64)), f"{what}: n_k differs"
    np.testing.assert_allclose(g.get(binding.THETA), o.theta, rtol=RTOL, atol=0, err_msg=what)
    np.testing.assert_allclose(g.get(binding.PHI), o.phi, rtol=RTOL, atol=0, err_msg=what)


def toy(seed, D, V, density, cmax, empty_doc=True):
    rng = np.random.default_rng(seed)
    counts = rng.integers(1, cmax + 1, size=(D, V)) * (rng.uniform(size=(D, V)) < density)
    if empty_doc and D > 3:
        counts[2, :] = 0
        counts[D - 1, :] = 0
    if V > 5:
        counts[:, 4] = 0
    return csc_from_dense(counts)


def test_tiny_config_ten_sweeps_bit_exact():
    """Tiny workload: D=1000, V=2000, K=16, m=10 fixed, 10 sweeps; every sweep compared in full."""
    p = synth.PRESETS["tiny"]
    X = corpus_to_csc(synth.preset("tiny"))
    o = oracle.OracleLDA(X, p["K"], p["alpha"], p["beta"], seed=0, m0=p["m"], G=8)
    g = make_gpu(X, p["K"], p["alpha"], p["beta"], 0, p["m"], 8)
    assert g.task_count == int(oracle.task_base(X, 8)[-1])
    assert_state_equal(g, o, "init")
    for s in range(p["sweeps"]):
        o.sweep(p["m"])
        g.sweep(p["m"])
        assert_state_equal(g, o, f"sweep {s + 1}")
    assert g.pass_index == o.t == 11
    g.close()


@pytest.mark.parametrize("K", [1, 2, 3, 5, 16, 17, 40, 64, 100, 256, 300, 512, 516, 640, 768, 1000])
def test_topic_counts_incl_ragged_K(K):
    """K not a multiple of 4 or 16, K=1; blocks of topics read in one batch of loads (up to 256, 512) and in
    three, five, three and two batches of one, one, two and four loads (300, 516 and 640, 768, 1000); a last block
    that is partly or wholly past K; ragged last thread block; empty docs."""
    X = toy(seed=K, D=37, V=53, density=0.35, cmax=12)
    m = 7
    o = oracle.OracleLDA(X, K, 0.2, 0.01, seed=99, m0=m, G=4)
    g = make_gpu(X, K, 0.2, 0.01, 99, m, 4)
    assert_state_equal(g, o, "init")
    for s in range(3):
        o.sweep(m); g.sweep(m)
        assert_state_equal(g, o, f"K={K} sweep {s + 1}")
    g.close()


@pytest.mark.parametrize("G,m", [(1, 1), (1, 30), (2, 100), (8, 100), (1000, 100), (1000, 500), (3, 1000)])
def test_group_sizes_and_copy_counts(G, m):
    """tokens_per_draw from 1 (the per-token multinomial of Section 4) to 'whole nonzero'; m from 1 to 1000
    (large m*c forces several binomial pieces and the complement branch)."""
    X = toy(seed=5, D=60, V=40, density=0.3, cmax=40)
    K = 24
    o = oracle.OracleLDA(X, K, 0.1, 0.01, seed=3, m0=m, G=G)
    g = make_gpu(X, K, 0.1, 0.01, 3, m, G, on_device=True)
    assert_state_equal(g, o, "init")
    for s in range(2):
        o.sweep(m); g.sweep(m)
        assert_state_equal(g, o, f"G={G} m={m} sweep {s + 1}")
    g.close()


def test_word_counts_through_the_pair_list():
    """Twelve words, each in nearly every document with counts up to 30: every task has a slot in the word-ordered
    pair list, a word's slots run over several chunks of the reduce kernel and a chunk holds several words; the
    uniform start (many nonzero topics per task) fills slots beyond their 15 pairs."""
    rng = np.random.default_rng(11)
    counts = rng.integers(1, 31, size=(700, 12)) * (rng.uniform(size=(700, 12)) < 0.9)
    X = csc_from_dense(counts)
    K, m = 48, 40
    o = oracle.OracleLDA(X, K, 0.5, 0.05, seed=21, m0=m, G=4)
    g = make_gpu(X, K, 0.5, 0.05, 21, m, 4, on_device=True)
    assert_state_equal(g, o, "init")
    for s in range(3):
        o.sweep(m); g.sweep(m)
        assert_state_equal(g, o, f"sweep {s + 1}")
    g.close()


def test_full_slots_continue_in_chunks_or_fall_back():
    """A flat start with 100 copies per token and 64 topics: most tasks place far more than the 15 pairs of a slot.
    The pairs beyond go to chunks of the pool (chains of up to four), and to the word rows themselves once the pool is
    used up.  Whatever the pool's size - all of it, nothing, one batch and a bit, about a third of what the sweep
    needs - the counts are those of the oracle."""
    rng = np.random.default_rng(12)
    counts = rng.integers(1, 31, size=(700, 12)) * (rng.uniform(size=(700, 12)) < 0.9)
    X = csc_from_dense(counts)
    K, m = 64, 100
    o = oracle.OracleLDA(X, K, 0.5, 0.05, seed=22, m0=1, G=4)
    gs = []
    for limit in (-1, 0, 300, 30000):
        g = make_gpu(X, K, 0.5, 0.05, 22, 1, 4, on_device=True)
        allocated = g.debug_chunk_limit(-1)
        assert allocated >= g.task_count * 4, "every task of this matrix has a slot and may need four chunks"
        assert g.debug_chunk_limit(limit) == (allocated if limit < 0 else limit)
        gs.append((limit, g))
    for s in range(3):
        o.sweep(m)
        for limit, g in gs:
            g.sweep(m)
            assert_state_equal(g, o, f"sweep {s + 1}, chunk limit {limit}")
    for _, g in gs:
        g.close()


def test_annealed_medium_shape():
    """Medium workload shape at reduced document count: K=64, Zipf word skew, m annealed linearly 1..20."""
    p = synth.PRESETS["medium"]
    X = corpus_to_csc(synth.preset("medium", scale=0.04))          # 2000 documents, V=20000
    ms = schedule.linear(10.5, 20)
    assert ms[0] == 1 and ms[-1] == 20
    o = oracle.OracleLDA(X, p["K"], p["alpha"], p["beta"], seed=1, m0=ms[0], G=8)
    g = make_gpu(X, p["K"], p["alpha"], p["beta"], 1, ms[0], 8)
    assert_state_equal(g, o, "init")
    for s, m in enumerate(ms[:8]):
        o.sweep(m); g.sweep(m)
        assert_state_equal(g, o, f"sweep {s + 1} m={m}")
    g.close()


def test_news_shape_slice_k256_m100():
    """News workload shape (K=256, m=100, alpha=50/K, Zipf 1.1, log-normal lengths) on a 600-document slice
    with the full 100k vocabulary: spans many thread blocks, checkpoint blocks and a ragged tail."""
    p = synth.PRESETS["news"]
    X = corpus_to_csc(synth.preset("news", scale=0.002))
    o = oracle.OracleLDA(X, p["K"], p["alpha"], p["beta"], seed=7, m0=p["m"], G=8)
    g = make_gpu(X, p["K"], p["alpha"], p["beta"], 7, p["m"], 8)
    assert_state_equal(g, o, "init")
    for s in range(3):
        o.sweep(p["m"]); g.sweep(p["m"])
        assert_state_equal(g, o, f"sweep {s + 1}")
    g.close()


def test_minibatch_blend_and_new_batch():
    """rho < 1 blending (Algorithm 3, last step) and a second minibatch with phi kept (Section 5.2)."""
    Xa = toy(seed=11, D=50, V=64, density=0.3, cmax=6)
    Xb = toy(seed=12, D=33, V=64, density=0.4, cmax=6, empty_doc=False)
    K = 12
    o = oracle.OracleLDA(Xa, K, 0.1, 0.01, seed=5, m0=4, G=8)
    g = make_gpu(Xa, K, 0.1, 0.01, 5, 4, 8)
    for t, m in enumerate([4, 8, 16]):
        rho = float(np.float32(schedule.rho(t + 1)))
        o.sweep(m, rho); g.sweep(m, rho)
        assert_state_equal(g, o, f"batch a sweep {t}")
    o.set_batch(Xb, 16); g.set_batch(Xb.D, Xb.colptr, Xb.rowidx, Xb.val, 16)
    assert np.array_equal(g.get(binding.NDK), o.ndk)
    np.testing.assert_allclose(g.get(binding.THETA), o.theta, rtol=RTOL)
    np.testing.assert_allclose(g.get(binding.PHI), o.phi, rtol=RTOL)
    rho = float(np.float32(schedule.rho(5)))
    o.sweep(16, rho); g.sweep(16, rho)
    assert_state_equal(g, o, "batch b sweep")
    g.close()


def test_debug_draw_matches_oracle_tasks_and_next_sweep():
    X = toy(seed=21, D=40, V=30, density=0.4, cmax=20)
    K, m, G = 32, 50, 4
    o = oracle.OracleLDA(X, K, 0.1, 0.01, seed=8, m0=m, G=G)
    g = make_gpu(X, K, 0.1, 0.01, 8, m, G)
    o.sweep(m); g.sweep(m)
    n_tasks = g.task_count
    ids = np.random.default_rng(0).choice(n_tasks, size=min(n_tasks, 500), replace=False)
    got = g.debug_draw(m, ids)
    ref = oracle.draw_tasks(X, K, G, m, 8, oracle.pass_word(o.t), o.theta, o.phi, ids)
    assert np.array_equal(got, ref)
    assert np.all(got.sum(axis=1) % m == 0)
    o.sweep(m); g.sweep(m)                      # the hook must not have changed the state
    assert_state_equal(g, o, "after debug_draw")
    g.close()


def test_heldout_loglik():
    c = synth.generate(D=500, V=400, K=6, alpha=0.1, beta=0.05, seed=3, mean_len=80.0)
    X = corpus_to_csc(c)
    train, test = X.slice_docs(0, 450), X.slice_docs(450, 500)
    o = oracle.OracleLDA(train, 6, 0.1, 0.05, seed=4, m0=10, G=8)
    g = make_gpu(train, 6, 0.1, 0.05, 4, 10, 8)
    for _ in range(5):
        o.sweep(10); g.sweep(10)
    ll_o = o.loglik(test, 3, 10)
    ll_g = g.loglik(test.D, test.colptr, test.rowidx, test.val, 3, 10)
    assert abs(ll_g - ll_o) <= LL_ATOL
    assert_state_equal(g, o, "loglik must not disturb the training state")
    # K = 1 closed form: ll = sum_w tok_test(w) log phi_w / tokens_test
    g1 = make_gpu(train, 1, 0.1, 0.05, 4, 10, 8)
    phi = g1.get(binding.PHI)[:, 0].astype(np.float64)
    tok_t = np.zeros(X.V); np.add.at(tok_t, test.rowidx, test.val)
    ref = float((tok_t * np.log(phi)).sum() / tok_t.sum())
    assert abs(g1.loglik(test.D, test.colptr, test.rowidx, test.val, 2, 10) - ref) <= LL_ATOL
    g.close(); g1.close()


def test_set_state_and_resume_is_bit_identical():
    """theta, phi and the pass index restore a run exactly (the stream is counter-based)."""
    X = toy(seed=31, D=30, V=40, density=0.4, cmax=9)
    K, m = 20, 25
    g = make_gpu(X, K, 0.1, 0.01, 6, m, 8)
    g.sweep(m)
    theta, phi, t = g.get(binding.THETA), g.get(binding.PHI), g.pass_index
    g.sweep(m)
    want = g.get(binding.NWK)
    g2 = make_gpu(X, K, 0.1, 0.01, 6, m, 8)
    g2.set(binding.THETA, theta); g2.set(binding.PHI, phi); g2.pass_index = t
    g2.sweep(m)
    assert np.array_equal(g2.get(binding.NWK), want)
    g.close(); g2.close()


def test_large_topic_totals_on_device():
    """Topic totals beyond 2^24 (float conversion of 64-bit sums) and phi from oracle-side counts."""
    X = csc_from_dense(np.array([[60000, 50000, 3], [40000, 1, 70000]]))
    K, m = 2, 200                                # totals up to 4.4e7 > 2^24
    o = oracle.OracleLDA(X, K, 0.1, 0.01, seed=2, m0=m, G=100000)
    g = make_gpu(X, K, 0.1, 0.01, 2, m, 100000)
    assert_state_equal(g, o, "init")
    o.sweep(m); g.sweep(m)
    assert_state_equal(g, o, "sweep")
    g.close()


def test_errors_are_reported_not_crashes():
    X = toy(seed=1, D=5, V=8, density=0.5, cmax=3, empty_doc=False)
    with pytest.raises(binding.SameLdaError) as e:
        binding.SameLDA(X.D, X.V, X.colptr, X.rowidx, X.val, 0, 0.1, 0.01, 1, 1, 8)
    assert e.value.code == -1
    bad = X.rowidx.copy(); bad[0] = 99
    with pytest.raises(binding.SameLdaError) as e:
        binding.SameLDA(X.D, X.V, X.colptr, bad, X.val, 4, 0.1, 0.01, 1, 1, 8)
    assert e.value.code == -2
    badv = X.val.copy(); badv[1] = 1.5
    with pytest.raises(binding.SameLdaError) as e:
        binding.SameLDA(X.D, X.V, X.colptr, X.rowidx, badv, 4, 0.1, 0.01, 1, 1, 8)
    assert e.value.code == -2
    g = make_gpu(X, 4, 0.1, 0.01, 1, 1, 8)
    with pytest.raises(binding.SameLdaError):
        g.sweep(0)
    with pytest.raises(binding.SameLdaError):
        g.sweep(1, 0.0)
    g.sweep(1)
    g.close()


def test_accumulator_range_guard():
    """The count matrices are 32-bit: a sweep whose m times the tokens of one word or one document would not fit is
    refused, and the message names the word or document; one copy less per token is accepted and conserved."""
    X = oracle.CSC(2, 1, np.array([0, 1, 2], np.int32), np.zeros(2, np.int32), np.array([8e6, 8e6], np.float32))
    g = make_gpu(X, 2, 0.1, 0.01, 1, 1, 1000)              # the word holds 1.6e7 tokens: m = 268 fits, 269 does not
    g.sweep(268)
    assert int(g.get(binding.NWK).sum(dtype=np.int64)) == 268 * 16_000_000
    assert np.array_equal(g.get(binding.NDK).sum(axis=1, dtype=np.int64), [268 * 8_000_000] * 2)
    with pytest.raises(binding.SameLdaError) as e:
        g.sweep(269)
    assert e.value.code == -2 and "word 0" in str(e.value)
    with pytest.raises(binding.SameLdaError) as e:
        g.sweep_poisson(268.0)                              # a Poisson total may exceed its mean
    assert e.value.code == -2
    g.sweep_poisson(250.0)
    g.synchronize()
    g.close()
    # one document of two words: the document is the first to overflow
    X = oracle.CSC(1, 2, np.array([0, 2], np.int32), np.array([0, 1], np.int32), np.array([8e6, 8e6], np.float32))
    g = make_gpu(X, 2, 0.1, 0.01, 1, 1, 1000)
    with pytest.raises(binding.SameLdaError) as e:
        g.sweep(269)
    assert e.value.code == -2 and "document 0" in str(e.value)
    with pytest.raises(binding.SameLdaError) as e:
        g.loglik(X.D, X.colptr, X.rowidx, X.val, 1, 300)   # held-out matrices are checked too
    assert e.value.code == -2
    g.close()


def test_empty_matrix():
    X = oracle.CSC(3, 10, np.zeros(4, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
    g = make_gpu(X, 4, 0.1, 0.01, 1, 5, 8)
    g.sweep(5)
    assert g.get(binding.NDK).sum() == 0
    np.testing.assert_allclose(g.get(binding.THETA), 0.1, rtol=1e-6)
    np.testing.assert_allclose(g.get(binding.PHI), 0.1, rtol=1e-6)       # beta / (V * beta)
    g.close()


@pytest.mark.parametrize("K", [1024, 2048])
def test_many_topics_news_shape(K):
    """K=1024 (the many-topics workload) and the largest supported K: above K=512 the high bits of a queued
    topic live in a register beside the queue, and the checkpoint area grows; news-shaped slice, m=100."""
    X = corpus_to_csc(synth.preset("news_k1024", scale=0.0004))
    alpha = 50.0 / K
    o = oracle.OracleLDA(X, K, alpha, 0.01, seed=11, m0=1, G=32)
    g = make_gpu(X, K, alpha, 0.01, 11, 1, 32, on_device=True)
    assert_state_equal(g, o, "init")
    for s, m in enumerate([1, 100, 100]):
        o.sweep(m); g.sweep(m)
        assert_state_equal(g, o, f"K={K} sweep {s + 1} m={m}")
    g.close()


def test_streamed_minibatches_abstract_shape():
    """Abstract-collection shape (V=140k, Poisson 90, Zipf 1.05): three minibatches streamed through
    same_lda_set_batch with a geometric m schedule and rho_t blending; K reduced to keep the oracle fast."""
    c = synth.generate(D=900, V=140_000, K=64, alpha=0.1, beta=0.01, seed=4, length="poisson", mean_len=90.0, zipf_s=1.05)
    X = corpus_to_csc(c)
    batches = [X.slice_docs(0, 300), X.slice_docs(300, 600), X.slice_docs(600, 900)]
    ms = schedule.geometric(1, 100, 3)
    K = 64
    o = oracle.OracleLDA(batches[0], K, 0.1, 0.01, seed=9, m0=ms[0], G=32)
    g = make_gpu(batches[0], K, 0.1, 0.01, 9, ms[0], 32)
    for t, (B, m) in enumerate(zip(batches, ms)):
        if t > 0:
            o.set_batch(B, m); g.set_batch(B.D, B.colptr, B.rowidx, B.val, m)
        rho = float(np.float32(schedule.rho(t)))
        o.sweep(m, rho); g.sweep(m, rho)
        assert_state_equal(g, o, f"minibatch {t} m={m} rho={rho}")
    g.close()


def test_staged_minibatches_overlap_order_and_wrong_announcement():
    """The same stream of minibatches with the next minibatch staged (copy, work list, initial pass on the
    library's second stream) while the current sweep is still running, from pinned host memory and from device
    memory; once with a wrong sweeps_ahead (the commit then redraws the initial pass) and once replacing a
    staged minibatch that is never committed.  Results must equal the set_batch sequence of the oracle."""
    c = synth.generate(D=1200, V=30_000, K=32, alpha=0.1, beta=0.01, seed=14, length="poisson", mean_len=80.0, zipf_s=1.05)
    X = corpus_to_csc(c)
    batches = [X.slice_docs(300 * i, 300 * (i + 1)) for i in range(4)]
    ms = [2, 5, 20, 50]
    K = 32
    o = oracle.OracleLDA(batches[0], K, 0.1, 0.01, seed=19, m0=ms[0], G=16)
    g = make_gpu(batches[0], K, 0.1, 0.01, 19, ms[0], 16)
    dev = torch.device("cuda:0")

    def arrays(B, where):
        a = [torch.from_numpy(B.colptr), torch.from_numpy(B.rowidx), torch.from_numpy(B.val)]
        return [t.pin_memory() for t in a] if where == "pinned" else [t.to(dev) for t in a]

    for t, m in enumerate(ms):
        rho = float(np.float32(schedule.rho(t)))
        o.sweep(m, rho)
        g.sweep(m, rho)                                  # asynchronous: still running while the next batch is staged
        if t + 1 < len(ms):
            B = batches[t + 1]
            o.set_batch(B, ms[t + 1])
            if t == 1:                                   # a staged minibatch that is replaced before any commit
                g.stage_batch(batches[0].D, *arrays(batches[0], "device"), 3, 0)
            keep = arrays(B, "pinned" if t % 2 == 0 else "device")
            torch.cuda.synchronize()
            g.stage_batch(B.D, *keep, ms[t + 1], 1 if t == 2 else 0)     # t == 2 announces a sweep that never comes
            g.commit_batch()
            assert g.D == B.D
            np.testing.assert_allclose(g.get(binding.THETA), o.theta, rtol=RTOL, err_msg=f"theta after commit {t + 1}")
    assert_state_equal(g, o, "after the last minibatch")
    assert g.pass_index == o.t
    with pytest.raises(binding.SameLdaError):
        g.commit_batch()                                 # nothing staged
    g.close()


# --------------------------------------------------------------------------- #
def test_random_small_configurations_all_sweep_forms():
    """Eighty seeded random configurations (shapes, densities, counts up to 3000, K from 1 to 513 including ragged
    ones, group sizes, priors, seeds), each swept two to four times with a random mix of the multinomial form
    (with and without a blend), the Poisson form (real m from 0.3 up) and the sampled parameter step."""
    rng = np.random.default_rng(20240)
    for c in range(80):
        D, V = int(rng.integers(1, 60)), int(rng.integers(1, 50))
        dens = float(rng.choice([0.05, 0.2, 0.5, 1.0]))
        cmax = int(rng.choice([1, 3, 12, 60, 400, 3000]))
        K = int(rng.choice([1, 2, 3, 4, 7, 15, 16, 17, 31, 32, 33, 48, 64, 100, 128, 200, 256, 300, 513]))
        G = int(rng.choice([1, 2, 7, 64, 1024]))
        counts = rng.integers(1, cmax + 1, size=(D, V)) * (rng.uniform(size=(D, V)) < dens)
        if counts.sum() == 0:
            counts[0, 0] = 1
        X = csc_from_dense(counts)
        alpha, beta = float(rng.choice([0.01, 0.1, 0.5, 2.0])), float(rng.choice([0.001, 0.01, 0.3]))
        m0, seed = int(rng.choice([1, 2, 10])), int(rng.integers(0, 2 ** 62))
        mmax = max(1, min(1000, 20000 // cmax))
        what = f"configuration {c}: D={D} V={V} density={dens} cmax={cmax} K={K} G={G} alpha={alpha} beta={beta} m0={m0}"
        o = oracle.OracleLDA(X, K, alpha, beta, seed=seed, m0=m0, G=G)
        g = make_gpu(X, K, alpha, beta, seed, m0, G)
        for s in range(int(rng.integers(2, 5))):
            kind = str(rng.choice(["multinomial", "multinomial", "poisson", "sampled"]))
            if kind == "multinomial":
                m, rho = int(rng.integers(1, mmax + 1)), float(rng.choice([1.0, 1.0, 0.7, 0.25]))
                o.sweep(m, rho); g.sweep(m, rho)
            elif kind == "poisson":
                m = float(np.float32(rng.choice([0.3, 1.0, 2.5, 17.0, 100.0, mmax * 0.9])))
                rho = float(rng.choice([1.0, 0.5]))
                o.sweep_poisson(m, rho); g.sweep_poisson(m, rho)
            else:
                m = int(rng.integers(1, min(mmax, 300) + 1))
                o.sweep_sampled(m); g.sweep_sampled(m)
            assert_state_equal(g, o, f"{what}, sweep {s + 1} ({kind}, m={m})")
        g.close()


def test_random_api_sequences():
    """Forty seeded random sequences of calls on one handle: sweeps in the three forms, new minibatches through
    set_batch or stage + commit (from host, pinned and device memory, with right and wrong announcements and
    sweeps in between), held-out likelihoods, and a restored state; the oracle follows every step."""
    rng = np.random.default_rng(77)
    dev = torch.device("cuda:0")

    def rand_matrix(V, cmax):
        D, dens = int(rng.integers(1, 50)), float(rng.choice([0.1, 0.4, 1.0]))
        counts = rng.integers(1, cmax + 1, size=(D, V)) * (rng.uniform(size=(D, V)) < dens)
        if counts.sum() == 0:
            counts[0, 0] = 1
        return csc_from_dense(counts)

    def arrays(B, where):
        if where == "host":
            return [B.colptr, B.rowidx, B.val]
        a = [torch.from_numpy(B.colptr), torch.from_numpy(B.rowidx), torch.from_numpy(B.val)]
        return [t.pin_memory() for t in a] if where == "pinned" else [t.to(dev) for t in a]

    for c in range(40):
        V, cmax = int(rng.integers(2, 60)), int(rng.choice([1, 5, 40, 300]))
        K, G = int(rng.choice([1, 3, 8, 16, 20, 32, 64, 100, 256])), int(rng.choice([1, 4, 1024]))
        mmax = max(1, min(200, 6000 // cmax))
        X, seed, m0 = rand_matrix(V, cmax), int(rng.integers(0, 2 ** 62)), int(rng.choice([1, 3]))
        o = oracle.OracleLDA(X, K, 0.1, 0.02, seed=seed, m0=m0, G=G)
        g = make_gpu(X, K, 0.1, 0.02, seed, m0, G)
        done = []
        for s in range(int(rng.integers(3, 9))):
            op = str(rng.choice(["sweep", "sweep", "poisson", "sampled", "set_batch", "stage", "loglik", "restore"]))
            done.append(op)
            what = f"sequence {c} (V={V} cmax={cmax} K={K} G={G}): {done}"
            if op == "sweep":
                m, rho = int(rng.integers(1, mmax + 1)), float(rng.choice([1.0, 0.6]))
                o.sweep(m, rho); g.sweep(m, rho)
            elif op == "poisson":
                m = float(np.float32(rng.uniform(0.2, mmax)))
                o.sweep_poisson(m); g.sweep_poisson(m)
            elif op == "sampled":
                m = int(rng.integers(1, mmax + 1))
                o.sweep_sampled(m); g.sweep_sampled(m)
            elif op == "set_batch":
                B, mi = rand_matrix(V, cmax), int(rng.integers(1, 4))
                o.set_batch(B, mi); g.set_batch(B.D, *arrays(B, str(rng.choice(["host", "device"]))), mi)
            elif op == "stage":
                B, mi = rand_matrix(V, cmax), int(rng.integers(1, 4))
                announced, real = int(rng.integers(0, 3)), int(rng.integers(0, 3))
                keep = arrays(B, str(rng.choice(["pinned", "device", "host"])))
                g.stage_batch(B.D, *keep, mi, announced)
                for _ in range(real):
                    m = int(rng.integers(1, mmax + 1))
                    o.sweep(m); g.sweep(m)
                o.set_batch(B, mi); g.commit_batch()
            elif op == "loglik":
                T, f, me = rand_matrix(V, cmax), int(rng.integers(0, 3)), int(rng.integers(1, 10))
                assert abs(g.loglik(T.D, T.colptr, T.rowidx, T.val, f, me) - o.loglik(T, f, me)) <= LL_ATOL, what
                continue
            else:
                g.set(binding.THETA, o.theta); g.set(binding.PHI, o.phi); g.pass_index = o.t
                continue
            assert g.pass_index == o.t, what
            assert_state_equal(g, o, what)
        g.close()


# The sampled parameter step (Algorithm 2, third step): theta and phi as Dirichlet draws
@pytest.mark.parametrize("K,G,ms", [(16, 8, [10, 1, 3]), (40, 3, [100, 2]), (5, 1000, [400, 1])])
def test_sampled_sweeps_match_the_oracle(K, G, ms):
    """Counts bit-exact, theta and phi to 1e-5: one differently decided acceptance of a Gamma variable
    would show as a wholly different value.  m = 1 with small priors takes the small-shape branch."""
    X = toy(seed=18, D=70, V=50, density=0.3, cmax=40)
    o = oracle.OracleLDA(X, K, 0.1, 0.01, seed=5, m0=3, G=G)
    g = make_gpu(X, K, 0.1, 0.01, 5, 3, G, on_device=True)
    for s, m in enumerate(ms):
        o.sweep_sampled(m); g.sweep_sampled(m)
        assert_state_equal(g, o, f"K={K} G={G} sampled sweep {s + 1} m={m}")
    o.sweep(7); g.sweep(7)                                  # and back to the collapsed update on the same handle
    assert_state_equal(g, o, "collapsed sweep after sampled ones")
    assert g.pass_index == o.t
    g.close()


def test_sampled_sweep_news_shape_slice():
    """News workload shape (K=256, V=100000) on a 600-document slice: most n_wk are zero, so most Gamma
    variables of phi have shape m*beta (1 at m=100, 0.01 at m=1: both branches) and the sums run over 1563 blocks."""
    p = synth.PRESETS["news"]
    X = corpus_to_csc(synth.preset("news", scale=0.002))
    o = oracle.OracleLDA(X, p["K"], p["alpha"], p["beta"], seed=9, m0=1, G=32)
    g = make_gpu(X, p["K"], p["alpha"], p["beta"], 9, 1, 32)
    o.sweep_sampled(100); g.sweep_sampled(100)
    assert_state_equal(g, o, "sampled m=100")
    o.sweep_sampled(1); g.sweep_sampled(1)
    assert_state_equal(g, o, "sampled m=1")
    np.testing.assert_allclose(g.get(binding.PHI).astype(np.float64).sum(axis=0), 1.0, atol=1e-4)
    g.close()


# Poisson form of the factored draw (Section 4, second part; Algorithm 3's sampling line)
@pytest.mark.parametrize("K,G,ms", [(16, 8, [10.0, 0.5, 3.25]), (24, 1, [1.0, 30.0]), (40, 3, [100.0, 2.5]),
                                    (5, 1000, [400.0, 0.1])])
def test_poisson_sweeps_bit_exact(K, G, ms):
    """Sweeps in the Poisson form with integer and non-integer m (below 1 too); large m * c gives rates far
    above 32 (pieces shared by the wave); K=40 and K=5 take the ragged path."""
    X = toy(seed=8, D=70, V=50, density=0.3, cmax=40)
    o = oracle.OracleLDA(X, K, 0.1, 0.01, seed=5, m0=3, G=G)
    g = make_gpu(X, K, 0.1, 0.01, 5, 3, G, on_device=True)
    assert_state_equal(g, o, "init")
    for s, m in enumerate(ms):
        o.sweep_poisson(m); g.sweep_poisson(m)
        assert_state_equal(g, o, f"K={K} G={G} poisson sweep {s + 1} m={m}")
    g.close()


def test_poisson_news_shape_slice_and_mixed_forms():
    """News workload shape (K=256) on a 600-document slice: Poisson sweeps at m=100 (frequent words go through
    the pair list), alternating with the multinomial form and a blend, on one handle and one stream of passes."""
    p = synth.PRESETS["news"]
    X = corpus_to_csc(synth.preset("news", scale=0.002))
    o = oracle.OracleLDA(X, p["K"], p["alpha"], p["beta"], seed=9, m0=1, G=32)
    g = make_gpu(X, p["K"], p["alpha"], p["beta"], 9, 1, 32)
    assert_state_equal(g, o, "init")
    o.sweep_poisson(100.0); g.sweep_poisson(100.0)
    assert_state_equal(g, o, "poisson m=100")
    o.sweep(20); g.sweep(20)
    assert_state_equal(g, o, "multinomial m=20")
    o.sweep_poisson(37.5, 0.6); g.sweep_poisson(37.5, 0.6)
    assert_state_equal(g, o, "poisson m=37.5 rho=0.6")
    assert g.pass_index == o.t == 4
    # the copies of a token no longer total exactly m * c
    ntok = np.bincount(np.repeat(np.arange(X.D), np.diff(X.colptr)), weights=X.val, minlength=X.D)
    assert np.any(g.get(binding.NDK).sum(axis=1) != 37.5 * ntok)
    g.close()


def test_poisson_debug_draw_matches_oracle_tasks():
    X = toy(seed=12, D=50, V=30, density=0.4, cmax=25)
    K, G, m = 32, 4, 12.5
    o = oracle.OracleLDA(X, K, 0.2, 0.05, seed=31, m0=5, G=G)
    g = make_gpu(X, K, 0.2, 0.05, 31, 5, G)
    ids = np.arange(0, g.task_count, 3)
    want = oracle.draw_tasks_poisson(X, K, G, m, 31, oracle.pass_word(o.t), o.theta, o.phi, ids)
    got = g.debug_draw_poisson(m, ids)
    assert np.array_equal(got, want)
    o.sweep_poisson(m); g.sweep_poisson(m)
    assert_state_equal(g, o, "sweep after the hook")
    g.close()


def test_poisson_rejects_bad_m():
    X = toy(seed=1, D=10, V=10, density=0.5, cmax=3)
    g = make_gpu(X, 4, 0.1, 0.01, 1, 2, 8)
    for bad in (0.0, -1.0, float("nan"), float("inf"), 1e9):
        with pytest.raises(binding.SameLdaError):
            g.sweep_poisson(bad)
    g.sweep_poisson(0.25)
    g.synchronize()
    g.close()


# --------------------------------------------------------------------------- #
# the normaliser as a stand-alone sampled dense-dense product (Section 5.3)
@pytest.mark.parametrize("K", [1, 3, 16, 40, 256, 1024])
def test_sddmm_against_double_oracle(K):
    """mu of every nonzero from the current theta and phi: binary32 tree sum on the GPU against the oracle's
    double sum; host and device output; K not a multiple of 4 takes the scalar path."""
    X = toy(seed=15, D=90, V=70, density=0.25, cmax=5)
    o = oracle.OracleLDA(X, K, 0.3, 0.02, seed=2, m0=4, G=8)
    g = make_gpu(X, K, 0.3, 0.02, 2, 4, 8)
    o.sweep(7); g.sweep(7)
    want = oracle.sddmm(X, o.theta, o.phi)
    got = g.sddmm()
    np.testing.assert_allclose(got, want, rtol=1e-5, atol=0)
    out = torch.empty(X.nnz, dtype=torch.float32, device="cuda:0")
    g.sddmm(out)
    g.synchronize()
    assert np.array_equal(out.cpu().numpy(), got)
    assert_state_equal(g, o, "state untouched by sddmm")
    g.close()


@pytest.mark.parametrize("K", [16, 64, 256, 512, 1024])
def test_short_documents_every_scan_shape(K):
    """Documents of one to three words, some empty: a refill's new tasks then change document every lane or two, so the
    scan's runs inside one document are one or two lanes long, with single lanes left over (the pipeline's prologue,
    tail and lone-lane cases, for blocks of one batch, of two, and for the scan in contiguous pieces)."""
    rng = np.random.default_rng(K)
    D, V = 700, 60
    per = rng.integers(0, 4, size=D)
    colptr = np.concatenate([[0], np.cumsum(per)]).astype(np.int32)
    rowidx = np.concatenate([np.sort(rng.choice(V, size=int(n), replace=False)) for n in per] + [np.zeros(0, np.int64)]).astype(np.int32)
    val = rng.integers(1, 6, size=int(per.sum())).astype(np.float32)
    X = oracle.CSC(D, V, colptr, rowidx, val)
    o = oracle.OracleLDA(X, K, 0.2, 0.05, seed=11, m0=3, G=8)
    g = make_gpu(X, K, 0.2, 0.05, 11, 3, 8)
    assert_state_equal(g, o, "after init")
    for t, m in enumerate([1, 7, 40]):
        o.sweep(m); g.sweep(m)
        assert_state_equal(g, o, f"sweep {t} (m={m})")
    g.close()


@pytest.mark.parametrize("nnz", [1, 5, 31, 32, 33, 64, 97])
def test_sddmm_few_nonzeros(nnz):
    """Fewer nonzeros than a wave's chunk of 32, exactly one and two chunks, and ragged ends (the kernel for up to 256
    topics loads the ids of a chunk with one instruction and the rows of every round of four unconditionally)."""
    rng = np.random.default_rng(nnz)
    D, V, K = 4, 200, 64
    per = np.full(D, nnz // D); per[: nnz % D] += 1
    colptr = np.concatenate([[0], np.cumsum(per)]).astype(np.int32)
    rowidx = np.concatenate([np.sort(rng.choice(V, size=int(n), replace=False)) for n in per]).astype(np.int32)
    val = rng.integers(1, 4, size=nnz).astype(np.float32)
    X = oracle.CSC(D, V, colptr, rowidx, val)
    o = oracle.OracleLDA(X, K, 0.3, 0.02, seed=3, m0=4, G=8)
    g = make_gpu(X, K, 0.3, 0.02, 3, 4, 8)
    o.sweep(5); g.sweep(5)
    np.testing.assert_allclose(g.sddmm(), oracle.sddmm(X, o.theta, o.phi), rtol=1e-5, atol=0)
    g.close()


def test_sddmm_empty_matrix():
    X = oracle.CSC(3, 10, np.zeros(4, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
    g = make_gpu(X, 4, 0.1, 0.01, 1, 5, 8)
    assert g.sddmm().shape == (0,)
    g.close()
