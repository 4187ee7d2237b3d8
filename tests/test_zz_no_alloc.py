"""The entry point that allocates nothing (same_lda_debug_draw_noalloc, for callers that cannot call hipMalloc)
against the existing same_lda_debug_draw, through the C ABI: two calls in a row, the second with a smaller
input, bit for bit; sizes beyond its stated maximum are refused."""
import numpy as np
import pytest

import oracle
from helpers import csc_from_dense
from paper_1409_5402_amd import binding

pytestmark = pytest.mark.gpu


def test_no_alloc_debug_draw_matches_the_allocating_one_twice():
    rng = np.random.default_rng(3)
    counts = rng.integers(1, 30, size=(300, 60)) * (rng.uniform(size=(300, 60)) < 0.4)
    X = csc_from_dense(counts)
    K, m, G = 48, 25, 4
    g = binding.SameLDA(X.D, X.V, X.colptr, X.rowidx, X.val, K, 0.1, 0.01, seed=12, m0=m, tokens_per_draw=G)
    g.sweep(m)
    n_tasks = g.task_count
    ids_a = rng.choice(n_tasks, size=3000, replace=False)
    ids_b = rng.choice(n_tasks, size=700, replace=False)           # the second call is smaller: stale rows must not show
    for ids in (ids_a, ids_b):
        want = g.debug_draw(m, ids)
        got = g.debug_draw_noalloc(m, ids)
        assert np.array_equal(got, want)
        assert np.all(got.sum(axis=1) % m == 0) and got.sum() > 0
    # and against the oracle, like the allocating hook's own test
    theta, phi = g.get(binding.THETA), g.get(binding.PHI)
    ref = oracle.draw_tasks(X, K, G, m, 12, oracle.pass_word(g.pass_index), theta, phi, ids_b)
    assert np.array_equal(g.debug_draw_noalloc(m, ids_b), ref)
    assert g.debug_draw_noalloc(m, np.zeros(0, np.int64)).shape == (0, K)
    with pytest.raises(binding.SameLdaError) as e:
        g.debug_draw_noalloc(m, np.zeros(4097, np.int64))
    assert e.value.code == -1 and "at most" in str(e.value)
    with pytest.raises(binding.SameLdaError):
        g.debug_draw_noalloc(m, np.array([n_tasks], np.int64))      # a task id out of range
    g.sweep(m)                                                      # the state is untouched: the next sweep matches the oracle
    o_ndk, _, _ = oracle.run_pass(X, K, G, m, 12, oracle.pass_word(g.pass_index - 1), theta, phi)
    assert np.array_equal(g.get(binding.NDK), o_ndk)
    g.close()
