"""CPU-only checks of the host logic: the C-ABI library loads and exports every declared symbol,
argument validation that needs no GPU, the schedules and the corpus generator."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_1409_5402_amd import binding, schedule, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "same_lda.h")).read()
    declared = sorted(set(re.findall(r"\b(same_lda_[a-z_]+)\s*\(", header)))
    assert "same_lda_init" in declared and "same_lda_sweep" in declared
    assert "same_lda_loglik" in declared and "same_lda_free" in declared
    assert sorted(binding.EXPORTS) == declared
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_validation_without_gpu():
    """Errors found before any device call: no GPU needed, nothing is launched."""
    X = (2, 5, np.array([0, 1, 2], np.int32), np.array([0, 1], np.int32), np.array([1, 2], np.float32))
    for K, alpha, beta, m0, G in [(0, 0.1, 0.01, 1, 8), (5000, 0.1, 0.01, 1, 8), (4, 0.0, 0.01, 1, 8),
                                  (4, 0.1, -1.0, 1, 8), (4, 0.1, 0.01, 1, 0)]:
        with pytest.raises(binding.SameLdaError) as e:
            binding.SameLDA(*X, K, alpha, beta, 1, m0, G, stream=0)
        assert e.value.code == -1 and str(e.value)
    lib = binding.load()
    assert lib.same_lda_sweep(None, 1, 1.0) == -1
    lib.same_lda_free(None)


def test_schedules():
    assert schedule.constant(100, 3) == [100, 100, 100]
    lin = schedule.linear(100, 19)                       # 2*100*t/20 = 10 t
    assert lin == [10 * t for t in range(1, 20)]
    assert schedule.linear(10.5, 20) == list(range(1, 21))
    inv = schedule.invlinear(100, 19)
    assert inv == lin[::-1]
    lg = schedule.logarithmic(100, 50)
    assert lg[0] == 1 and all(b >= a for a, b in zip(lg, lg[1:]))
    assert abs(sum(lg) / 50 - 100) < 1.5                 # the average stays m
    geo = schedule.geometric(1, 100, 80)
    assert geo[0] == 1 and geo[-1] == 100 and all(b >= a for a, b in zip(geo, geo[1:]))
    assert schedule.rho(0) == 1.0 and schedule.rho(3) == pytest.approx(0.5)
    assert schedule.rho(99, tau0=1.0, gamma=0.5) == pytest.approx(0.1)


def test_generator_shapes_and_determinism():
    c = synth.generate(D=200, V=500, K=8, alpha=0.1, beta=0.01, seed=5, mean_len=50.0, zipf_s=1.1)
    c2 = synth.generate(D=200, V=500, K=8, alpha=0.1, beta=0.01, seed=5, mean_len=50.0, zipf_s=1.1)
    for a, b in [(c.colptr, c2.colptr), (c.rowidx, c2.rowidx), (c.val, c2.val)]:
        assert np.array_equal(a.numpy(), b.numpy())
    colptr, rowidx, val = c.colptr.numpy(), c.rowidx.numpy(), c.val.numpy()
    assert colptr[0] == 0 and colptr[-1] == c.nnz and np.all(np.diff(colptr) >= 0)
    assert rowidx.min() >= 0 and rowidx.max() < 500
    assert np.all(val >= 1) and np.all(val == np.floor(val))
    for d in range(200):                                 # ascending word ids inside a document
        seg = rowidx[colptr[d]:colptr[d + 1]]
        assert np.all(np.diff(seg) > 0)
    st = c.stats()
    assert abs(st["tokens"] / 200 - 50.0) < 3.0
    # Zipf skew: low word ids carry most tokens
    tok = np.zeros(500); np.add.at(tok, rowidx, val)
    assert tok[:50].sum() > tok[250:].sum()
    s = c.slice_docs(10, 20)
    assert s.D == 10 and s.nnz == colptr[20] - colptr[10]
