"""Thin ctypes binding of libsame_lda.so (argument marshalling only).

Every step of the sweep runs in the HIP library; this module converts Python objects to the
plain pointers of the C ABI.  PyTorch appears only as the owner of device memory and streams.
There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_char_p, c_double, c_float, c_int32, c_int64, c_size_t, c_uint32, c_uint64, c_void_p

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsame_lda.so")

THETA, PHI, NDK, NWK, NK = 0, 1, 2, 3, 4
# Tokens of a nonzero drawn as one multinomial (one task).  Large groups measure fastest (fewer tasks,
# and a nonzero's copies share one scan); m * min(count, this) must stay below 2^24.
DEFAULT_TOKENS_PER_DRAW = 1024
_DTYPES = {THETA: np.float32, PHI: np.float32, NDK: np.uint32, NWK: np.uint32, NK: np.uint64}

EXPORTS = ["same_lda_init", "same_lda_sweep", "same_lda_sweep_poisson", "same_lda_sweep_sampled", "same_lda_loglik", "same_lda_free",
           "same_lda_set_batch", "same_lda_stage_batch", "same_lda_commit_batch", "same_lda_debug_draw_poisson", "same_lda_sddmm",
           "same_lda_vb_exp_elog_beta", "same_lda_vb_estep",
           "same_lda_get", "same_lda_set", "same_lda_get_pass", "same_lda_set_pass", "same_lda_task_count",
           "same_lda_debug_draw", "same_lda_debug_draw_noalloc", "same_lda_debug_chunk_limit", "same_lda_set_timing", "same_lda_get_timing", "same_lda_selftest",
           "same_lda_synchronize",
           "same_lda_last_error"]


class SameLdaError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"same_lda error {code}: {text}")
        self.code = code


class _Csc(Structure):
    _fields_ = [("D", c_int32), ("V", c_int32), ("nnz", c_int64), ("colptr", c_void_p),
                ("rowidx", c_void_p), ("val", c_void_p), ("on_device", c_int32)]


_lib = None


def load(path: str | None = None) -> ctypes.CDLL:
    """Loads the built library; raises if it is missing (build it with paper_1409_5402_amd.build).  `path` (or the
    environment variable SAME_LDA_LIB) names another build of the same library, e.g. the event-counting build of
    bench.py --mode stats; the first load of a process decides."""
    global _lib
    if _lib is None:
        path = path or os.environ.get("SAME_LDA_LIB") or LIB_PATH
        if not os.path.exists(path):
            raise FileNotFoundError(f"{path} is missing: run paper_1409_5402_amd.build.build() first")
        try:
            import torch  # noqa: F401  (where torch is installed, its HIP runtime must be the one loaded first:
        except ImportError:             # the library then binds to the same runtime as the tensors it is given)
            pass
        L = ctypes.CDLL(path)
        L.same_lda_init.argtypes = [POINTER(c_void_p), POINTER(_Csc), c_int32, c_float, c_float, c_uint64,
                                    c_int32, c_int32, c_void_p]
        L.same_lda_sweep.argtypes = [c_void_p, c_int32, c_float]
        L.same_lda_sweep_sampled.argtypes = [c_void_p, c_int32]
        L.same_lda_sweep_poisson.argtypes = [c_void_p, c_float, c_float]
        L.same_lda_debug_draw_poisson.argtypes = [c_void_p, c_float, c_void_p, c_int32, c_void_p]
        L.same_lda_loglik.argtypes = [c_void_p, POINTER(_Csc), c_int32, c_int32, POINTER(c_double)]
        L.same_lda_free.argtypes = [c_void_p]
        L.same_lda_free.restype = None
        L.same_lda_set_batch.argtypes = [c_void_p, POINTER(_Csc), c_int32]
        L.same_lda_stage_batch.argtypes = [c_void_p, POINTER(_Csc), c_int32, c_int32]
        L.same_lda_commit_batch.argtypes = [c_void_p]
        L.same_lda_get.argtypes = [c_void_p, c_int32, c_void_p, c_size_t, c_int32]
        L.same_lda_set.argtypes = [c_void_p, c_int32, c_void_p, c_size_t, c_int32]
        L.same_lda_get_pass.argtypes = [c_void_p, POINTER(c_int32)]
        L.same_lda_set_pass.argtypes = [c_void_p, c_int32]
        L.same_lda_task_count.argtypes = [c_void_p, POINTER(c_int64)]
        L.same_lda_debug_draw.argtypes = [c_void_p, c_int32, c_void_p, c_int32, c_void_p]
        L.same_lda_debug_draw_noalloc.argtypes = [c_void_p, c_int32, c_void_p, c_int32, c_void_p]
        L.same_lda_debug_chunk_limit.argtypes = [c_void_p, c_int64, POINTER(c_int64)]
        L.same_lda_sddmm.argtypes = [c_void_p, c_void_p, c_int32]
        L.same_lda_vb_exp_elog_beta.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p]
        L.same_lda_vb_estep.argtypes = [c_void_p, c_void_p, c_void_p, c_float, c_int32, c_void_p, c_void_p]
        L.same_lda_set_timing.argtypes = [c_void_p, c_int32]
        L.same_lda_get_timing.argtypes = [c_void_p, POINTER(c_double), POINTER(c_int64)]
        L.same_lda_selftest.argtypes = [POINTER(c_int64)]
        L.same_lda_synchronize.argtypes = [c_void_p]
        L.same_lda_last_error.argtypes = [c_void_p]
        L.same_lda_last_error.restype = c_char_p
        for name in EXPORTS:
            if name not in ("same_lda_free", "same_lda_last_error"):
                getattr(L, name).restype = c_int32
        _lib = L
    return _lib


def _is_torch(x) -> bool:
    return type(x).__module__.startswith("torch")


def _csc(D, V, colptr, rowidx, val):
    """Builds the C view of a matrix from three numpy arrays (host) or three torch tensors."""
    keep = []
    if _is_torch(colptr):
        import torch
        dev = colptr.device
        arrs = []
        for a, dt in ((colptr, torch.int32), (rowidx, torch.int32), (val, torch.float32)):
            a = a.to(dtype=dt).contiguous()
            assert a.device == dev
            arrs.append(a)
        keep = arrs
        ptrs = [a.data_ptr() if a.numel() else None for a in arrs]
        on_device = 1 if dev.type == "cuda" else 0
        nnz = int(arrs[1].numel())
    else:
        arrs = [np.ascontiguousarray(colptr, np.int32), np.ascontiguousarray(rowidx, np.int32),
                np.ascontiguousarray(val, np.float32)]
        keep = arrs
        ptrs = [a.ctypes.data if a.size else None for a in arrs]
        on_device = 0
        nnz = int(arrs[1].size)
    c = _Csc(int(D), int(V), nnz, ptrs[0], ptrs[1], ptrs[2], on_device)
    return c, keep


def selftest() -> int:
    """Runs the library's device self-test; returns the number of mismatches (0 = pass)."""
    L = load()
    n = c_int64()
    rc = L.same_lda_selftest(byref(n))
    if rc != 0:
        raise SameLdaError(rc, L.same_lda_last_error(None).decode())
    return n.value


class SameLDA:
    """A SAME Gibbs LDA model resident on the current GPU (one handle of the C library)."""

    def __init__(self, D, V, colptr, rowidx, val, K, alpha, beta, seed, m0, tokens_per_draw=DEFAULT_TOKENS_PER_DRAW, stream=None):
        self._lib = load()
        self._h = c_void_p()
        self.V, self.K, self.D = int(V), int(K), int(D)
        self.nnz = int(rowidx.shape[0])
        if stream is None:
            try:
                import torch
                stream = torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0
            except ImportError:
                stream = 0
        c, keep = _csc(D, V, colptr, rowidx, val)
        rc = self._lib.same_lda_init(byref(self._h), byref(c), int(K), float(alpha), float(beta), int(seed),
                                     int(m0), int(tokens_per_draw), c_void_p(stream or None))
        del keep
        if rc != 0:
            raise SameLdaError(rc, self._lib.same_lda_last_error(None).decode())

    def _check(self, rc):
        if rc != 0:
            raise SameLdaError(rc, self._lib.same_lda_last_error(self._h).decode())

    def sweep(self, m, rho=1.0):
        self._check(self._lib.same_lda_sweep(self._h, int(m), float(rho)))

    def sweep_sampled(self, m):
        self._check(self._lib.same_lda_sweep_sampled(self._h, int(m)))

    def sweep_poisson(self, m, rho=1.0):
        self._check(self._lib.same_lda_sweep_poisson(self._h, float(m), float(rho)))

    def set_batch(self, D, colptr, rowidx, val, m_init):
        c, keep = _csc(D, self.V, colptr, rowidx, val)
        self._check(self._lib.same_lda_set_batch(self._h, byref(c), int(m_init)))
        self.D, self.nnz = int(D), int(rowidx.shape[0])
        del keep

    def stage_batch(self, D, colptr, rowidx, val, m_init, sweeps_ahead=0):
        c, keep = _csc(D, self.V, colptr, rowidx, val)
        self._check(self._lib.same_lda_stage_batch(self._h, byref(c), int(m_init), int(sweeps_ahead)))
        self._staged_D, self._staged_nnz = int(D), int(rowidx.shape[0])
        del keep

    def commit_batch(self):
        self._check(self._lib.same_lda_commit_batch(self._h))
        self.D, self.nnz = self._staged_D, self._staged_nnz

    def loglik(self, D, colptr, rowidx, val, foldin_sweeps, m_eval) -> float:
        c, keep = _csc(D, self.V, colptr, rowidx, val)
        out = c_double()
        self._check(self._lib.same_lda_loglik(self._h, byref(c), int(foldin_sweeps), int(m_eval), byref(out)))
        del keep
        return out.value

    def _shape(self, which):
        return {THETA: (self.D, self.K), PHI: (self.V, self.K), NDK: (self.D, self.K),
                NWK: (self.V, self.K), NK: (self.K,)}[which]

    def get(self, which) -> np.ndarray:
        out = np.empty(self._shape(which), dtype=_DTYPES[which])
        self._check(self._lib.same_lda_get(self._h, which, out.ctypes.data if out.size else None, out.nbytes, 0))
        return out

    def set(self, which, arr):
        """arr: a numpy array (host) or a torch tensor (host or device) of the matrix' shape and dtype."""
        if _is_torch(arr):
            import torch
            t = arr.contiguous()
            assert tuple(t.shape) == self._shape(which) and t.dtype == torch.float32
            nbytes = t.numel() * t.element_size()
            self._check(self._lib.same_lda_set(self._h, which, t.data_ptr() if nbytes else None, nbytes,
                                               1 if t.device.type == "cuda" else 0))
            return
        a = np.ascontiguousarray(arr, dtype=_DTYPES[which])
        assert a.shape == self._shape(which)
        self._check(self._lib.same_lda_set(self._h, which, a.ctypes.data if a.size else None, a.nbytes, 0))

    @property
    def pass_index(self) -> int:
        v = c_int32()
        self._check(self._lib.same_lda_get_pass(self._h, byref(v)))
        return v.value

    @pass_index.setter
    def pass_index(self, v):
        self._check(self._lib.same_lda_set_pass(self._h, int(v)))

    @property
    def task_count(self) -> int:
        v = c_int64()
        self._check(self._lib.same_lda_task_count(self._h, byref(v)))
        return v.value

    def debug_draw(self, m, task_ids) -> np.ndarray:
        ids = np.ascontiguousarray(task_ids, np.int64)
        out = np.zeros((ids.shape[0], self.K), np.uint32)
        self._check(self._lib.same_lda_debug_draw(self._h, int(m), ids.ctypes.data if ids.size else None,
                                                  ids.shape[0], out.ctypes.data if out.size else None))
        return out

    def debug_draw_noalloc(self, m, task_ids) -> np.ndarray:
        ids = np.ascontiguousarray(task_ids, np.int64)
        out = np.zeros((ids.shape[0], self.K), np.uint32)
        self._check(self._lib.same_lda_debug_draw_noalloc(self._h, int(m), ids.ctypes.data if ids.size else None,
                                                          ids.shape[0], out.ctypes.data if out.size else None))
        return out

    def debug_chunk_limit(self, max_chunks: int = -1) -> int:
        """Chunks of the pair-list pool the sweeps may use from now on (negative: all); returns the number in use."""
        n = c_int64(0)
        self._check(self._lib.same_lda_debug_chunk_limit(self._h, int(max_chunks), ctypes.byref(n)))
        return int(n.value)

    def debug_draw_poisson(self, m, task_ids) -> np.ndarray:
        ids = np.ascontiguousarray(task_ids, np.int64)
        out = np.zeros((ids.shape[0], self.K), np.uint32)
        self._check(self._lib.same_lda_debug_draw_poisson(self._h, float(m), ids.ctypes.data if ids.size else None,
                                                          ids.shape[0], out.ctypes.data if out.size else None))
        return out

    def sddmm(self, out=None):
        """mu of every nonzero of the resident matrix; ``out``: a float32 torch tensor on the device (filled
        asynchronously) or None (a numpy array is returned)."""
        if out is not None:
            self._check(self._lib.same_lda_sddmm(self._h, out.data_ptr(), 1))
            return out
        mu = np.zeros(self.nnz, np.float32)
        self._check(self._lib.same_lda_sddmm(self._h, mu.ctypes.data if mu.size else None, 0))
        return mu

    def vb_exp_elog_beta(self, lam, b_out, shift_out):
        """Rows of exp E[log beta] of lambda divided by their largest entry (b_out [V][K]) and the logarithm of that
        entry (shift_out [V]); all float32 torch tensors on the device; asynchronous."""
        self._check(self._lib.same_lda_vb_exp_elog_beta(self._h, lam.data_ptr(), b_out.data_ptr(), shift_out.data_ptr()))
        return b_out, shift_out

    def vb_estep(self, b, shift, alpha: float, iters: int, gamma, log_mu=None):
        """`iters` iterations of the variational E-step on the resident matrix; b [V][K], shift [V] (or None),
        gamma [D][K] (updated in place) and log_mu [nnz] (optional) are float32 torch tensors on the device;
        asynchronous."""
        self._check(self._lib.same_lda_vb_estep(self._h, b.data_ptr(), shift.data_ptr() if shift is not None else None,
                                                float(alpha), int(iters), gamma.data_ptr(),
                                                log_mu.data_ptr() if log_mu is not None else None))
        return gamma

    def set_timing(self, enabled: bool):
        self._check(self._lib.same_lda_set_timing(self._h, 1 if enabled else 0))

    def get_timing(self):
        ms, n = c_double(), c_int64()
        self._check(self._lib.same_lda_get_timing(self._h, byref(ms), byref(n)))
        return ms.value, n.value

    def synchronize(self):
        self._check(self._lib.same_lda_synchronize(self._h))

    def close(self):
        if self._h:
            self._lib.same_lda_free(self._h)
            self._h = c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
