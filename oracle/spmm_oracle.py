"""ORACLE -- test infrastructure only.

ctypes front end of ``spmm_oracle.c`` (the paper's Listing 1, Section 3.1,
evaluated serially in double over CSR storage) and the parity metric that
compares a single-precision result with it.

Only tests, ``__graft_entry__.smoke()`` and the benchmark's ``cpu_baseline``
leg may import this module.  It imports nothing from the HIP package.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIBS = {}


def _lib(parallel):
    key = bool(parallel)
    if key not in _LIBS:
        serial, omp = _build.build(force=False)
        lib = ctypes.CDLL(omp if key else serial)
        lib.spmm_oracle_f64.restype = ctypes.c_int
        lib.spmm_oracle_f64.argtypes = [
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p]
        lib.spmm_oracle_threads.restype = ctypes.c_int
        _LIBS[key] = lib
    return _LIBS[key]


def threads(parallel=False):
    """Threads the oracle's row loop uses in the chosen build."""
    return int(_lib(parallel).spmm_oracle_threads())


def spmm(row_ptr, col_idx, vals, B, K=None, want_abs=True, parallel=False):
    """C_ref = A @ B in double (stored-order serial sums) and the normaliser S.

    row_ptr/col_idx: int32 CSR of A (M x K); vals: float32; B: float32 (K x N),
    row-major.  Returns (C_ref, S) as float64 arrays of shape (M, N); S is None
    when want_abs is False.  ``parallel`` selects the OpenMP build of the same
    source (timing only; identical results).
    """
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    B = np.ascontiguousarray(B, dtype=np.float32)
    if B.ndim != 2:
        raise ValueError("B must be 2-D (K x N)")
    M = row_ptr.shape[0] - 1
    if K is None:
        K = B.shape[0]
    if B.shape[0] != K:
        raise ValueError("B has %d rows, A has %d columns" % (B.shape[0], K))
    N = B.shape[1]
    C = np.empty((M, N), dtype=np.float64)
    S = np.empty((M, N), dtype=np.float64) if want_abs else None
    rc = _lib(parallel).spmm_oracle_f64(
        M, K, N, row_ptr.ctypes.data, col_idx.ctypes.data, vals.ctypes.data,
        B.ctypes.data, C.ctypes.data, S.ctypes.data if want_abs else None)
    if rc != 0:
        raise ValueError("malformed CSR input (oracle code %d)" % rc)
    return C, S


def parity_error(C_test, C_ref, S):
    """Parity metric of the target statement: per-element |C_test - C_ref| / S.

    Returns (max_rel_err over elements with S > 0, n_bad_zero) where
    n_bad_zero counts elements with S == 0 (no term, or every product zero)
    whose tested value is not exactly zero.
    """
    C_test = np.asarray(C_test, dtype=np.float64)
    if C_test.shape != C_ref.shape:
        raise ValueError("shape mismatch %s vs %s" % (C_test.shape, C_ref.shape))
    pos = S > 0
    diff = np.abs(C_test - C_ref)
    max_rel = float(np.max(diff[pos] / S[pos])) if pos.any() else 0.0
    if not np.all(np.isfinite(C_test)):
        max_rel = float("inf")
    n_bad_zero = int(np.count_nonzero(C_test[~pos] != 0.0))
    return max_rel, n_bad_zero
