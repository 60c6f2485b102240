"""ctypes face of ``bsse_oracle.c``.  TEST INFRASTRUCTURE ONLY (see the C file's header).

All arithmetic is in the C file; this module only marshals numpy arrays.
"""
import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build()
        lib = ctypes.CDLL(path)
        lib.bsse_oracle_sweep.restype = ctypes.c_int
        lib.bsse_oracle_sweep.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.bsse_oracle_value_under_profile.restype = ctypes.c_double
        lib.bsse_oracle_value_under_profile.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


@dataclass
class SweepResult:
    best_value: float
    best_index: int
    best_br: np.ndarray            # int32[K]
    values: Optional[np.ndarray]   # float64[C] or None
    br: Optional[np.ndarray]       # int32[C, K] or None
    gap: Optional[np.ndarray]      # float64[C, K] or None
    scale: Optional[np.ndarray]    # float64[C, K] or None
    threads: int


def _payoffs64(A, B, prior):
    A = np.ascontiguousarray(A, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    prior = np.ascontiguousarray(prior, dtype=np.float64)
    if A.ndim != 3 or A.shape != B.shape or prior.shape != (A.shape[0],):
        raise ValueError("A, B must be [K][m][n] of one shape and prior [K]")
    return A, B, prior


def sweep(A, B, prior, X, per_candidate=True, diagnostics=False, nthreads=1) -> SweepResult:
    """Sweep the rows of X ([C][m], float32 or float64; float32 is widened, not altered)."""
    A, B, prior = _payoffs64(A, B, prior)
    K, m, n = A.shape
    X = np.asarray(X)
    if X.dtype == np.float32:
        X = np.ascontiguousarray(X)
        is32 = 1
    else:
        X = np.ascontiguousarray(X, dtype=np.float64)
        is32 = 0
    if X.ndim != 2 or X.shape[1] != m:
        raise ValueError("X must be [C][m]")
    C = X.shape[0]
    V = np.empty(C, np.float64) if per_candidate else None
    br = np.empty((C, K), np.int32) if per_candidate else None
    gap = np.empty((C, K), np.float64) if diagnostics else None
    scale = np.empty((C, K), np.float64) if diagnostics else None
    bv = ctypes.c_double(float("nan"))
    bi = ctypes.c_int64(-1)
    bbr = np.full(K, -1, np.int32)
    used = _load().bsse_oracle_sweep(m, n, K, _p(A), _p(B), _p(prior), _p(X), is32, C,
                                     _p(V), _p(br), _p(gap), _p(scale),
                                     ctypes.byref(bv), ctypes.byref(bi), _p(bbr), int(nthreads))
    if used < 0:
        raise MemoryError("oracle allocation failed")
    return SweepResult(bv.value, bi.value, bbr, V, br, gap, scale, used)


def value_under_profile(A, prior, x, br):
    """(value, abs-scale) of candidate x when type t is told to play br[t]."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    prior = np.ascontiguousarray(prior, dtype=np.float64)
    K, m, n = A.shape
    x = np.ascontiguousarray(x, dtype=np.float64)
    br = np.ascontiguousarray(br, dtype=np.int32)
    s = ctypes.c_double(0.0)
    v = _load().bsse_oracle_value_under_profile(m, n, K, _p(A), _p(prior), _p(x), _p(br),
                                                ctypes.byref(s))
    return v, s.value
