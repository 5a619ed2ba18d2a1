"""ctypes front end of the CPU oracle (``ozimmu_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py``; never by the product path.  Marshals numpy arrays
(column-major, float64) into the C functions; holds no arithmetic of the method.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ozimmu_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

OK, BAD_ARG, NONFINITE, UNREACHABLE = 0, 1, 2, 4
MAX_SLICES = 64


def build(force=False):
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
             "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oz_oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads():
    return lib().oz_oracle_num_threads()


def _f64(X):
    X = np.asarray(X, dtype=np.float64)
    if X.ndim != 2:
        raise ValueError("matrix expected")
    return np.asfortranarray(X)


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle status {code}")
        self.code = code


def _check(rc, allow=()):
    if rc != OK and rc not in allow:
        raise OracleError(rc)
    return rc


def exponents(side, X):
    """Scale exponents e with alpha = 2**e: per row (side 'A') or per column (side 'B')."""
    X = _f64(X)
    rows, cols = X.shape
    e = np.zeros(rows if side == "A" else cols, dtype=np.int32)
    _check(lib().oz_oracle_exponents(ctypes.c_char(side.encode()), rows, cols, _p(X, ctypes.c_double),
                                     max(rows, 1), _p(e, ctypes.c_int32)))
    return e


def split(side, X, s, t=7, e=None):
    """Returns (planes[s, rows, cols] int8, e)."""
    X = _f64(X)
    rows, cols = X.shape
    if e is None:
        e = exponents(side, X)
    e = np.ascontiguousarray(e, dtype=np.int32)
    planes = np.zeros((s, cols, rows), dtype=np.int8)  # each plane column-major rows x cols
    _check(lib().oz_oracle_split(ctypes.c_char(side.encode()), rows, cols, _p(X, ctypes.c_double),
                                 max(rows, 1), s, t, _p(e, ctypes.c_int32), _p(planes, ctypes.c_int8)))
    return planes.transpose(0, 2, 1), e


def split_nearest(side, X, s, t=7, e=None):
    """Round-to-nearest slices relative to the scale 2**(e+1).  Returns (planes[s, rows, cols] int8, e)
    with e the exponents of Algorithm 1 (not yet increased by one)."""
    X = _f64(X)
    rows, cols = X.shape
    if e is None:
        e = exponents(side, X)
    e = np.ascontiguousarray(e, dtype=np.int32)
    planes = np.zeros((s, cols, rows), dtype=np.int8)
    _check(lib().oz_oracle_split_nearest(ctypes.c_char(side.encode()), rows, cols, _p(X, ctypes.c_double),
                                         max(rows, 1), s, t, _p(e, ctypes.c_int32), _p(planes, ctypes.c_int8)))
    return planes.transpose(0, 2, 1), e


def slice_product(Al, Bh):
    """Exact int64 product of two int8 slice matrices."""
    Al = np.asfortranarray(np.asarray(Al, dtype=np.int8))
    Bh = np.asfortranarray(np.asarray(Bh, dtype=np.int8))
    m, k = Al.shape
    k2, n = Bh.shape
    assert k == k2
    P = np.zeros((n, m), dtype=np.int64)
    _check(lib().oz_oracle_slice_product(m, n, k, _p(Al, ctypes.c_int8), _p(Bh, ctypes.c_int8),
                                         _p(P, ctypes.c_int64)))
    return P.T


def dgemm(A, B, s, t=7, order=0, full=False, return_exponents=False):
    """C ~ A @ B by Algorithm 1; order 0 = by diagonals, 1 = literal loop nest."""
    A = _f64(A)
    B = _f64(B)
    m, k = A.shape
    k2, n = B.shape
    assert k == k2
    C = np.zeros((n, m), dtype=np.float64)
    eA = np.zeros(m, dtype=np.int32)
    eB = np.zeros(n, dtype=np.int32)
    _check(lib().oz_oracle_dgemm(m, n, k, _p(A, ctypes.c_double), max(m, 1), _p(B, ctypes.c_double),
                                 max(k, 1), _p(C, ctypes.c_double), max(m, 1), s, t, order, int(full),
                                 _p(eA, ctypes.c_int32), _p(eB, ctypes.c_int32)))
    if return_exponents:
        return C.T, eA, eB
    return C.T


def dgemm2(A, B, sA, sB, t=7, order=0, full=False, return_exponents=False):
    """C ~ A @ B with sA slices of A and sB slices of B (products with l + h <= max(sA, sB) + 1)."""
    A = _f64(A)
    B = _f64(B)
    m, k = A.shape
    k2, n = B.shape
    assert k == k2
    C = np.zeros((n, m), dtype=np.float64)
    eA = np.zeros(m, dtype=np.int32)
    eB = np.zeros(n, dtype=np.int32)
    _check(lib().oz_oracle_dgemm2(m, n, k, _p(A, ctypes.c_double), max(m, 1), _p(B, ctypes.c_double),
                                  max(k, 1), _p(C, ctypes.c_double), max(m, 1), sA, sB, t, order, int(full),
                                  _p(eA, ctypes.c_int32), _p(eB, ctypes.c_int32)))
    if return_exponents:
        return C.T, eA, eB
    return C.T


def dgemm3(A, B, sA, sB, t=7, order=0, full=False, nearest=False, Q=1, return_exponents=False):
    """dgemm2 with the two variants: slices by round-to-nearest, and diagonals accumulated in exact
    levels of Q diagonals.  Returned exponents are those of the scales used (e + 1 when nearest)."""
    A = _f64(A)
    B = _f64(B)
    m, k = A.shape
    k2, n = B.shape
    assert k == k2
    C = np.zeros((n, m), dtype=np.float64)
    eA = np.zeros(m, dtype=np.int32)
    eB = np.zeros(n, dtype=np.int32)
    _check(lib().oz_oracle_dgemm3(m, n, k, _p(A, ctypes.c_double), max(m, 1), _p(B, ctypes.c_double),
                                  max(k, 1), _p(C, ctypes.c_double), max(m, 1), sA, sB, t, order, int(full),
                                  int(nearest), Q, _p(eA, ctypes.c_int32), _p(eB, ctypes.c_int32)))
    if return_exponents:
        return C.T, eA, eB
    return C.T


def chi(sA, sB):
    return lib().oz_oracle_chi(sA, sB)


def estimate_slices2(A, B, tol, t=7, s_max=32):
    """Returns (sA, sB, status, kappa_A, kappa_B): cheapest pair meeting the tolerance."""
    A = _f64(A)
    B = _f64(B)
    m, k = A.shape
    k2, n = B.shape
    assert k == k2
    sA = ctypes.c_int(0)
    sB = ctypes.c_int(0)
    kA = ctypes.c_double(0.0)
    kB = ctypes.c_double(0.0)
    rc = _check(lib().oz_oracle_estimate_slices2(m, n, k, _p(A, ctypes.c_double), max(m, 1),
                                                 _p(B, ctypes.c_double), max(k, 1), ctypes.c_double(tol), t,
                                                 s_max, ctypes.byref(sA), ctypes.byref(sB), ctypes.byref(kA),
                                                 ctypes.byref(kB)), allow=(UNREACHABLE,))
    return sA.value, sB.value, rc, kA.value, kB.value


def kappa(side, X):
    X = _f64(X)
    rows, cols = X.shape
    out = ctypes.c_double(0.0)
    _check(lib().oz_oracle_kappa(ctypes.c_char(side.encode()), rows, cols, _p(X, ctypes.c_double),
                                 max(rows, 1), ctypes.byref(out)))
    return out.value


def estimate_slices(A, B, tol, t=7, s_max=32):
    """Returns (s, status, kappa_A, kappa_B); status is OK or UNREACHABLE."""
    A = _f64(A)
    B = _f64(B)
    m, k = A.shape
    k2, n = B.shape
    assert k == k2
    s = ctypes.c_int(0)
    kA = ctypes.c_double(0.0)
    kB = ctypes.c_double(0.0)
    rc = _check(lib().oz_oracle_estimate_slices(m, n, k, _p(A, ctypes.c_double), max(m, 1),
                                                _p(B, ctypes.c_double), max(k, 1), ctypes.c_double(tol), t,
                                                s_max, ctypes.byref(s), ctypes.byref(kA), ctypes.byref(kB)),
                allow=(UNREACHABLE,))
    return s.value, rc, kA.value, kB.value
