"""CPU oracle: unblocked long-double LDL^T log-determinant and Leibniz determinant.

TEST INFRASTRUCTURE ONLY.  Import this from tests, from the smoke check and from
the benchmark's CPU-baseline leg; the GPU library never touches it.  The
arithmetic lives in ``ldlt_oracle.c`` (see its header for the definition it
follows: Sec. 2.2 and App. D of the paper, symmetric/LDL^T case).
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
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        i64 = ctypes.c_int64
        pd = ctypes.POINTER(ctypes.c_double)
        for name, ptr_t in (("oracle_ldlt_f64", ctypes.c_void_p), ("oracle_ldlt_f32", ctypes.c_void_p)):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [ptr_t, i64, i64, pd, ctypes.POINTER(ctypes.c_int),
                           ctypes.POINTER(i64), ctypes.POINTER(i64),
                           ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        for name in ("oracle_cholesky_f64", "oracle_cholesky_f32"):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [ctypes.c_void_p, i64, i64, pd, ctypes.POINTER(i64),
                           ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        for name in ("oracle_ldlt_pivoted_f64", "oracle_ldlt_pivoted_f32"):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [ctypes.c_void_p, i64, i64, i64, ctypes.c_int, pd, ctypes.POINTER(ctypes.c_int),
                           ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.c_void_p, ctypes.c_void_p,
                           ctypes.c_void_p, ctypes.c_void_p]
        for name in ("oracle_lu_f64", "oracle_lu_f32"):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [ctypes.c_void_p, i64, i64, i64, pd, ctypes.POINTER(ctypes.c_int),
                           ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.c_void_p, ctypes.c_void_p,
                           ctypes.c_void_p]
        lib.oracle_leibniz_f64.restype = ctypes.c_int
        lib.oracle_leibniz_f64.argtypes = [ctypes.c_void_p, ctypes.c_int, pd,
                                           ctypes.POINTER(ctypes.c_int), pd]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


@dataclass
class OracleResult:
    logabsdet: float          # log|det A|  (-inf when singular)
    sign: int                 # -1, 0, +1   (numpy.linalg.slogdet convention)
    status: int               # 0 ok, 1 exact zero pivot
    bad_pivot_index: int      # index of the zero pivot, else -1
    negative_pivots: int
    diag: Optional[np.ndarray] = None      # pivots d_j (float64)
    cum_logabs: Optional[np.ndarray] = None  # logdet of leading principal blocks
    L: Optional[np.ndarray] = None         # unit lower factor (float64)


def ldlt_logdet(a: np.ndarray, want_diag: bool = False, want_L: bool = False) -> OracleResult:
    """log|det A| and sign of the symmetric matrix whose LOWER triangle is in ``a``.

    ``a`` is a 2-D float64 or float32 array (row-major); only a[i, j] with
    i >= j is read.  The arithmetic is long double on the exact input bits.
    """
    lib = _load()
    if a.ndim != 2 or a.shape[0] != a.shape[1]:
        raise ValueError("square matrix expected")
    if a.dtype not in (np.float64, np.float32):
        raise ValueError("float64 or float32 expected")
    a = np.ascontiguousarray(a)
    n = a.shape[0]
    lda = a.strides[0] // a.itemsize if n > 0 else 1
    fn = lib.oracle_ldlt_f64 if a.dtype == np.float64 else lib.oracle_ldlt_f32
    lad = ctypes.c_double(0.0)
    sg = ctypes.c_int(0)
    bad = ctypes.c_int64(-1)
    neg = ctypes.c_int64(0)
    d = np.empty(n, dtype=np.float64) if want_diag else None
    cum = np.empty(n, dtype=np.float64) if want_diag else None
    L = np.empty((n, n), dtype=np.float64) if want_L else None
    st = fn(a.ctypes.data, n, max(lda, 1), ctypes.byref(lad), ctypes.byref(sg),
            ctypes.byref(bad), ctypes.byref(neg),
            d.ctypes.data if d is not None else None,
            cum.ctypes.data if cum is not None else None,
            L.ctypes.data if L is not None else None)
    if st == 2:
        raise MemoryError("oracle allocation failed")
    return OracleResult(lad.value, sg.value, st, bad.value, neg.value, d, cum,
                        L if st == 0 else None)


@dataclass
class CholeskyResult:
    logdet: float             # 2 sum log L_jj  (NaN when not positive definite)
    status: int               # 0 ok, 3 a pivot was not positive
    bad_pivot_index: int      # index of that pivot, else -1
    diag: Optional[np.ndarray] = None        # L_jj
    cum_logdet: Optional[np.ndarray] = None  # logdet of leading principal blocks
    L: Optional[np.ndarray] = None           # lower-triangular factor


def cholesky_logdet(a: np.ndarray, want_diag: bool = False, want_L: bool = False) -> CholeskyResult:
    """logdet of the symmetric positive-definite matrix whose LOWER triangle is in ``a``,
    by unblocked Cholesky in long double on the exact input bits (float64 or float32)."""
    lib = _load()
    if a.ndim != 2 or a.shape[0] != a.shape[1]:
        raise ValueError("square matrix expected")
    if a.dtype not in (np.float64, np.float32):
        raise ValueError("float64 or float32 expected")
    a = np.ascontiguousarray(a)
    n = a.shape[0]
    lda = a.strides[0] // a.itemsize if n > 0 else 1
    fn = lib.oracle_cholesky_f64 if a.dtype == np.float64 else lib.oracle_cholesky_f32
    ld = ctypes.c_double(0.0)
    bad = ctypes.c_int64(-1)
    d = np.empty(n, dtype=np.float64) if want_diag else None
    cum = np.empty(n, dtype=np.float64) if want_diag else None
    L = np.empty((n, n), dtype=np.float64) if want_L else None
    st = fn(a.ctypes.data, n, max(lda, 1), ctypes.byref(ld), ctypes.byref(bad),
            d.ctypes.data if d is not None else None,
            cum.ctypes.data if cum is not None else None,
            L.ctypes.data if L is not None else None)
    if st == 2:
        raise MemoryError("oracle allocation failed")
    return CholeskyResult(ld.value, st, bad.value, d if st == 0 else None, cum if st == 0 else None,
                          L if st == 0 else None)


@dataclass
class PivotedResult:
    logabsdet: float
    sign: int
    status: int               # 0 ok, 1 exact zero pivot
    bad_pivot_index: int      # step at which every candidate pivot was zero, else -1
    negative_pivots: int
    perm: np.ndarray          # a[perm][:, perm] = L diag(d) L^T
    slack: np.ndarray         # |pivot taken| / |largest candidate| at each step
    diag: np.ndarray          # pivots d_j in the order they were taken
    L: Optional[np.ndarray] = None


def ldlt_pivoted(a: np.ndarray, group: int = 64, choose: bool = True, want_L: bool = False) -> PivotedResult:
    """LDL^T of the symmetric matrix whose LOWER triangle is in ``a`` with diagonal
    pivoting inside groups of ``group`` consecutive indices (Sec. 2.2: pivoting inside a
    block, none between blocks), long double on the exact input bits.  ``choose=False``
    swaps nothing and only reports, in ``slack``, how each pivot compares with the one the
    rule would have taken (to check a permutation found elsewhere, permute first)."""
    lib = _load()
    if a.ndim != 2 or a.shape[0] != a.shape[1]:
        raise ValueError("square matrix expected")
    if a.dtype not in (np.float64, np.float32):
        raise ValueError("float64 or float32 expected")
    a = np.ascontiguousarray(a)
    n = a.shape[0]
    lda = a.strides[0] // a.itemsize if n > 0 else 1
    fn = lib.oracle_ldlt_pivoted_f64 if a.dtype == np.float64 else lib.oracle_ldlt_pivoted_f32
    lad = ctypes.c_double(0.0)
    sg = ctypes.c_int(0)
    bad = ctypes.c_int64(-1)
    neg = ctypes.c_int64(0)
    perm = np.empty(n, dtype=np.int64)
    slack = np.empty(n, dtype=np.float64)
    d = np.empty(n, dtype=np.float64)
    L = np.empty((n, n), dtype=np.float64) if want_L else None
    st = fn(a.ctypes.data, n, max(lda, 1), int(group), 1 if choose else 0, ctypes.byref(lad),
            ctypes.byref(sg), ctypes.byref(bad), ctypes.byref(neg), perm.ctypes.data,
            slack.ctypes.data, d.ctypes.data, L.ctypes.data if L is not None else None)
    if st == 2:
        raise MemoryError("oracle allocation failed or bad group size")
    return PivotedResult(lad.value, sg.value, st, bad.value, neg.value, perm, slack, d,
                         L if st == 0 else None)


@dataclass
class LUResult:
    logabsdet: float
    sign: int                 # sign of the permutation times the signs of the pivots
    status: int               # 0 ok, 1 exact zero pivot
    bad_pivot_index: int
    negative_pivots: int
    perm: np.ndarray          # a[perm, :] = L U
    diag: np.ndarray          # pivots U_jj
    LU: Optional[np.ndarray] = None   # L strictly below the diagonal (unit diagonal implied), U on and above


def lu_logdet(a: np.ndarray, group: int = 64, want_LU: bool = False) -> LUResult:
    """log|det A| and sign of a general square matrix (all entries are read) by Gaussian
    elimination with the pivot of each column taken among the rows of its group of ``group``
    consecutive indices (Sec. 2.2, Alg. 1: M = P L U; pivoting inside a block, none between
    blocks), long double on the exact input bits."""
    lib = _load()
    if a.ndim != 2 or a.shape[0] != a.shape[1]:
        raise ValueError("square matrix expected")
    if a.dtype not in (np.float64, np.float32):
        raise ValueError("float64 or float32 expected")
    a = np.ascontiguousarray(a)
    n = a.shape[0]
    lda = a.strides[0] // a.itemsize if n > 0 else 1
    fn = lib.oracle_lu_f64 if a.dtype == np.float64 else lib.oracle_lu_f32
    lad = ctypes.c_double(0.0)
    sg = ctypes.c_int(0)
    bad = ctypes.c_int64(-1)
    neg = ctypes.c_int64(0)
    perm = np.empty(n, dtype=np.int64)
    d = np.empty(n, dtype=np.float64)
    LU = np.empty((n, n), dtype=np.float64) if want_LU else None
    st = fn(a.ctypes.data, n, max(lda, 1), int(group), ctypes.byref(lad), ctypes.byref(sg), ctypes.byref(bad),
            ctypes.byref(neg), perm.ctypes.data, d.ctypes.data, LU.ctypes.data if LU is not None else None)
    if st == 2:
        raise MemoryError("oracle allocation failed or bad group size")
    return LUResult(lad.value, sg.value, st, bad.value, neg.value, perm, d, LU if st == 0 else None)


def leibniz_logdet(a: np.ndarray):
    """Brute-force determinant over all permutations (n <= 10), long double.

    Reads the full matrix.  Returns (logabsdet, sign, det).
    """
    lib = _load()
    a = np.ascontiguousarray(a, dtype=np.float64)
    n = a.shape[0]
    lad = ctypes.c_double(0.0)
    sg = ctypes.c_int(0)
    det = ctypes.c_double(0.0)
    st = lib.oracle_leibniz_f64(a.ctypes.data, n, ctypes.byref(lad), ctypes.byref(sg), ctypes.byref(det))
    if st != 0:
        raise ValueError("n must be <= 10")
    return lad.value, sg.value, det.value


def num_threads() -> int:
    return _load().oracle_num_threads()
