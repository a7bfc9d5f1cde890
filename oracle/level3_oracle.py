"""ctypes front-end of the C oracle in level3_oracle.c  --  TEST INFRASTRUCTURE ONLY.

SYMM, SYRK and TRMM by their BLAS definitions (the paper's routine table, Section 3.1), FP64, on numpy
host arrays in BLAS storage (flat buffer + leading dimension).  Returns (ref, d_ref) as float64 arrays of
the logical shape; SYRK marks the entries outside the referenced triangle with NaN.  No arithmetic
happens in this file.
"""
import ctypes

import numpy as np

from . import gemm_oracle as _g

ROW_MAJOR, COL_MAJOR = 101, 102
NO_TRANS, TRANS = 111, 112
UPPER, LOWER = 121, 122
NON_UNIT, UNIT = 131, 132
LEFT, RIGHT = 141, 142

_ready = False


def _lib():
    global _ready
    L = _g.lib()
    if not _ready:
        i64, dbl, vp, ci = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_int
        L.oracle_symm.argtypes = [ci, ci, ci, ci, i64, i64, dbl, vp, i64, vp, i64, dbl, vp, i64, vp, vp]
        L.oracle_symm.restype = None
        L.oracle_syrk.argtypes = [ci, ci, ci, ci, i64, i64, dbl, vp, i64, dbl, vp, i64, vp, vp]
        L.oracle_syrk.restype = None
        L.oracle_trmm.argtypes = [ci, ci, ci, ci, ci, ci, i64, i64, dbl, vp, i64, vp, i64, vp, vp]
        L.oracle_trmm.restype = None
        _ready = True
    return L


def _flat(a, dtype, count, what):
    a = np.ascontiguousarray(a).reshape(-1)
    want = np.float32 if dtype == "f32" else np.float16
    if a.dtype != want:
        raise TypeError(f"{what}: expected {want}, got {a.dtype}")
    if a.size < count:
        raise ValueError(f"{what}: {a.size} elements, need {count}")
    return a


def _span(layout, rows, cols, ld):
    """elements a rows x cols matrix with leading dimension ld occupies"""
    if rows == 0 or cols == 0:
        return 0
    major, minor = (cols, rows) if layout == COL_MAJOR else (rows, cols)
    assert ld >= minor
    return (major - 1) * ld + minor


def _p(a):
    return ctypes.c_void_p(a.ctypes.data)


def symm(dtype, layout, side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc):
    ka = m if side == LEFT else n
    A = _flat(A, dtype, _span(layout, ka, ka, lda) if alpha != 0 else 0, "A")
    B = _flat(B, dtype, _span(layout, m, n, ldb) if alpha != 0 else 0, "B")
    C = _flat(C, dtype, _span(layout, m, n, ldc) if beta != 0 else 0, "C")
    c_ref, d_ref = np.empty((m, n), np.float64), np.empty((m, n), np.float64)
    _lib().oracle_symm(int(dtype == "f16"), layout, side, uplo, m, n, float(alpha), _p(A), lda, _p(B), ldb, float(beta),
                       _p(C), ldc, _p(c_ref), _p(d_ref))
    return c_ref, d_ref


def syrk(dtype, layout, uplo, trans, n, k, alpha, A, lda, beta, C, ldc):
    rows, cols = (n, k) if trans == NO_TRANS else (k, n)
    A = _flat(A, dtype, _span(layout, rows, cols, lda) if alpha != 0 else 0, "A")
    C = _flat(C, dtype, _span(layout, n, n, ldc) if beta != 0 else 0, "C")
    c_ref, d_ref = np.empty((n, n), np.float64), np.empty((n, n), np.float64)
    _lib().oracle_syrk(int(dtype == "f16"), layout, uplo, trans, n, k, float(alpha), _p(A), lda, float(beta), _p(C), ldc,
                       _p(c_ref), _p(d_ref))
    return c_ref, d_ref


def trmm(dtype, layout, side, uplo, trans, diag, m, n, alpha, A, lda, B, ldb):
    ka = m if side == LEFT else n
    A = _flat(A, dtype, _span(layout, ka, ka, lda) if alpha != 0 else 0, "A")
    B = _flat(B, dtype, _span(layout, m, n, ldb) if alpha != 0 else 0, "B")
    b_ref, d_ref = np.empty((m, n), np.float64), np.empty((m, n), np.float64)
    _lib().oracle_trmm(int(dtype == "f16"), layout, side, uplo, trans, diag, m, n, float(alpha), _p(A), lda, _p(B), ldb,
                       _p(b_ref), _p(d_ref))
    return b_ref, d_ref
