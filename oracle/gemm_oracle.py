"""ctypes front-end of the C oracle in gemm_oracle.c  --  TEST INFRASTRUCTURE ONLY.

Takes numpy host arrays exactly as a BLAS caller would lay them out in memory
(flat storage + leading dimension) and returns FP64 (m, n) arrays:
the exact-definition result C_ref and the error denominator
D = |alpha| (|op(A)| |op(B)|) + |beta| |C_old|.

Definition followed: the BLAS GEMM the paper names in Section 1 / Section 3.1, and its
batched form of Section 4.6.  No arithmetic happens in this file.
"""
import ctypes
import os

import numpy as np

from . import build as _build

ROW_MAJOR, COL_MAJOR = 101, 102
NO_TRANS, TRANS = 111, 112

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = ctypes.CDLL(path)
        i64, dbl, vp = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        ci = ctypes.c_int
        _lib.oracle_sgemm.argtypes = [ci, ci, ci, i64, i64, i64, dbl, vp, i64, vp, i64, dbl, vp, i64, vp, vp]
        _lib.oracle_sgemm.restype = None
        _lib.oracle_hgemm.argtypes = _lib.oracle_sgemm.argtypes
        _lib.oracle_hgemm.restype = None
        _lib.oracle_gemm_entries.argtypes = [ci, ci, ci, ci, i64, dbl, vp, i64, vp, i64, dbl, vp, i64,
                                             vp, vp, i64, vp, vp]
        _lib.oracle_gemm_entries.restype = None
        _lib.oracle_sgemm_batched.argtypes = [ci, ci, ci, i64, i64, i64, vp, vp, vp, i64, vp, vp, i64,
                                              vp, vp, vp, i64, i64, vp, vp]
        _lib.oracle_sgemm_batched.restype = None
        _lib.oracle_hgemm_batched.argtypes = _lib.oracle_sgemm_batched.argtypes
        _lib.oracle_hgemm_batched.restype = None
        _lib.oracle_gemv.argtypes = [ci, ci, ci, i64, i64, dbl, vp, i64, vp, i64, dbl, vp, i64, vp, vp]
        _lib.oracle_gemv.restype = None
        _lib.oracle_half_to_double.argtypes = [vp, i64, vp]
        _lib.oracle_half_to_double.restype = None
        _lib.oracle_threads.argtypes = []
        _lib.oracle_threads.restype = ci
    return _lib


def threads() -> int:
    return int(lib().oracle_threads())


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def _flat(a, dtype):
    a = np.ascontiguousarray(a).reshape(-1)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def _need(layout, trans, rows, cols, ld):
    """smallest flat length that holds op-stored matrix of logical (rows x cols) after op"""
    r, c = (rows, cols) if trans == NO_TRANS else (cols, rows)   # stored extents
    if r == 0 or c == 0:
        return 0
    if layout == COL_MAJOR:
        return (c - 1) * ld + r
    return (r - 1) * ld + c


def _check(layout, ta, tb, m, n, k, A, lda, B, ldb, C, ldc, alpha_zero, beta_zero):
    assert layout in (ROW_MAJOR, COL_MAJOR) and ta in (NO_TRANS, TRANS) and tb in (NO_TRANS, TRANS)
    if not alpha_zero:
        assert A.size >= _need(layout, ta, m, k, lda), "A too short"
        assert B.size >= _need(layout, tb, k, n, ldb), "B too short"
    if not beta_zero:
        assert C.size >= _need(layout, NO_TRANS, m, n, ldc), "C too short"


def gemm(dtype, layout, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc):
    """Full oracle.  dtype 'f32' (float32 arrays) or 'f16' (float16 arrays, read as bit patterns).
    Returns (C_ref, D), both float64 of shape (m, n)."""
    np_t = {"f32": np.float32, "f16": np.float16}[dtype]
    A, B, C = _flat(A, np_t), _flat(B, np_t), _flat(C, np_t)
    _check(layout, ta, tb, m, n, k, A, lda, B, ldb, C, ldc, alpha == 0 or k == 0, beta == 0)
    c_ref = np.empty((m, n), dtype=np.float64)
    d_ref = np.empty((m, n), dtype=np.float64)
    fn = lib().oracle_sgemm if dtype == "f32" else lib().oracle_hgemm
    fn(layout, ta, tb, m, n, k, float(alpha), _ptr(A), lda, _ptr(B), ldb, float(beta), _ptr(C), ldc,
       _ptr(c_ref), _ptr(d_ref))
    return c_ref, d_ref


def gemm_entries(dtype, layout, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, rows, cols):
    """Oracle for selected output entries (rows[s], cols[s]).  Returns (C_ref, D) of shape (count,)."""
    np_t = {"f32": np.float32, "f16": np.float16}[dtype]
    A, B, C = _flat(A, np_t), _flat(B, np_t), _flat(C, np_t)
    _check(layout, ta, tb, m, n, k, A, lda, B, ldb, C, ldc, alpha == 0 or k == 0, beta == 0)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    assert rows.shape == cols.shape and rows.ndim == 1
    if rows.size:
        assert rows.min() >= 0 and rows.max() < m and cols.min() >= 0 and cols.max() < n
    c_ref = np.empty(rows.size, dtype=np.float64)
    d_ref = np.empty(rows.size, dtype=np.float64)
    lib().oracle_gemm_entries(1 if dtype == "f16" else 0, layout, ta, tb, k, float(alpha), _ptr(A), lda,
                              _ptr(B), ldb, float(beta), _ptr(C), ldc, _ptr(rows), _ptr(cols),
                              rows.size, _ptr(c_ref), _ptr(d_ref))
    return c_ref, d_ref


def sgemm_batched(layout, ta, tb, m, n, k, alphas, A, a_off, lda, B, b_off, ldb, betas, C, c_off, ldc):
    """Batched FP32 oracle.  Returns (C_ref, D) of shape (batch, m, n)."""
    return gemm_batched("f32", layout, ta, tb, m, n, k, alphas, A, a_off, lda, B, b_off, ldb, betas, C, c_off, ldc)


def gemm_batched(dtype, layout, ta, tb, m, n, k, alphas, A, a_off, lda, B, b_off, ldb, betas, C, c_off, ldc):
    """Batched oracle for FP32 ("f32") or FP16 storage ("f16", float16 arrays).  Returns (C_ref, D) of shape
    (batch, m, n)."""
    np_t = np.float32 if dtype == "f32" else np.float16
    A, B, C = _flat(A, np_t), _flat(B, np_t), _flat(C, np_t)
    alphas, betas = _flat(alphas, np.float32), _flat(betas, np.float32)
    a_off, b_off, c_off = (_flat(x, np.int64) for x in (a_off, b_off, c_off))
    batch = alphas.size
    assert betas.size == batch and a_off.size == batch and b_off.size == batch and c_off.size == batch
    if batch:
        assert a_off.min() >= 0 and b_off.min() >= 0 and c_off.min() >= 0
        assert a_off.max() + _need(layout, ta, m, k, lda) <= A.size, "A too short"
        assert b_off.max() + _need(layout, tb, k, n, ldb) <= B.size, "B too short"
        assert c_off.max() + _need(layout, NO_TRANS, m, n, ldc) <= C.size, "C too short"
    c_ref = np.empty((batch, m, n), dtype=np.float64)
    d_ref = np.empty((batch, m, n), dtype=np.float64)
    fn = lib().oracle_sgemm_batched if dtype == "f32" else lib().oracle_hgemm_batched
    fn(layout, ta, tb, m, n, k, _ptr(alphas), _ptr(A), _ptr(a_off), lda, _ptr(B), _ptr(b_off), ldb, _ptr(betas),
       _ptr(C), _ptr(c_off), ldc, batch, _ptr(c_ref), _ptr(d_ref))
    return c_ref, d_ref


def gemm_strided_batched(dtype, layout, ta, tb, m, n, k, alpha, A, lda, stride_a, B, ldb, stride_b, beta, C, ldc,
                         stride_c, batch):
    """Strided batched oracle for either storage type (see sgemm_strided_batched)."""
    idx = np.arange(batch, dtype=np.int64)
    return gemm_batched(dtype, layout, ta, tb, m, n, k, np.full(batch, alpha, dtype=np.float32), A, idx * stride_a,
                        lda, B, idx * stride_b, ldb, np.full(batch, beta, dtype=np.float32), C, idx * stride_c, ldc)


def sgemm_strided_batched(layout, ta, tb, m, n, k, alpha, A, lda, stride_a, B, ldb, stride_b, beta, C, ldc,
                          stride_c, batch):
    """Strided batched oracle.  Section 4.6 defines the strided routine as the generic one without the
    offset and scalar arrays: instance b sits at b*stride and every instance uses the same alpha, beta.
    That definition is written out here: the arrays are built and the generic oracle is called."""
    idx = np.arange(batch, dtype=np.int64)
    return sgemm_batched(layout, ta, tb, m, n, k, np.full(batch, alpha, dtype=np.float32), A, idx * stride_a, lda,
                         B, idx * stride_b, ldb, np.full(batch, beta, dtype=np.float32), C, idx * stride_c, ldc)


def gemv(dtype, layout, trans, m, n, alpha, A, lda, x, incx, beta, y, incy):
    """BLAS GEMV oracle: y_ref, d_ref (float64, length m or n).  A is m x n as stored; x, y flat with increments."""
    np_t = np.float32 if dtype == "f32" else np.float16
    rows, length = (m, n) if trans == NO_TRANS else (n, m)
    A, x, y = _flat(A, np_t), _flat(x, np_t), _flat(y, np_t)
    assert incx >= 1 and incy >= 1
    if alpha != 0 and rows and length:
        assert A.size >= _need(layout, NO_TRANS, m, n, lda), "A too short"
        assert x.size >= (length - 1) * incx + 1, "x too short"
    if beta != 0 and rows:
        assert y.size >= (rows - 1) * incy + 1, "y too short"
    y_ref = np.empty(rows, dtype=np.float64)
    d_ref = np.empty(rows, dtype=np.float64)
    lib().oracle_gemv(int(dtype == "f16"), layout, trans, m, n, float(alpha), _ptr(A), lda, _ptr(x), incx, float(beta),
                      _ptr(y), incy, _ptr(y_ref), _ptr(d_ref))
    return y_ref, d_ref


def half_to_double(bits):
    bits = _flat(bits, np.uint16)
    out = np.empty(bits.size, dtype=np.float64)
    lib().oracle_half_to_double(_ptr(bits), bits.size, _ptr(out))
    return out
