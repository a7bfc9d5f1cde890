"""Pins of the SYMM / SYRK / TRMM oracle (CPU only): numpy on explicitly built dense matrices, the
double-precision BLAS that scipy wraps, and closed forms.  The unreferenced triangle (and a unit
diagonal) always holds NaN, so reading the wrong half of a matrix fails every comparison."""
import itertools

import numpy as np
import pytest
import scipy.linalg.blas as blas

from oracle import level3_oracle as L3
from paper_1705_05249_amd import workloads as W

R, Cm, N, T = W.ROW_MAJOR, W.COL_MAJOR, W.NO_TRANS, W.TRANS
UP, LO, LEFT, RIGHT, UNIT, NONUNIT = L3.UPPER, L3.LOWER, L3.LEFT, L3.RIGHT, L3.UNIT, L3.NON_UNIT


def np_t(dtype):
    return np.float32 if dtype == "f32" else np.float16


def rand(g, shape, dtype):
    return g.uniform(-1, 1, size=shape).astype(np_t(dtype))


def keep_triangle(mat, uplo, unit=False):
    """copy with NaN outside the uplo triangle (and on the diagonal when it is an implicit one)"""
    out = mat.copy()
    n = mat.shape[0]
    i, j = np.indices((n, n))
    out[(i > j) if uplo == UP else (i < j)] = np.nan
    if unit:
        out[i == j] = np.nan
    return out


def store(mat, layout, pad):
    rows, cols = mat.shape
    ld = W.tight_ld(layout, N, rows, cols) + pad
    return W.pack(mat, layout, N, ld), ld


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout,side,uplo", list(itertools.product([Cm, R], [LEFT, RIGHT], [UP, LO])))
def test_symm_against_numpy(dtype, layout, side, uplo):
    m, n = 7, 5
    g = np.random.default_rng(100 + layout + side + uplo)
    ka = m if side == LEFT else n
    half = rand(g, (ka, ka), dtype).astype(np.float64)
    S = np.triu(half) + np.triu(half, 1).T
    A, lda = store(keep_triangle(S.astype(np_t(dtype)), uplo), layout, 2)
    Bm, Cmat = rand(g, (m, n), dtype), rand(g, (m, n), dtype)
    B, ldb = store(Bm, layout, 1)
    C, ldc = store(Cmat, layout, 3)
    c_ref, d_ref = L3.symm(dtype, layout, side, uplo, m, n, 1.5, A, lda, B, ldb, -0.5, C, ldc)
    S, B64, C64 = S.astype(np_t(dtype)).astype(np.float64), Bm.astype(np.float64), Cmat.astype(np.float64)
    want = 1.5 * (S @ B64 if side == LEFT else B64 @ S) - 0.5 * C64
    den = 1.5 * (np.abs(S) @ np.abs(B64) if side == LEFT else np.abs(B64) @ np.abs(S)) + 0.5 * np.abs(C64)
    assert np.max(np.abs(c_ref - want)) <= 1e-14 and np.max(np.abs(d_ref - den)) <= 1e-14


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout,uplo,trans", list(itertools.product([Cm, R], [UP, LO], [N, T])))
def test_syrk_against_numpy(dtype, layout, uplo, trans):
    n, k = 6, 9
    g = np.random.default_rng(200 + layout + uplo + trans)
    opA = rand(g, (n, k), dtype)
    A, lda = store(opA if trans == N else opA.T.copy(), layout, 2)
    Cmat = rand(g, (n, n), dtype)
    C, ldc = store(keep_triangle(Cmat, uplo), layout, 1)
    c_ref, d_ref = L3.syrk(dtype, layout, uplo, trans, n, k, -2.0, A, lda, 0.75, C, ldc)
    a64 = opA.astype(np.float64)
    want = -2.0 * (a64 @ a64.T) + 0.75 * Cmat.astype(np.float64)
    den = 2.0 * (np.abs(a64) @ np.abs(a64).T) + 0.75 * np.abs(Cmat.astype(np.float64))
    i, j = np.indices((n, n))
    inside = (i <= j) if uplo == UP else (i >= j)
    assert np.max(np.abs(c_ref[inside] - want[inside])) <= 1e-14 and np.max(np.abs(d_ref[inside] - den[inside])) <= 1e-14
    assert np.all(np.isnan(c_ref[~inside])) and np.all(d_ref[~inside] == 0)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout,side,uplo,trans,diag",
                         list(itertools.product([Cm, R], [LEFT, RIGHT], [UP, LO], [N, T], [NONUNIT, UNIT])))
def test_trmm_against_numpy(dtype, layout, side, uplo, trans, diag):
    m, n = 6, 8
    g = np.random.default_rng(300 + layout + side + uplo + trans + diag)
    ka = m if side == LEFT else n
    full = rand(g, (ka, ka), dtype)
    A, lda = store(keep_triangle(full, uplo, unit=diag == UNIT), layout, 1)
    Bm = rand(g, (m, n), dtype)
    B, ldb = store(Bm, layout, 2)
    b_ref, d_ref = L3.trmm(dtype, layout, side, uplo, trans, diag, m, n, 0.5, A, lda, B, ldb)
    Tm = (np.triu(full) if uplo == UP else np.tril(full)).astype(np.float64)
    if diag == UNIT:
        np.fill_diagonal(Tm, 1.0)
    op = Tm if trans == N else Tm.T
    B64 = Bm.astype(np.float64)
    want = 0.5 * (op @ B64 if side == LEFT else B64 @ op)
    den = 0.5 * (np.abs(op) @ np.abs(B64) if side == LEFT else np.abs(B64) @ np.abs(op))
    assert np.max(np.abs(b_ref - want)) <= 1e-14 and np.max(np.abs(d_ref - den)) <= 1e-14


def test_against_the_double_precision_blas():
    """column-major FP32 inputs widened exactly to FP64: dsymm / dsyrk / dtrmm compute the same sums"""
    g = np.random.default_rng(7)
    m, n, k = 9, 6, 11
    for side, uplo in itertools.product([LEFT, RIGHT], [UP, LO]):
        ka = m if side == LEFT else n
        half = rand(g, (ka, ka), "f32")
        S = np.triu(half) + np.triu(half, 1).T
        Bm, Cmat = rand(g, (m, n), "f32"), rand(g, (m, n), "f32")
        A, lda = store(keep_triangle(S, uplo), Cm, 0)
        B, ldb = store(Bm, Cm, 0)
        C, ldc = store(Cmat, Cm, 0)
        c_ref, _ = L3.symm("f32", Cm, side, uplo, m, n, 1.25, A, lda, B, ldb, 0.5, C, ldc)
        tri = np.triu(S) if uplo == UP else np.tril(S)
        want = blas.dsymm(1.25, np.asfortranarray(tri, dtype=np.float64), np.asfortranarray(Bm, dtype=np.float64), beta=0.5,
                          c=np.asfortranarray(Cmat, dtype=np.float64), side=int(side == RIGHT), lower=int(uplo == LO))
        assert np.max(np.abs(c_ref - want)) <= 1e-13
    for uplo, trans in itertools.product([UP, LO], [N, T]):
        opA = rand(g, (n, k), "f32")
        stored = opA if trans == N else opA.T.copy()
        A, lda = store(stored, Cm, 0)
        Cmat = rand(g, (n, n), "f32")
        C, ldc = store(keep_triangle(Cmat, uplo), Cm, 0)
        c_ref, _ = L3.syrk("f32", Cm, uplo, trans, n, k, 0.75, A, lda, -1.5, C, ldc)
        want = blas.dsyrk(0.75, np.asfortranarray(stored, dtype=np.float64), beta=-1.5,
                          c=np.asfortranarray(Cmat, dtype=np.float64), trans=int(trans == T), lower=int(uplo == LO))
        i, j = np.indices((n, n))
        inside = (i <= j) if uplo == UP else (i >= j)
        assert np.max(np.abs(c_ref[inside] - want[inside])) <= 1e-13
    for side, uplo, trans, diag in itertools.product([LEFT, RIGHT], [UP, LO], [N, T], [NONUNIT, UNIT]):
        ka = m if side == LEFT else n
        full = rand(g, (ka, ka), "f32")
        Bm = rand(g, (m, n), "f32")
        A, lda = store(keep_triangle(full, uplo, unit=diag == UNIT), Cm, 0)
        B, ldb = store(Bm, Cm, 0)
        b_ref, _ = L3.trmm("f32", Cm, side, uplo, trans, diag, m, n, -0.5, A, lda, B, ldb)
        want = blas.dtrmm(-0.5, np.asfortranarray(full, dtype=np.float64), np.asfortranarray(Bm, dtype=np.float64),
                          side=int(side == RIGHT), lower=int(uplo == LO), trans_a=int(trans == T), diag=int(diag == UNIT))
        assert np.max(np.abs(b_ref - want)) <= 1e-13


def test_closed_forms():
    n, k = 5, 7
    ones_tri = keep_triangle(np.ones((n, n), np.float32), LO)
    Bm = np.arange(1, n * 3 + 1, dtype=np.float32).reshape(n, 3)
    # a lower triangle of ones from the left makes running sums down each column
    b_ref, d_ref = L3.trmm("f32", Cm, LEFT, LO, N, NONUNIT, n, 3, 1.0, *store(ones_tri, Cm, 0), *store(Bm, Cm, 0))
    assert np.array_equal(b_ref, np.cumsum(Bm.astype(np.float64), axis=0)) and np.array_equal(d_ref, b_ref)
    # ... and transposed, running sums from the bottom
    b_ref, _ = L3.trmm("f32", Cm, LEFT, LO, T, NONUNIT, n, 3, 1.0, *store(ones_tri, Cm, 0), *store(Bm, Cm, 0))
    assert np.array_equal(b_ref, np.cumsum(Bm[::-1].astype(np.float64), axis=0)[::-1])
    # unit diagonal and nothing else: alpha * B
    eye = keep_triangle(np.zeros((n, n), np.float32), UP, unit=True)
    b_ref, _ = L3.trmm("f32", R, LEFT, UP, N, UNIT, n, 3, 3.0, *store(eye, R, 2), *store(Bm, R, 1))
    assert np.array_equal(b_ref, 3.0 * Bm)
    # symmetric identity: alpha * B + beta * C
    ident = keep_triangle(np.eye(n, dtype=np.float32), UP)
    Cmat = np.full((n, 3), 2.0, np.float32)
    c_ref, d_ref = L3.symm("f32", Cm, LEFT, UP, n, 3, 2.0, *store(ident, Cm, 0), *store(Bm, Cm, 0), -1.0, *store(Cmat, Cm, 0))
    assert np.array_equal(c_ref, 2.0 * Bm - 2.0) and np.array_equal(d_ref, 2.0 * Bm + 2.0)
    # rank-k update with a matrix of ones: every referenced entry is alpha * k + beta * c
    c_ref, _ = L3.syrk("f32", Cm, UP, N, n, k, 0.5, *store(np.ones((n, k), np.float32), Cm, 0), 2.0,
                       *store(keep_triangle(np.full((n, n), 3.0, np.float32), UP), Cm, 0))
    i, j = np.indices((n, n))
    assert np.all(c_ref[i <= j] == 0.5 * k + 6.0)


def test_scalar_conventions():
    n = 4
    nan = np.full((n, n), np.nan, np.float32)
    Cmat = np.arange(16, dtype=np.float32).reshape(n, n)
    # alpha == 0: A and B are not read
    c_ref, _ = L3.symm("f32", Cm, LEFT, UP, n, n, 0.0, *store(nan, Cm, 0), *store(nan, Cm, 0), 2.0, *store(Cmat, Cm, 0))
    assert np.array_equal(c_ref, 2.0 * Cmat)
    # beta == 0: C is not read
    c_ref, _ = L3.symm("f32", Cm, LEFT, UP, n, n, 1.0, *store(np.triu(np.ones((n, n), np.float32)), Cm, 0),
                       *store(np.ones((n, n), np.float32), Cm, 0), 0.0, *store(nan, Cm, 0))
    assert np.array_equal(c_ref, np.full((n, n), 4.0))
    c_ref, _ = L3.syrk("f32", Cm, LO, N, n, 3, 1.0, *store(np.ones((n, 3), np.float32), Cm, 0), 0.0, *store(nan, Cm, 0))
    i, j = np.indices((n, n))
    assert np.all(c_ref[i >= j] == 3.0)
    b_ref, _ = L3.trmm("f32", Cm, RIGHT, UP, N, NONUNIT, n, n, 0.0, *store(nan, Cm, 0), *store(nan, Cm, 0))
    assert np.array_equal(b_ref, np.zeros((n, n)))
