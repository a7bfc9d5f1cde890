"""GPU parity of the GEMM-derived level-3 routines (SYMM, SYRK, TRMM; paper Section 3.1, routine table)
against the CPU oracle, element by element, through the C ABI."""
import itertools

import numpy as np
import pytest

import helpers as H
from paper_1705_05249_amd import gemm as G
from paper_1705_05249_amd import workloads as W

pytestmark = pytest.mark.gpu

R, C, N, T = W.ROW_MAJOR, W.COL_MAJOR, W.NO_TRANS, W.TRANS
UP, LO, LEFT, RIGHT, UNIT, NONUNIT = W.UPPER, W.LOWER, W.LEFT, W.RIGHT, W.UNIT, W.NON_UNIT


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout,side,uplo", list(itertools.product([C, R], [LEFT, RIGHT], [UP, LO])))
@pytest.mark.parametrize("shape", [(1, 1), (33, 70), (200, 131), (256, 256)])
def test_symm_every_option(level3_oracle, dtype, layout, side, uplo, shape):
    m, n = shape
    case = W.level3_case("symm", dtype, layout, m, n, side=side, uplo=uplo, alpha=1.25, beta=-0.5, pad=(1, 2, 3),
                         case=m + n)
    H.check_level3(case, level3_oracle)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout,uplo,trans", list(itertools.product([C, R], [UP, LO], [N, T])))
@pytest.mark.parametrize("shape", [(1, 1), (70, 33), (131, 200), (256, 64)])
def test_syrk_every_option(level3_oracle, dtype, layout, uplo, trans, shape):
    n, k = shape
    case = W.level3_case("syrk", dtype, layout, n, n, k=k, uplo=uplo, trans=trans, alpha=-0.75, beta=1.5, pad=(2, 0, 1),
                         case=n + k)
    H.check_level3(case, level3_oracle)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout,side,uplo,trans,diag",
                         list(itertools.product([C, R], [LEFT, RIGHT], [UP, LO], [N, T], [NONUNIT, UNIT])))
@pytest.mark.parametrize("shape", [(1, 1), (45, 83), (256, 192)])
def test_trmm_every_option(level3_oracle, dtype, layout, side, uplo, trans, diag, shape):
    m, n = shape
    case = W.level3_case("trmm", dtype, layout, m, n, side=side, uplo=uplo, trans=trans, diag=diag, alpha=0.5,
                         pad=(3, 1, 0), case=m + n)
    H.check_level3(case, level3_oracle)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("routine", ["symm", "syrk", "trmm"])
def test_integer_inputs_are_exact(level3_oracle, dtype, routine):
    for layout, uplo, side in ((C, LO, LEFT), (R, UP, RIGHT)):
        case = W.level3_case(routine, dtype, layout, 130, 130 if routine == "syrk" else 97, k=77, side=side, uplo=uplo,
                             trans=T, alpha=2.0, beta=-1.0, pad=(1, 1, 1), integer=True, case=5)
        H.check_level3(case, level3_oracle)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_scalar_conventions(level3_oracle, dtype):
    """alpha == 0: A (and B) may hold NaN everywhere; beta == 0: C is overwritten even where it held NaN;
    k == 0: the rank-k update scales the triangle"""
    case = W.level3_case("symm", dtype, C, 40, 50, alpha=0.0, beta=0.5, case=1)
    case.A[:] = np.nan
    case.B[:] = np.nan
    H.check_level3(case, level3_oracle)
    case = W.level3_case("symm", dtype, R, 40, 50, side=RIGHT, uplo=LO, alpha=1.0, beta=0.0, case=2)
    case.C[~W.padding_mask(R, 40, 50, case.ldc, case.C.size)] = np.nan
    H.check_level3(case, level3_oracle)
    case = W.level3_case("syrk", dtype, C, 60, 60, k=0, uplo=LO, alpha=1.0, beta=2.0, case=3)
    H.check_level3(case, level3_oracle)
    case = W.level3_case("syrk", dtype, C, 60, 60, k=20, uplo=UP, alpha=0.0, beta=2.0, case=4)
    case.A[:] = np.nan
    H.check_level3(case, level3_oracle)
    case = W.level3_case("trmm", dtype, C, 30, 20, alpha=0.0, case=5)
    case.A[:] = np.nan
    H.check_level3(case, level3_oracle)


@pytest.mark.parametrize("routine,dtype,shape", [("symm", "f16", (1024, 768)), ("syrk", "f16", (1024, 512)),
                                                 ("trmm", "f16", (768, 1024)), ("symm", "f32", (1000, 333)),
                                                 ("syrk", "f32", (777, 1200)), ("trmm", "f32", (515, 640)),
                                                 ("symm", "f16", (1000, 520)), ("syrk", "f16", (1000, 136)),
                                                 ("trmm", "f16", (520, 1000))])
def test_sizes_that_span_many_tiles(level3_oracle, routine, dtype, shape):
    a, b = shape
    for layout, side, uplo, trans in ((C, LEFT, LO, N), (R, RIGHT, UP, T)):
        if routine == "syrk":
            case = W.level3_case("syrk", dtype, layout, a, a, k=b, uplo=uplo, trans=trans, alpha=1.0, beta=1.0, case=a)
        else:
            case = W.level3_case(routine, dtype, layout, a, b, side=side, uplo=uplo, trans=trans, alpha=1.0, beta=1.0, case=a)
        H.check_level3(case, level3_oracle)


def test_workspace_is_required():
    import torch
    case = W.level3_case("symm", "f32", C, 64, 64, alpha=1.0, beta=0.0)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    st, out = H.run_level3(case, workspace=small, check=False)
    assert st == -10 and np.array_equal(H.bits(out), H.bits(case.C))
    case = W.level3_case("trmm", "f32", C, 64, 64, alpha=1.0)
    only_a = torch.empty(64 * 64 * 4, dtype=torch.uint8, device="cuda")
    st, out = H.run_level3(case, workspace=only_a, check=False)
    assert st == -10 and np.array_equal(H.bits(out), H.bits(case.B))
    case = W.level3_case("syrk", "f16", C, 64, 64, k=8, alpha=1.0)
    st, out = H.run_level3(case, workspace=None, check=False)
    assert st == -10 and np.array_equal(H.bits(out), H.bits(case.C))


def _columns(flat, rows, ld, cols):
    """the chosen columns of a column-major matrix, tightly packed"""
    return np.ascontiguousarray(np.stack([flat[c * ld: c * ld + rows] for c in cols]).reshape(-1))


def test_benchmark_size_on_sampled_outputs(level3_oracle):
    """4096, FP16, column-major, lower, left: the calls the benchmark times, checked on sampled outputs.
    Columns of B (SYMM, TRMM) are independent problems, and so are the rows/columns of a rank-k update that
    belong to a subset of indices: the oracle computes those sub-problems in full."""
    n = 4096
    g = np.random.default_rng(77)
    cols = np.sort(g.choice(n, size=12, replace=False))
    case = W.level3_case("symm", "f16", C, n, n, side=LEFT, uplo=LO, alpha=1.0, beta=0.0, case=1)
    _, out = H.run_level3(case)
    ref, den = level3_oracle.symm("f16", C, LEFT, LO, n, len(cols), 1.0, case.A, case.lda,
                                  _columns(case.B, n, case.ldb, cols), n, 0.0, _columns(case.C, n, case.ldc, cols), n)
    got = np.stack([out[c * case.ldc: c * case.ldc + n] for c in cols], axis=1)
    assert H.rel_error(got, ref, den) <= H.TOL["f16"]

    case = W.level3_case("trmm", "f16", C, n, n, side=LEFT, uplo=LO, alpha=1.0, case=3)
    _, out = H.run_level3(case)
    ref, den = level3_oracle.trmm("f16", C, LEFT, LO, N, NONUNIT, n, len(cols), 1.0, case.A, case.lda,
                                  _columns(case.B, n, case.ldb, cols), n)
    got = np.stack([out[c * case.ldb: c * case.ldb + n] for c in cols], axis=1)
    assert H.rel_error(got, ref, den) <= H.TOL["f16"]

    case = W.level3_case("syrk", "f16", C, n, n, k=n, uplo=LO, alpha=1.0, beta=0.0, case=2)
    _, out = H.run_level3(case)
    pick = np.sort(g.choice(n, size=96, replace=False))
    A = W.unpack(case.A, C, n, n, case.lda)[pick]                       # the chosen rows of A: a 96 x k operand
    sub = W.pack(A, C, N)
    blank = np.zeros(len(pick) * len(pick), np.float16)
    ref, den = level3_oracle.syrk("f16", C, LO, N, len(pick), n, 1.0, sub, len(pick), 0.0, blank, len(pick))
    got = W.unpack(out, C, n, n, case.ldc)[np.ix_(pick, pick)]
    i, j = np.indices(got.shape)
    low = i >= j
    assert H.rel_error(got[low], ref[low], den[low]) <= H.TOL["f16"]
    old = W.unpack(case.C, C, n, n, case.ldc)[np.ix_(pick, pick)]
    assert np.array_equal(H.bits(np.ascontiguousarray(got[~low])), H.bits(np.ascontiguousarray(old[~low])))


def _with_forced_tile_kernel(case, level3_oracle, tag=None, suffix="_edge"):
    """Runs the case with a forced macro-tile kernel (default: the bounds-checked 64 x 64 one), so that the shape
    hint (narrowed K ranges for TRMM, skipped tiles for SYRK) is exercised in a chosen kernel family on a problem of
    several tiles.  The operand order the call ends up with decides which of the four kernels is legal."""
    tag = tag or ("smfma_64x64x32_w2x2" if case.dtype == "f32" else "hmfma_64x64x64_w2x2")
    try:
        for contig in ("mk", "kk", "mn", "kn"):
            G.mg_override_config(G.kernel_id(f"{tag}_{contig}{suffix}"), 1)
            st, _ = H.run_level3(case, check=False)
            if st == 0:
                return H.check_level3(case, level3_oracle)
            assert st == -11
        raise AssertionError("no macro-tile kernel accepted the problem")
    finally:
        G.mg_clear_override()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout,side,uplo,trans", list(itertools.product([C, R], [LEFT, RIGHT], [UP, LO], [N, T])))
def test_trmm_with_narrowed_k_ranges(level3_oracle, dtype, layout, side, uplo, trans):
    for diag, shape in ((NONUNIT, (200, 136)), (UNIT, (130, 260))):
        case = W.level3_case("trmm", dtype, layout, *shape, side=side, uplo=uplo, trans=trans, diag=diag, alpha=1.5,
                             pad=(1, 0, 2), case=17)
        _with_forced_tile_kernel(case, level3_oracle)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout,uplo,trans", list(itertools.product([C, R], [UP, LO], [N, T])))
def test_syrk_with_skipped_tiles(level3_oracle, dtype, layout, uplo, trans):
    case = W.level3_case("syrk", dtype, layout, 300, 300, k=100, uplo=uplo, trans=trans, alpha=1.0, beta=-2.0,
                         pad=(0, 0, 1), case=19)
    _with_forced_tile_kernel(case, level3_oracle)


@pytest.mark.parametrize("layout,side,uplo,trans", list(itertools.product([C, R], [LEFT, RIGHT], [UP, LO], [N, T])))
def test_trmm_hint_in_the_direct_to_lds_kernel(level3_oracle, layout, side, uplo, trans):
    """whole 256 x 256 tiles, FP16: the headline kernel family with narrowed K ranges (3 x 2 and 2 x 3 tiles)"""
    case = W.level3_case("trmm", "f16", layout, 768, 512, side=side, uplo=uplo, trans=trans, alpha=0.75, case=31)
    _with_forced_tile_kernel(case, level3_oracle, tag="hdma16_256x256x64_w2x4", suffix="")


@pytest.mark.parametrize("layout,uplo,trans", list(itertools.product([C, R], [UP, LO], [N, T])))
def test_syrk_hint_in_the_direct_to_lds_kernel(level3_oracle, layout, uplo, trans):
    case = W.level3_case("syrk", "f16", layout, 768, 768, k=192, uplo=uplo, trans=trans, alpha=1.0, beta=0.5, case=37)
    _with_forced_tile_kernel(case, level3_oracle, tag="hdma16_256x256x64_w2x4", suffix="")


@pytest.mark.parametrize("dtype,layout,side,uplo,trans", [("f16", C, LEFT, LO, N), ("f32", C, RIGHT, UP, N),
                                                          ("f16", R, LEFT, UP, T), ("f32", R, RIGHT, LO, T)])
def test_large_trmm_on_sampled_columns(level3_oracle, dtype, layout, side, uplo, trans):
    """many tiles of unequal work under automatic selection; 8 sampled columns (or, for a product from the right,
    rows) of B are independent problems the oracle solves in full"""
    n = 6144
    case = W.level3_case("trmm", dtype, layout, n, n, side=side, uplo=uplo, trans=trans, alpha=1.0, case=23)
    _, out = H.run_level3(case)
    g = np.random.default_rng(5)
    pick = np.sort(g.choice(n, size=8, replace=False))
    Bm = W.unpack(case.B, layout, n, n, case.ldb)
    got = W.unpack(out, layout, n, n, case.ldb)
    if side == LEFT:
        sub, want_shape = np.ascontiguousarray(Bm[:, pick]), (n, len(pick))
        got = got[:, pick]
    else:
        sub, want_shape = np.ascontiguousarray(Bm[pick, :]), (len(pick), n)
        got = got[pick, :]
    ld = W.tight_ld(layout, N, *want_shape)
    ref, den = level3_oracle.trmm(dtype, layout, side, uplo, trans, NONUNIT, *want_shape, 1.0, case.A, case.lda,
                                  W.pack(sub, layout, N, ld), ld)
    assert H.rel_error(got, ref, den) <= H.TOL[dtype]


@pytest.mark.parametrize("dtype,layout,uplo,trans", [("f16", C, LO, N), ("f32", R, LO, T), ("f16", R, UP, N)])
def test_large_syrk_on_sampled_entries(level3_oracle, dtype, layout, uplo, trans):
    n, k = 6144, 1024
    case = W.level3_case("syrk", dtype, layout, n, n, k=k, uplo=uplo, trans=trans, alpha=1.0, beta=0.0, case=29)
    _, out = H.run_level3(case)
    g = np.random.default_rng(6)
    pick = np.sort(g.choice(n, size=128, replace=False))
    stored = W.unpack(case.A, layout, *((n, k) if trans == N else (k, n)), case.lda)
    rows = stored[pick] if trans == N else stored[:, pick]
    ld = W.tight_ld(layout, N, *rows.shape)
    blank = np.zeros(len(pick) ** 2, np.float32 if dtype == "f32" else np.float16)
    ref, den = level3_oracle.syrk(dtype, layout, uplo, trans, len(pick), k, 1.0, W.pack(np.ascontiguousarray(rows), layout, N, ld),
                                  ld, 0.0, blank, len(pick))
    got = W.unpack(out, layout, n, n, case.ldc)[np.ix_(pick, pick)]
    old = W.unpack(case.C, layout, n, n, case.ldc)[np.ix_(pick, pick)]
    i, j = np.indices(got.shape)
    live = (i <= j) if uplo == UP else (i >= j)
    assert H.rel_error(got[live], ref[live], den[live]) <= H.TOL[dtype]
    assert np.array_equal(H.bits(np.ascontiguousarray(got[~live])), H.bits(np.ascontiguousarray(old[~live])))
