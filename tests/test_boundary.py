"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and turns every invalid argument into its status code before touching HIP."""
import ctypes
import os
import re

import pytest

from paper_1705_05249_amd import gemm as G

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
R, C, N, T = G.MG_ROW_MAJOR, G.MG_COL_MAJOR, G.MG_NO_TRANS, G.MG_TRANS
FAKE = 0x1000          # never dereferenced: every call below fails validation or returns early


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mg_gemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mg_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = declared_symbols()
    assert set(names) == set(G.EXPORTS)
    lib = G.lib()
    for name in names:
        assert getattr(lib, name) is not None


def sgemm(layout=C, ta=N, tb=N, m=4, n=5, k=6, lda=None, ldb=None, ldc=None, A=FAKE, B=FAKE, Cp=FAKE,
          alpha=1.0, beta=0.0, fn=None):
    col = layout == C
    lda = lda if lda is not None else max(1, (m if ta == N else k) if col else (k if ta == N else m))
    ldb = ldb if ldb is not None else max(1, (k if tb == N else n) if col else (n if tb == N else k))
    ldc = ldc if ldc is not None else max(1, m if col else n)
    fn = fn or G.mg_sgemm
    return fn(layout, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, Cp, ldc, None, 0, check=False)


@pytest.mark.parametrize("fn", [G.mg_sgemm, G.mg_hgemm])
def test_argument_errors(fn):
    assert sgemm(layout=100, fn=fn) == -1
    assert sgemm(ta=110, fn=fn) == -2
    assert sgemm(tb=114, fn=fn) == -3
    assert sgemm(layout=100, ta=0, fn=fn) == -1            # reported in status-code order
    assert sgemm(m=-1, fn=fn) == -4
    assert sgemm(n=-1, fn=fn) == -4
    assert sgemm(k=-1, fn=fn) == -4
    assert sgemm(m=2 ** 31, lda=2 ** 31, ldc=2 ** 31, fn=fn) == -4
    for layout in (R, C):
        for ta in (N, T):
            for tb in (N, T):
                col = layout == C
                a_lead = (4 if ta == N else 6) if col else (6 if ta == N else 4)
                b_lead = (6 if tb == N else 5) if col else (5 if tb == N else 6)
                c_lead = 4 if col else 5
                assert sgemm(layout, ta, tb, lda=a_lead - 1, fn=fn) == -5
                assert sgemm(layout, ta, tb, ldb=b_lead - 1, fn=fn) == -6
                assert sgemm(layout, ta, tb, ldc=c_lead - 1, fn=fn) == -7
    assert sgemm(lda=0, m=0, fn=fn) == -5                  # ld >= 1 even for empty matrices
    assert sgemm(A=None, fn=fn) == -8
    assert sgemm(B=None, fn=fn) == -8
    assert sgemm(Cp=None, fn=fn) == -8
    assert sgemm(ta=G.MG_CONJ_TRANS, m=0, fn=fn) == 0       # conj-trans accepted


@pytest.mark.parametrize("fn", [G.mg_sgemm, G.mg_hgemm])
def test_quick_returns_launch_nothing(fn):
    assert sgemm(m=0, A=None, B=None, Cp=None, fn=fn) == 0
    assert sgemm(n=0, A=None, B=None, Cp=None, fn=fn) == 0


def batched(m=4, n=4, k=4, batch=3, alphas=FAKE, betas=FAKE, A=FAKE, B=FAKE, Cp=FAKE, ao=FAKE, bo=FAKE, co=FAKE,
            layout=C, ta=N, tb=N, lda=4, ldb=4, ldc=4, fn=None):
    return (fn or G.mg_sgemm_batched)(layout, ta, tb, m, n, k, alphas, A, ao, lda, B, bo, ldb, betas, Cp, co, ldc, batch, stream=0,
                              check=False)


@pytest.mark.parametrize("fn", [G.mg_sgemm_batched, G.mg_hgemm_batched])
def test_batched_argument_errors(fn):
    batched = lambda **kw: globals()["batched"](fn=fn, **kw)
    assert batched(layout=7) == -1
    assert batched(ta=1) == -2
    assert batched(tb=1) == -3
    assert batched(k=-2) == -4
    assert batched(lda=3) == -5
    assert batched(ldb=3) == -6
    assert batched(ldc=3) == -7
    assert batched(batch=-1) == -9
    for name in ("alphas", "betas", "A", "B", "Cp", "ao", "bo", "co"):
        assert batched(**{name: None}) == -8
    assert batched(batch=0, alphas=None, A=None) == 0
    assert batched(m=0, alphas=None, A=None) == 0


def strided(m=4, n=4, k=4, batch=3, A=FAKE, B=FAKE, Cp=FAKE, sa=16, sb=16, sc=16, layout=C, ta=N, tb=N, lda=4, ldb=4,
            ldc=4, alpha=1.0, beta=1.0, fn=None):
    return (fn or G.mg_sgemm_strided_batched)(layout, ta, tb, m, n, k, alpha, A, lda, sa, B, ldb, sb, beta, Cp, ldc, sc, batch,
                                      stream=0, check=False)


@pytest.mark.parametrize("fn", [G.mg_sgemm_strided_batched, G.mg_hgemm_strided_batched])
def test_strided_batched_argument_errors(fn):
    strided = lambda **kw: globals()["strided"](fn=fn, **kw)
    assert strided(layout=7) == -1
    assert strided(ta=1) == -2
    assert strided(tb=1) == -3
    assert strided(m=-1) == -4
    assert strided(lda=3) == -5
    assert strided(ldb=3) == -6
    assert strided(ldc=3) == -7
    assert strided(batch=-1) == -9
    assert strided(sa=-1) == -14 and strided(sb=-1) == -14 and strided(sc=-1) == -14
    assert strided(A=None) == -8 and strided(B=None) == -8 and strided(Cp=None) == -8
    assert strided(batch=0, A=None, Cp=None) == 0
    assert strided(n=0, A=None, Cp=None) == 0


GEOM = dict(channels=3, height=8, width=9, kernel=(3, 3), pad=(1, 1), stride=(1, 1), dilation=(1, 1))


def conv(fn=None, filters=4, im=FAKE, weights=FAKE, out=FAKE, ws=None, ws_bytes=None, alpha=1.0, beta=0.0, **over):
    g = dict(GEOM, **over)
    name = fn or "mg_sconv2d"
    args = G._geometry(g["channels"], g["height"], g["width"], g["kernel"], g["pad"], g["stride"], g["dilation"])
    need = G.mg_conv2d_workspace_bytes(G.MG_F32, g["channels"], g["height"], g["width"], g["kernel"], g["pad"],
                                       g["stride"], g["dilation"], filters)
    ws_addr = (256 if ws is None else ws)
    return getattr(G.lib(), name)(*args, filters, alpha, im, weights, beta, out, ws_addr,
                                  need if ws_bytes is None else ws_bytes, 0)


@pytest.mark.parametrize("fn", ["mg_sconv2d", "mg_hconv2d"])
def test_conv_argument_errors(fn):
    """geometry and pointer errors are reported before any GPU work (no GPU here)"""
    for bad in (dict(channels=0), dict(height=0), dict(width=-1), dict(kernel=(0, 3)), dict(kernel=(3, 0)),
                dict(pad=(-1, 0)), dict(pad=(0, -1)), dict(stride=(0, 1)), dict(stride=(1, 0)),
                dict(dilation=(0, 1)), dict(dilation=(1, 0))):
        assert conv(fn, **bad) == -15, bad
    assert conv(fn, filters=-1) == -15
    assert conv(fn, height=1 << 20, width=1 << 20) == -4                  # column matrix beyond 2^31 elements
    # an image plane, a padded extent or a filter reach that a 32-bit index cannot hold (the output itself is small)
    assert conv(fn, height=1 << 16, width=1 << 15, kernel=(1, 1), stride=(1 << 12, 1 << 12)) == -4
    assert conv(fn, pad=((1 << 30) + 5, 0), stride=(1 << 30, 1)) == -4
    assert conv(fn, dilation=(1 << 30, 1), pad=(1 << 30, 0), stride=(1 << 30, 1)) == -4
    assert conv(fn, im=None) == -8 and conv(fn, weights=None) == -8 and conv(fn, out=None) == -8
    assert conv(fn, ws=0) == -10 and conv(fn, ws=264) == -10 and conv(fn, ws_bytes=255) == -10
    # empty outputs launch nothing: no filters, or a filter that does not fit the image
    assert conv(fn, filters=0, im=None, weights=None, out=None) == 0
    assert conv(fn, kernel=(9, 3), pad=(0, 0), im=None, weights=None, out=None) == 0


def test_im2col_argument_errors_and_geometry_queries():
    L = G.lib()
    args = G._geometry(**GEOM)
    for fn in (L.mg_sim2col, L.mg_him2col):
        assert fn(*args, None, FAKE, 0) == -8 and fn(*args, FAKE, None, 0) == -8
        assert fn(*G._geometry(**dict(GEOM, stride=(0, 1))), FAKE, FAKE, 0) == -15
        assert fn(*G._geometry(**dict(GEOM, kernel=(9, 9), pad=(0, 0))), None, None, 0) == 0      # empty output
    assert G.mg_conv2d_out_extent(224, 7, 3, 2, 1) == 112 and G.mg_conv2d_out_extent(5, 3, 0, 2, 1) == 2
    assert G.mg_conv2d_out_extent(2, 5, 0, 1, 1) == 0 and G.mg_conv2d_out_extent(5, 3, 0, 0, 1) == -1
    # workspace: the column matrix rounded up to 256 bytes (+ split-K scratch of the GEMM, none here)
    assert G.mg_conv2d_workspace_bytes(G.MG_F16, 3, 224, 224, (7, 7), (3, 3), (2, 2), (1, 1), 64) == 147 * 12544 * 2
    assert G.mg_conv2d_workspace_bytes(G.MG_F32, 3, 8, 9, (3, 3), (1, 1), (1, 1), (1, 1), 4) == 7936      # 27 * 72 * 4 = 7776, rounded up to a multiple of 256
    # a 1x1 filter with unit stride and no padding needs no column matrix
    assert G.mg_conv2d_workspace_bytes(G.MG_F32, 16, 8, 8, (1, 1), (0, 0), (1, 1), (1, 1), 8) == 0
    assert G.mg_conv2d_workspace_bytes(G.MG_F32, 16, 8, 8, (1, 1), (0, 0), (2, 1), (1, 1), 8) > 0
    assert G.mg_conv2d_workspace_bytes(7, 3, 8, 9, (3, 3), (1, 1), (1, 1), (1, 1), 4) == 0


@pytest.mark.parametrize("fn", ["mg_sgemv", "mg_hgemv"])
def test_gemv_argument_errors(fn):
    """every rejected call returns before anything touches a device"""
    f = getattr(G.lib(), fn)

    def call(layout=C, trans=N, m=4, n=3, A=FAKE, lda=4, x=FAKE, incx=1, y=FAKE, incy=1, alpha=1.0, beta=0.0):
        return f(layout, trans, m, n, alpha, A, lda, x, incx, beta, y, incy, None, 0, None)

    assert call(layout=7) == -1 and call(trans=5) == -2
    assert call(m=-1) == -4 and call(n=-1) == -4 and call(m=1 << 31) == -4
    assert call(lda=3) == -5 and call(layout=R, lda=2) == -5 and call(layout=R, lda=3, m=0) == 0
    assert call(incx=0) == -16 and call(incy=0) == -16 and call(incx=-1) == -16
    # more than 2^40 elements between the first and the last one of the matrix or of a vector
    assert call(m=4, n=1 << 30, lda=1 << 20) == -4 and call(m=1 << 30, n=2, lda=1 << 30, incx=1 << 12) == -4
    assert call(y=None) == -8 and call(A=None) == -8 and call(x=None) == -8
    # no output: nothing to do, whatever the pointers are
    assert call(m=0, lda=1, A=None, x=None, y=None) == 0
    assert call(trans=T, n=0, A=None, x=None, y=None) == 0


def test_gemv_workspace_query():
    """few outputs and a long sum ask for room for the partial sums; many outputs, or bad arguments, for none"""
    assert G.mg_gemv_workspace_bytes(G.MG_F32, C, N, 1 << 17, 1 << 12, 1 << 17) == 0
    few = G.mg_gemv_workspace_bytes(G.MG_F32, C, N, 4096, 1 << 15, 4096)
    assert few > 0 and few % (4096 * 4) == 0 and few <= 256 * 4096 * 4
    assert G.mg_gemv_workspace_bytes(G.MG_F16, C, T, 1 << 16, 16, 1 << 16) == 32 * 16 * 4     # 65536 / (4 * 512): 32 slices of four rounds each
    assert G.mg_gemv_workspace_bytes(G.MG_F32, C, N, 4096, 1 << 15, 100) == 0
    assert G.mg_gemv_workspace_bytes(9, C, N, 4096, 1 << 15, 4096) == 0


def test_level3_argument_errors():
    """SYMM / SYRK / TRMM: every rejected call returns before anything touches a device"""
    L = G.lib()
    UP, LO, LEFT, RIGHT, NU, UN = G.MG_UPPER, G.MG_LOWER, G.MG_LEFT, G.MG_RIGHT, G.MG_NON_UNIT, G.MG_UNIT
    for fn in (L.mg_ssymm, L.mg_hsymm):
        def symm(layout=C, side=LEFT, uplo=UP, m=4, n=3, A=FAKE, lda=4, B=FAKE, ldb=4, Cp=FAKE, ldc=4, alpha=1.0, ws=None):
            return fn(layout, side, uplo, m, n, alpha, A, lda, B, ldb, 0.0, Cp, ldc, ws, 0, None)
        assert symm(layout=5) == -1 and symm(side=7) == -17 and symm(uplo=0) == -18
        assert symm(m=-1) == -4 and symm(lda=3) == -5 and symm(side=RIGHT, lda=2) == -5 and symm(side=RIGHT, lda=3) == -10
        assert symm(ldb=3) == -6 and symm(ldc=3) == -7 and symm(layout=R, ldb=3, ldc=3) == -10
        assert symm(Cp=None) == -8 and symm(A=None) == -8 and symm(B=None) == -8
        assert symm(m=0, A=None, B=None, Cp=None, lda=1, ldb=1, ldc=1) == 0
        assert symm() == -10 and symm(ws=FAKE) == -10        # no workspace / misaligned and too small
    for fn in (L.mg_ssyrk, L.mg_hsyrk):
        def syrk(layout=C, uplo=LO, trans=N, n=4, k=3, A=FAKE, lda=4, Cp=FAKE, ldc=4, ws=None):
            return fn(layout, uplo, trans, n, k, 1.0, A, lda, 0.0, Cp, ldc, ws, 0, None)
        assert syrk(layout=5) == -1 and syrk(uplo=9) == -18 and syrk(trans=0) == -2 and syrk(n=-1) == -4 and syrk(k=-1) == -4
        assert syrk(lda=3) == -5 and syrk(trans=T, lda=3) == -10 and syrk(trans=T, lda=2) == -5
        assert syrk(layout=R, lda=3) == -10 and syrk(layout=R, lda=2) == -5 and syrk(ldc=3) == -7
        assert syrk(Cp=None) == -8 and syrk(A=None) == -8 and syrk(n=0, A=None, Cp=None, lda=1, ldc=1) == 0
    for fn in (L.mg_strmm, L.mg_htrmm):
        def trmm(layout=C, side=LEFT, uplo=UP, trans=N, diag=NU, m=4, n=3, A=FAKE, lda=4, B=FAKE, ldb=4, ws=None):
            return fn(layout, side, uplo, trans, diag, m, n, 1.0, A, lda, B, ldb, ws, 0, None)
        assert trmm(layout=5) == -1 and trmm(side=0) == -17 and trmm(uplo=0) == -18 and trmm(trans=0) == -2 and trmm(diag=0) == -19
        assert trmm(m=-1) == -4 and trmm(lda=3) == -5 and trmm(ldb=3) == -6 and trmm(diag=UN) == -10
        assert trmm(B=None) == -8 and trmm(A=None) == -8 and trmm(n=0, A=None, B=None) == 0


def test_level3_workspace_queries():
    F32, F16 = G.MG_F32, G.MG_F16
    assert G.mg_symm_workspace_bytes(F32, C, G.MG_LEFT, 100, 7) == 40192          # 100 * 100 * 4 = 40000 rounded up to 256
    assert G.mg_symm_workspace_bytes(F16, R, G.MG_RIGHT, 100, 7) == 256            # 7 * 7 * 2
    assert G.mg_syrk_workspace_bytes(F16, C, N, 64, 5) == 64 * 64 * 2
    assert G.mg_trmm_workspace_bytes(F32, C, G.MG_LEFT, T, 64, 32) == 64 * 64 * 4 + 64 * 32 * 4
    assert G.mg_symm_workspace_bytes(F32, C, 0, 100, 7) == 0 and G.mg_symm_workspace_bytes(9, C, G.MG_LEFT, 100, 7) == 0
    assert G.mg_syrk_workspace_bytes(F32, C, N, 0, 5) == 0 and G.mg_trmm_workspace_bytes(F32, 3, G.MG_LEFT, N, 4, 4) == 0
    # a short, wide product adds room for the split sum of the GEMM behind it
    assert G.mg_syrk_workspace_bytes(F32, C, N, 64, 1 << 16) > 64 * 64 * 4


def test_status_strings_and_version():
    seen = set()
    for code in range(0, -20, -1):
        s = G.status_string(code)
        assert s and s != "unknown status" and s not in seen
        seen.add(s)
    assert G.status_string(-99) == "unknown status"
    assert re.fullmatch(r"\d+\.\d+", G.mg_version())


def test_kernel_table_and_override_validation():
    table = G.kernel_table()
    assert len(table) == G.mg_kernel_count() >= 5
    assert len({t["name"] for t in table}) == len(table)
    for i, t in enumerate(table):
        assert t["kernel_id"] == i and t["dtype"] in (G.MG_F32, G.MG_F16) and t["split_k"] == 1
    assert G.mg_kernel_name(-1) == "?" and G.mg_kernel_name(10 ** 6) == "?"
    cfg = G.mg_config()
    assert G.lib().mg_kernel_info(len(table), ctypes.byref(cfg)) == -11
    assert G.mg_override_config(-1, 1, check=False) == -11
    assert G.mg_override_config(0, 0, check=False) == -11
    batched_ids = [t["kernel_id"] for t in table if t["family"] == G.MG_FAMILY_BATCHED]
    plain_ids = [t["kernel_id"] for t in table if t["family"] != G.MG_FAMILY_BATCHED]
    assert G.mg_override_config(batched_ids[0], 1, check=False) == -11
    assert G.mg_override_batched_config(plain_ids[0], check=False) == -11
    G.mg_clear_override()


def test_query_selected_and_override_roundtrip():
    try:
        sel = G.mg_query_selected(G.MG_F32, C, N, N, 256, 256, 256, 256, 256, 256, 1.5, 0.5)
        assert sel["dtype"] == G.MG_F32 and sel["family"] in (G.MG_FAMILY_DIRECT, G.MG_FAMILY_MFMA)
        scale = G.mg_query_selected(G.MG_F16, R, T, N, 64, 64, 64, 64, 64, 64, 0.0, 2.0)
        assert scale["family"] == G.MG_FAMILY_SCALE and scale["dtype"] == G.MG_F16
        direct = G.kernel_id("direct_f32_64x64x16")
        G.mg_override_config(direct, 1)
        forced = G.mg_query_selected(G.MG_F32, C, N, N, 4096, 4096, 4096, 4096, 4096, 4096)
        assert forced["kernel_id"] == direct
        # the FP32 override does not leak into FP16 calls
        other = G.mg_query_selected(G.MG_F16, C, N, N, 4096, 4096, 4096, 4096, 4096, 4096)
        assert other["dtype"] == G.MG_F16
        # a forced kernel that is illegal for the call is an error, not a silent fallback
        assert G.mg_override_config(direct, 4, check=False) == 0
        cfg = G.mg_config()
        st = G.lib().mg_query_selected(G.MG_F32, C, N, N, 64, 64, 64, 64, 64, 64, 1.0, 0.0, 256, ctypes.byref(cfg))
        assert st == -11
    finally:
        G.mg_clear_override()
    assert G.mg_gemm_workspace_bytes(G.MG_F32, C, N, N, 4096, 4096, 4096, 4096, 4096, 4096) == 0
    # few tiles and a long K: split-K is selected, and the query says how much scratch it needs
    sel = G.mg_query_selected(G.MG_F16, C, N, N, 512, 196, 4608, 512, 4608, 512)
    need = G.mg_gemm_workspace_bytes(G.MG_F16, C, N, N, 512, 196, 4608, 512, 4608, 512)
    assert sel["split_k"] > 1 and need == sel["split_k"] * 512 * 196 * 4
    # a sum short enough for the kernel whose eight wavefronts share it: one launch, no scratch
    sel = G.mg_query_selected(G.MG_F16, C, N, N, 512, 196, 2304, 512, 2304, 512)
    assert sel["name"] == "htiny_32x32_mk" and sel["split_k"] == 1
    assert G.mg_gemm_workspace_bytes(G.MG_F16, C, N, N, 512, 196, 2304, 512, 2304, 512) == 0
    assert G.mg_gemm_workspace_bytes(G.MG_F32, 0, N, N, 256, 256, 256, 256, 256, 256) == 0


def test_fringe_planning_and_override():
    """the fringe (last rows / columns of C computed beside the tiles) is a property of the column-major view of an
    FP32 call; the query reports it, the override switches it"""
    def q(layout, m, n, k, **kw):
        lda, ldb, ldc = (k, n, n) if layout == R else (k, k, m)          # A transposed (col) / plain (row), tight
        return G.mg_query_selected(kw.get("dtype", G.MG_F32), layout, T if layout == C else N, N, m, n, k, lda, ldb, ldc, 1.0, 1.0)
    try:
        G.mg_clear_override()
        sel = q(C, 4097, 129, 4095)
        assert sel["fringe"] == 16 * 1 + 1 and sel["name"].endswith("_edge") and sel["family"] == G.MG_FAMILY_MFMA
        assert q(R, 4096, 131, 4096)["fringe"] == 16 * 3             # row-major: the columns of C are the view's rows
        assert q(C, 4096, 4096, 4096)["fringe"] == 0                 # whole tiles
        assert q(C, 4101, 129, 4095)["fringe"] == 1                  # five beyond a multiple of 64: tiled
        assert q(C, 4097, 129, 128)["fringe"] == 0                   # short sum: bound by memory, not worth it
        assert q(C, 8193, 129, 4096)["fringe"] == 1                  # one tile row in 129: too small a saving
        assert q(C, 4097, 129, 4095, dtype=G.MG_F16)["fringe"] == 0  # FP32 only
        need_auto = G.mg_gemm_workspace_bytes(G.MG_F32, C, T, N, 4097, 129, 4095, 4095, 4095, 4097)
        G.mg_override_fringe(G.MG_FRINGE_OFF)
        assert q(C, 4097, 129, 4095)["fringe"] == 0
        G.mg_override_fringe(G.MG_FRINGE_ON)
        assert q(C, 4097, 129, 128)["fringe"] == 17 and q(C, 8193, 129, 4096)["fringe"] == 17
        assert q(C, 4097, 40, 4096)["fringe"] == 0                   # fewer than 64 columns: nothing left to tile
        # a forced kernel that cannot leave a fringe aside refuses the call instead of dropping it silently
        G.mg_override_config(G.kernel_id("direct_f32_64x64x16"), 1)
        cfg = G.mg_config()
        st = G.lib().mg_query_selected(G.MG_F32, C, T, N, 4097, 129, 4095, 4095, 4095, 4097, 1.0, 1.0, 256, ctypes.byref(cfg))
        assert st == -11
        G.mg_override_fringe(G.MG_FRINGE_AUTO)
        assert q(C, 4097, 129, 4095)["fringe"] == 0                  # automatic mode leaves a forced kernel's problem whole
        assert G.mg_override_fringe(3, check=False) == -11 and G.mg_override_fringe(-1, check=False) == -11
    finally:
        G.mg_clear_override()
    assert need_auto % (4097 * 129 * 4) == 0                         # partial sums cover all of C, fringe included
