"""Shared plumbing of the GPU parity tests: move a seeded case to the GPU, call the C ABI through
the Python binding, bring C back, compare with the CPU oracle element by element."""
import numpy as np

from paper_1705_05249_amd import workloads as W

TOL = {"f32": 1e-5, "f16": 2e-3}        # max |C - C_ref| / (|alpha| |A||B| + |beta| |C|)


from paper_1705_05249_amd.measure import rel_error, to_gpu  # noqa: E402,F401  (re-exported for the tests)


def workspace_for(case):
    import torch
    from paper_1705_05249_amd import gemm as G
    need = G.mg_gemm_workspace_bytes(G.MG_F32 if case.dtype == "f32" else G.MG_F16, case.layout, case.ta, case.tb,
                                     case.m, case.n, case.k, case.lda, case.ldb, case.ldc)
    return torch.empty(max(need, 256), dtype=torch.uint8, device="cuda") if need else None


def run_gpu(case, workspace="auto", check=True, offset_elems=(0, 0, 0)):
    """Runs one GemmCase; returns (status, flat C buffer after the call as numpy).
    offset_elems shifts the three base pointers inside larger allocations (alignment tests)."""
    import torch
    from paper_1705_05249_amd import gemm as G
    fn = G.mg_sgemm if case.dtype == "f32" else G.mg_hgemm
    bufs = []
    for arr, off in zip((case.A, case.B, case.C), offset_elems):
        host = arr if arr.size else np.zeros(1, dtype=arr.dtype)
        if off:
            host = np.concatenate([np.zeros(off, dtype=arr.dtype), host])
        bufs.append(to_gpu(host))
    views = [b[off:] for b, off in zip(bufs, offset_elems)]
    ws = workspace_for(case) if isinstance(workspace, str) else workspace
    st = fn(case.layout, case.ta, case.tb, case.m, case.n, case.k, case.alpha, views[0], case.lda, views[1],
            case.ldb, case.beta, views[2], case.ldc, ws, None, check=check)
    torch.cuda.synchronize()
    out = views[2].cpu().numpy()[: case.C.size]
    return st, out


def bits(a):
    return a.view(np.uint32 if a.dtype == np.float32 else np.uint16)


def assert_padding_untouched(case, out):
    mask = W.padding_mask(case.layout, case.m, case.n, case.ldc, case.C.size)
    assert np.array_equal(bits(out)[mask], bits(case.C)[mask]), f"{case.name}: bytes outside C were written"



def check_case(case, oracle, sampled=False, workspace="auto", offset_elems=(0, 0, 0), seed=1, sample=None):
    """Full (or sampled) element-by-element comparison of one case against the oracle; `sample`: keyword
    arguments for the choice of sampled entries (fewer complete rows and columns on the largest problems)."""
    st, out = run_gpu(case, workspace=workspace, offset_elems=offset_elems)
    assert st == 0
    assert_padding_untouched(case, out)
    got = W.unpack(out, case.layout, case.m, case.n, case.ldc)
    args = (case.dtype, case.layout, case.ta, case.tb, case.m, case.n, case.k, case.alpha, case.A, case.lda,
            case.B, case.ldb, case.beta, case.C, case.ldc)
    if sampled:
        rows, cols = W.sample_entries(case.m, case.n, seed=seed, **(sample or {}))
        c_ref, d_ref = oracle.gemm_entries(*args, rows, cols)
        got = got[rows, cols]
    else:
        c_ref, d_ref = oracle.gemm(*args)
    if case.exact:
        assert np.array_equal(got.astype(np.float64), c_ref), f"{case.name}: not bit-exact on integer inputs"
        return 0.0
    err = rel_error(got, c_ref, d_ref)
    assert err <= TOL[case.dtype], f"{case.name}: relative error {err:.3e} > {TOL[case.dtype]:.1e}"
    return err


def run_batched_gpu(bc, check=True):
    import torch
    from paper_1705_05249_amd import gemm as G
    t = {name: to_gpu(getattr(bc, name)) for name in ("A", "B", "C", "a_off", "b_off", "c_off", "alphas", "betas")}
    fn = G.mg_sgemm_batched if bc.dtype == "f32" else G.mg_hgemm_batched
    st = fn(bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, t["alphas"], t["A"], t["a_off"], bc.lda, t["B"], t["b_off"],
            bc.ldb, t["betas"], t["C"], t["c_off"], bc.ldc, bc.batch, check=check)
    torch.cuda.synchronize()
    return st, t["C"].cpu().numpy()


def batched_outputs(bc, out):
    """(batch, m, n) array of the C matrices inside the flat buffer, plus mask of bytes outside them"""
    mask = np.ones(out.size, dtype=bool)
    major, minor = (bc.n, bc.m) if bc.layout == W.COL_MAJOR else (bc.m, bc.n)
    idx = (np.arange(major, dtype=np.int64)[:, None] * bc.ldc + np.arange(minor, dtype=np.int64)[None, :])
    full = bc.c_off[:, None, None] + idx[None, :, :]                    # (batch, major, minor)
    mask[full.reshape(-1)] = False
    mats = out[full]
    if bc.layout == W.COL_MAJOR:
        mats = mats.transpose(0, 2, 1)
    return mats, mask


def check_batched(bc, oracle, exact=False):
    st, out = run_batched_gpu(bc)
    assert st == 0
    mats, mask = batched_outputs(bc, out)
    assert np.array_equal(bits(out)[mask], bits(bc.C)[mask]), f"{bc.name}: gap / padding bytes were written"
    c_ref, d_ref = oracle.gemm_batched(bc.dtype, bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, bc.alphas, bc.A, bc.a_off,
                                       bc.lda, bc.B, bc.b_off, bc.ldb, bc.betas, bc.C, bc.c_off, bc.ldc)
    if exact:
        assert np.array_equal(mats.astype(np.float64), c_ref), f"{bc.name}: not bit-exact on integer inputs"
        return 0.0
    err = rel_error(mats, c_ref, d_ref)
    assert err <= TOL[bc.dtype], f"{bc.name}: relative error {err:.3e}"
    return err


# ------------------------------------------------------------------ convolution (IM2COL + GEMM)

def conv_geometry(case):
    return (case.channels, case.height, case.width, case.kernel, case.pad, case.stride, case.dilation)


def run_conv(case, workspace="auto"):
    """Runs one ConvCase through mg_sconv2d / mg_hconv2d; returns out (filters, OH, OW) as numpy."""
    import torch
    from paper_1705_05249_amd import gemm as G
    fn = G.mg_sconv2d if case.dtype == "f32" else G.mg_hconv2d
    code = G.MG_F32 if case.dtype == "f32" else G.MG_F16
    im, w, out = to_gpu(case.im), to_gpu(case.weights), to_gpu(case.out)
    if isinstance(workspace, str):
        need = G.mg_conv2d_workspace_bytes(code, *conv_geometry(case), case.filters)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda") if need else None
    fn(*conv_geometry(case), case.filters, case.alpha, im, w, case.beta, out, workspace)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def check_conv(case, conv_oracle, workspace="auto"):
    """GPU convolution against the direct-loop oracle; returns the relative error (0 for exact cases)."""
    from paper_1705_05249_amd import gemm as G
    ref, den = conv_oracle.conv2d(case.dtype, *conv_geometry(case), case.filters, case.alpha, case.im, case.weights,
                                  case.beta, case.out)
    assert ref.shape[1:] == case.out_hw
    assert tuple(G.mg_conv2d_out_extent(s, k, p, st, d) for s, k, p, st, d in
                 zip((case.height, case.width), case.kernel, case.pad, case.stride, case.dilation)) == case.out_hw
    got = run_conv(case, workspace)
    if case.exact:
        assert np.array_equal(got.astype(np.float64), ref), f"{case.name}: not bit-exact on integer inputs"
        return 0.0
    err = rel_error(got, ref, den)
    assert err <= TOL[case.dtype], f"{case.name}: relative error {err:.3e}"
    return err


def run_gemv(case, check=True, workspace="auto"):
    """Runs one GemvCase through the C ABI; returns (status, flat y buffer after the call)."""
    import torch
    from paper_1705_05249_amd import gemm as G
    fn = G.mg_sgemv if case.dtype == "f32" else G.mg_hgemv
    if isinstance(workspace, str):
        need = G.mg_gemv_workspace_bytes(G.MG_F32 if case.dtype == "f32" else G.MG_F16, case.layout, case.trans,
                                         case.m, case.n, case.lda)
        workspace = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
    A = to_gpu(case.A if case.A.size else np.zeros(1, dtype=case.A.dtype))
    x, y = to_gpu(case.x), to_gpu(case.y)
    st = fn(case.layout, case.trans, case.m, case.n, case.alpha, A, case.lda, x, case.incx, case.beta, y,
            case.incy, workspace, None, check=check)
    torch.cuda.synchronize()
    return st, y.cpu().numpy()


def check_gemv(case, oracle, workspace="auto"):
    """Element-by-element comparison of a GEMV call with the oracle; the slots between the elements of y
    must keep their bytes.  Returns the error."""
    y_ref, d_ref = oracle.gemv(case.dtype, case.layout, case.trans, case.m, case.n, case.alpha, case.A, case.lda,
                               case.x, case.incx, case.beta, case.y, case.incy)
    _, out = run_gemv(case, workspace=workspace)
    rows = case.outputs
    got = out[: (rows - 1) * case.incy + 1: case.incy] if rows else out[:0]
    mask = np.ones(out.size, dtype=bool)
    if rows:
        mask[: (rows - 1) * case.incy + 1: case.incy] = False
    assert np.array_equal(bits(out)[mask], bits(case.y)[mask]), f"{case.name}: bytes outside y were written"
    if case.exact:
        assert np.array_equal(got.astype(np.float64), y_ref), f"{case.name}: integer-valued case must be exact"
        return 0.0
    err = rel_error(got, y_ref, d_ref)
    assert err <= TOL[case.dtype], f"{case.name}: relative error {err:.3e}"
    return err


def level3_workspace(case):
    import torch
    from paper_1705_05249_amd import gemm as G
    code = G.MG_F32 if case.dtype == "f32" else G.MG_F16
    if case.routine == "symm":
        need = G.mg_symm_workspace_bytes(code, case.layout, case.side, case.m, case.n)
    elif case.routine == "syrk":
        need = G.mg_syrk_workspace_bytes(code, case.layout, case.trans, case.n, case.k)
    else:
        need = G.mg_trmm_workspace_bytes(code, case.layout, case.side, case.trans, case.m, case.n)
    return torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")


def run_level3(case, workspace="auto", check=True):
    """Runs one Level3Case through the C ABI; returns (status, flat output buffer after the call)."""
    import torch
    from paper_1705_05249_amd import gemm as G
    half = case.dtype == "f16"
    ws = level3_workspace(case) if isinstance(workspace, str) else workspace
    A = to_gpu(case.A if case.A.size else np.zeros(1, dtype=case.A.dtype))
    if case.routine == "symm":
        B, out = to_gpu(case.B), to_gpu(case.C)
        st = (G.mg_hsymm if half else G.mg_ssymm)(case.layout, case.side, case.uplo, case.m, case.n, case.alpha, A, case.lda,
                                                  B, case.ldb, case.beta, out, case.ldc, ws, None, check=check)
    elif case.routine == "syrk":
        out = to_gpu(case.C)
        st = (G.mg_hsyrk if half else G.mg_ssyrk)(case.layout, case.uplo, case.trans, case.n, case.k, case.alpha, A, case.lda,
                                                  case.beta, out, case.ldc, ws, None, check=check)
    else:
        out = to_gpu(case.B)
        st = (G.mg_htrmm if half else G.mg_strmm)(case.layout, case.side, case.uplo, case.trans, case.diag, case.m, case.n,
                                                  case.alpha, A, case.lda, out, case.ldb, ws, None, check=check)
    torch.cuda.synchronize()
    return st, out.cpu().numpy()


def check_level3(case, level3_oracle, workspace="auto"):
    """Element-by-element comparison with the oracle; bytes outside the result (padding, SYRK's other
    triangle) must be untouched.  Returns the error."""
    L3 = level3_oracle
    if case.routine == "symm":
        ref, den = L3.symm(case.dtype, case.layout, case.side, case.uplo, case.m, case.n, case.alpha, case.A, case.lda,
                           case.B, case.ldb, case.beta, case.C, case.ldc)
        before, ld = case.C, case.ldc
    elif case.routine == "syrk":
        ref, den = L3.syrk(case.dtype, case.layout, case.uplo, case.trans, case.n, case.k, case.alpha, case.A, case.lda,
                           case.beta, case.C, case.ldc)
        before, ld = case.C, case.ldc
    else:
        ref, den = L3.trmm(case.dtype, case.layout, case.side, case.uplo, case.trans, case.diag, case.m, case.n, case.alpha,
                           case.A, case.lda, case.B, case.ldb)
        before, ld = case.B, case.ldb
    st, out = run_level3(case, workspace=workspace)
    assert st == 0
    pad = W.padding_mask(case.layout, case.m, case.n, ld, before.size)
    assert np.array_equal(bits(out)[pad], bits(before)[pad]), f"{case.name}: bytes outside the matrix were written"
    got = W.unpack(out, case.layout, case.m, case.n, ld)
    live = np.ones((case.m, case.n), dtype=bool)
    if case.routine == "syrk":
        i, j = np.indices((case.n, case.n))
        live = (i <= j) if case.uplo == W.UPPER else (i >= j)
        old = W.unpack(before, case.layout, case.n, case.n, ld)
        assert np.array_equal(bits(np.ascontiguousarray(got[~live])), bits(np.ascontiguousarray(old[~live]))), \
            f"{case.name}: the other triangle of C changed"
    got, ref, den = got[live], ref[live], den[live]
    if case.exact:
        assert np.array_equal(got.astype(np.float64), ref), f"{case.name}: not bit-exact on integer inputs"
        return 0.0
    err = rel_error(got, ref, den)
    assert err <= TOL[case.dtype], f"{case.name}: relative error {err:.3e} > {TOL[case.dtype]:.1e}"
    return err
