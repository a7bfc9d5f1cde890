"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bar: bit-exact on integer-valued inputs; max |C - C_ref| / (|alpha| |A||B| + |beta| |C|) <= 1e-5 (FP32)
and <= 2e-3 (FP16 storage, FP32 accumulation) on random inputs.  Bytes outside the C matrix (leading
dimension padding, gaps between batched instances) must come back unchanged.
"""
import ctypes
import sys

import numpy as np
import pytest

from paper_1705_05249_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu

R, C, N, T = W.ROW_MAJOR, W.COL_MAJOR, W.NO_TRANS, W.TRANS
VARIANTS = [(lay, ta, tb) for lay in (R, C) for ta in (N, T) for tb in (N, T)]


def announce(*what):
    print("[case]", *what, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_1705_05249_amd import gemm
    gemm.lib()
    gemm.mg_clear_override()
    yield gemm
    gemm.mg_clear_override()


# ------------------------------------------------------------------ group 1: 256^3

@pytest.mark.parametrize("integer", [True, False])
def test_config1(G, oracle, integer):
    case = W.config1(integer)
    announce(case.name)
    H.check_case(case, oracle)


# ------------------------------------------------------------------ group 2: squares, 8 storage variants

@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
@pytest.mark.parametrize("size,beta,integer", [(192, 0.7, False), (200, 0.0, False), (321, 0.5, True), (512, 0.0, True)])
def test_config2_oracle_sized(G, oracle, layout, ta, tb, size, beta, integer):
    case = W.config2_like(size, layout, ta, tb, beta, seed_case=size, integer=integer)
    announce(case.name, layout, ta, tb, beta, "int" if integer else "rand")
    H.check_case(case, oracle)


@pytest.mark.parametrize("beta", W.CONFIG2_BETAS)
@pytest.mark.parametrize("size", W.CONFIG2_SIZES)
def test_config2_full_sizes_sampled(G, oracle, size, beta):
    """all 8 storage variants of one size and beta must match the same logical result
    (the oracle is evaluated on complete sampled rows/columns and scattered entries)"""
    logical = W.config2_logical(size)
    # six complete rows and columns at 8192 (sixteen below): the eight variants of the largest size take about
    # 50 s, most of it building, moving and unpacking the 256 MB host arrays
    sample = {"rows": 6, "cols": 6, "scattered": 2048} if size >= 8192 else None
    for layout, ta, tb in VARIANTS:
        case = W.config2_variant(size, layout, ta, tb, beta, logical)
        announce(case.name)
        H.check_case(case, oracle, sampled=True, seed=size, sample=sample)


# ------------------------------------------------------------------ group 3: FP16 storage

@pytest.mark.parametrize("index", range(len(W.CONFIG3_SHAPES)))
@pytest.mark.parametrize("integer", [False, True])
def test_config3(G, oracle, index, integer):
    m, n, k = W.CONFIG3_SHAPES[index]
    if integer and k > 512:
        # keep |sum| <= 2048 so the FP16 result is exact: shrink k only
        case = W.hgemm_case(m, n, 512, case=100 + index, integer=True, name=f"c3int_{m}x{n}x512")
    else:
        case = W.config3(index, integer)
    announce(case.name)
    H.check_case(case, oracle, sampled=(m * n * case.k > 2 ** 31))


@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
@pytest.mark.parametrize("shape,alpha,beta", [((130, 72, 200), 1.0, 0.0), ((64, 257, 96), 0.5, 2.0), ((256, 256, 64), 1.0, 1.0)])
def test_hgemm_variants(G, oracle, layout, ta, tb, shape, alpha, beta):
    m, n, k = shape
    case = W.hgemm_case(m, n, k, case=m + n + k, layout=layout, ta=ta, tb=tb, alpha=alpha, beta=beta)
    announce(case.name, layout, ta, tb)
    H.check_case(case, oracle)


def test_hgemm_subnormal_inputs_are_not_flushed(G, oracle):
    m = n = 64
    k = 32
    A = np.full((m, k), 2.0 ** -24, dtype=np.float16)
    B = np.full((k, n), 1024.0, dtype=np.float16)
    case = W.make_case("subnormal", "f16", C, N, N, A, B, np.zeros((m, n), np.float16), 1.0, 0.0)
    _, out = H.run_gpu(case)
    assert np.all(out.astype(np.float64) == k * 2.0 ** -14)


def test_split_k_runs_only_with_workspace(G, oracle):
    """a shape for which split-K is selected: with the workspace the query asks for it runs split, without
    any workspace it silently runs unsplit; both give parity"""
    case = W.hgemm_case(512, 196, 4608, case=3)     # too long a sum for the kernel whose wavefronts share it
    code = G.MG_F16
    sel = G.mg_query_selected(code, case.layout, case.ta, case.tb, case.m, case.n, case.k, case.lda, case.ldb, case.ldc)
    assert sel["split_k"] > 1
    H.check_case(case, oracle)                      # workspace sized by mg_gemm_workspace_bytes
    H.check_case(case, oracle, workspace=None)      # no workspace: unsplit fallback
    import torch
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    H.check_case(case, oracle, workspace=small)     # too small a workspace: unsplit fallback as well


# ------------------------------------------------------------------ group 4: batched

@pytest.mark.parametrize("size", W.CONFIG4_SIZES)
@pytest.mark.parametrize("batch", W.CONFIG4_BATCHES)
def test_config4(G, oracle, size, batch):
    bc = W.config4_fast(size, batch) if batch > 1000 else W.config4(size, batch)
    announce(bc.name)
    H.check_batched(bc, oracle)


@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
def test_batched_variants_ragged_exact(G, oracle, layout, ta, tb):
    for (m, n, k, batch, pad) in ((5, 7, 6, 9, 0), (16, 16, 16, 33, 0), (33, 17, 70, 5, 3), (64, 64, 64, 3, 1),
                                  (70, 130, 9, 2, 0), (1, 1, 1, 4, 0)):
        bc = W.batched_case(m, n, k, batch, case=m * n + k, layout=layout, ta=ta, tb=tb, integer=True,
                            shuffle_offsets=True,
                            lda=W.tight_ld(layout, ta, m, k) + pad, ldb=W.tight_ld(layout, tb, k, n) + 2 * pad,
                            ldc=W.tight_ld(layout, N, m, n) + pad)
        announce(bc.name, layout, ta, tb)
        H.check_batched(bc, oracle, exact=True)


def test_batched_equals_loop_of_singles(G, oracle):
    """the batched routine and a loop of non-batched calls agree (both within tolerance of the oracle,
    and with each other to a few ulps of the denominator)"""
    import torch
    bc = W.batched_case(16, 16, 16, 20, case=5)
    _, out = H.run_batched_gpu(bc)
    mats, _ = H.batched_outputs(bc, out)
    A, B, Cd = H.to_gpu(bc.A), H.to_gpu(bc.B), H.to_gpu(bc.C)
    for i in range(bc.batch):
        G.mg_sgemm(bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, float(bc.alphas[i]), A[int(bc.a_off[i]):], bc.lda,
                   B[int(bc.b_off[i]):], bc.ldb, float(bc.betas[i]), Cd[int(bc.c_off[i]):], bc.ldc)
    torch.cuda.synchronize()
    singles, _ = H.batched_outputs(bc, Cd.cpu().numpy())
    _, d_ref = oracle.sgemm_batched(bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, bc.alphas, bc.A, bc.a_off, bc.lda,
                                    bc.B, bc.b_off, bc.ldb, bc.betas, bc.C, bc.c_off, bc.ldc)
    assert np.max(np.abs(mats.astype(np.float64) - singles.astype(np.float64)) / d_ref) <= 2e-6


def test_batched_alpha_zero_and_beta_zero_per_instance(G, oracle):
    bc = W.batched_case(16, 16, 16, 6, case=9)
    bc.alphas[1] = 0.0
    bc.betas[2] = 0.0
    la = 256
    bc.A[bc.a_off[1]: bc.a_off[1] + la] = np.nan         # must not be used: alpha == 0
    bc.C[bc.c_off[2]: bc.c_off[2] + la] = np.nan         # must not be read: beta == 0
    st, out = H.run_batched_gpu(bc)
    mats, _ = H.batched_outputs(bc, out)
    c_ref, d_ref = oracle.sgemm_batched(bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, bc.alphas, bc.A, bc.a_off,
                                        bc.lda, bc.B, bc.b_off, bc.ldb, bc.betas, bc.C, bc.c_off, bc.ldc)
    assert H.rel_error(mats, c_ref, d_ref) <= H.TOL["f32"]


def test_batched_whole_column_kernel_conventions(G, oracle):
    """the 64^3 FP32 kernel whose lanes are rows of C (A along m, B along k; B goes through LDS): padded leading
    dimensions (columns no longer adjacent in memory), shuffled offsets, alpha == 0 and beta == 0 per instance with NaN
    where nothing may be read, an odd batch count (a work-group with idle wavefronts); bit-exact on integers; padding
    between columns and the gaps between instances untouched; the row-major N/N call is the same canonical problem"""
    try:
        G.mg_override_batched_config(G.kernel_id("batched_rows_64_mk_full"))      # (a shape it does not take would be an error)
        for layout, lda, ldb, ldc in ((C, 70, 67, 65), (C, None, None, None), (R, 66, 71, 64)):
            bc = W.batched_case(64, 64, 64, 7, case=64, layout=layout, ta=N, tb=N, integer=True, lda=lda, ldb=ldb, ldc=ldc,
                                shuffle_offsets=True)
            bc.alphas[1] = 0.0
            bc.betas[2] = 0.0
            bc.alphas[5] = 0.0
            bc.betas[5] = 0.0
            la = W.storage_len(layout, N, 64, 64, bc.lda)
            lc = W.storage_len(layout, N, 64, 64, bc.ldc)
            for i in (1, 5):
                bc.A[bc.a_off[i]: bc.a_off[i] + la] = np.nan         # must not be used: alpha == 0
            for i in (2, 5):
                live = ~W.padding_mask(layout, 64, 64, bc.ldc, lc)
                view = bc.C[bc.c_off[i]: bc.c_off[i] + lc]
                view[live] = np.nan                                  # must not be read: beta == 0
            announce("rows64", bc.name, layout, bc.lda, bc.ldb, bc.ldc)
            H.check_batched(bc, oracle, exact=True)
    finally:
        G.mg_clear_override()


# ------------------------------------------------------------------ FP16-storage batched GEMM

@pytest.mark.parametrize("size", W.CONFIG4_SIZES)
def test_half_batched_workload_sizes(G, oracle, size):
    """the batched workload's shapes (s = 8, 16, 32, 64; 1000 instances, 7-element gaps) in FP16 storage"""
    bc = W.batched_case(size, size, size, 1000, case=size, dtype="f16")
    announce(bc.name)
    H.check_batched(bc, oracle)


@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
def test_half_batched_variants_ragged_exact(G, oracle, layout, ta, tb):
    for (m, n, k, batch, pad) in ((5, 7, 6, 9, 0), (16, 16, 16, 33, 0), (33, 17, 70, 5, 3), (64, 64, 64, 3, 1),
                                  (70, 130, 9, 2, 0), (1, 1, 1, 4, 0)):
        bc = W.batched_case(m, n, k, batch, case=m * n + k, layout=layout, ta=ta, tb=tb, integer=True,
                            shuffle_offsets=True, dtype="f16",
                            lda=W.tight_ld(layout, ta, m, k) + pad, ldb=W.tight_ld(layout, tb, k, n) + 2 * pad,
                            ldc=W.tight_ld(layout, N, m, n) + pad)
        announce(bc.name, layout, ta, tb)
        H.check_batched(bc, oracle, exact=True)


@pytest.mark.parametrize("layout,ta,tb", [(C, N, N), (R, T, N), (C, T, T)])
@pytest.mark.parametrize("shape", [(16, 16, 16, 300), (33, 20, 70, 9), (64, 64, 64, 5)])
def test_half_strided_batched(G, oracle, layout, ta, tb, shape):
    import torch
    m, n, k, batch = shape
    bc = W.batched_case(m, n, k, batch, case=m + n + k, layout=layout, ta=ta, tb=tb, integer=True, dtype="f16")
    sa, sb, sc = (int(x[1] - x[0]) for x in (bc.a_off, bc.b_off, bc.c_off))
    alpha, beta = 1.5, 0.5
    A, B, Cs = H.to_gpu(bc.A), H.to_gpu(bc.B), H.to_gpu(bc.C)
    announce("strided f16", bc.name, layout, ta, tb)
    G.mg_hgemm_strided_batched(layout, ta, tb, m, n, k, alpha, A, bc.lda, sa, B, bc.ldb, sb, beta, Cs, bc.ldc, sc, batch)
    torch.cuda.synchronize()
    out = Cs.cpu().numpy()
    mats, mask = H.batched_outputs(bc, out)
    assert np.array_equal(H.bits(out)[mask], H.bits(bc.C)[mask])
    c_ref, _ = oracle.gemm_strided_batched("f16", layout, ta, tb, m, n, k, alpha, bc.A, bc.lda, sa, bc.B, bc.ldb, sb,
                                           beta, bc.C, bc.ldc, sc, batch)
    assert np.array_equal(mats.astype(np.float64), c_ref)


def test_half_batched_per_instance_conventions(G, oracle):
    """alpha_i == 0 skips A and B (NaN there), beta_i == 0 skips C (NaN there), per instance"""
    bc = W.batched_case(16, 16, 16, 6, case=77, integer=True, dtype="f16")
    bc.alphas[1] = 0.0
    bc.A[bc.a_off[1]: bc.a_off[1] + 256] = np.nan
    bc.betas[2] = 0.0
    bc.C[bc.c_off[2]: bc.c_off[2] + 256] = np.nan
    H.check_batched(bc, oracle, exact=True)


# ------------------------------------------------------------------ strided batched (same data as the generic form)

@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
@pytest.mark.parametrize("shape", [(16, 16, 16, 300), (8, 8, 8, 77), (33, 20, 70, 9), (64, 64, 64, 5), (70, 130, 9, 3)])
def test_strided_batched(G, oracle, layout, ta, tb, shape):
    """strided == generic with offsets b*stride and constant scalars: against the oracle (bit-exact on
    integers), against the generic routine on the same buffers (bitwise), gaps untouched"""
    import torch
    m, n, k, batch = shape
    bc = W.batched_case(m, n, k, batch, case=m + n + k, layout=layout, ta=ta, tb=tb, integer=True)
    sa, sb, sc = (int(x[1] - x[0]) for x in (bc.a_off, bc.b_off, bc.c_off))
    alpha, beta = 1.5, 0.5
    A, B, Cs = H.to_gpu(bc.A), H.to_gpu(bc.B), H.to_gpu(bc.C)
    announce("strided", bc.name, layout, ta, tb)
    G.mg_sgemm_strided_batched(layout, ta, tb, m, n, k, alpha, A, bc.lda, sa, B, bc.ldb, sb, beta, Cs, bc.ldc, sc, batch)
    torch.cuda.synchronize()
    out = Cs.cpu().numpy()
    mats, mask = H.batched_outputs(bc, out)
    assert np.array_equal(H.bits(out)[mask], H.bits(bc.C)[mask])
    c_ref, _ = oracle.sgemm_strided_batched(layout, ta, tb, m, n, k, alpha, bc.A, bc.lda, sa, bc.B, bc.ldb, sb, beta,
                                            bc.C, bc.ldc, sc, batch)
    assert np.array_equal(mats.astype(np.float64), c_ref)
    # the generic routine on the same data
    bc.alphas[:] = alpha
    bc.betas[:] = beta
    _, out_generic = H.run_batched_gpu(bc)
    assert np.array_equal(H.bits(out), H.bits(out_generic))


def test_strided_batched_scalars_and_random(G, oracle):
    import torch
    bc = W.batched_case(16, 16, 16, 50, case=31)
    stride = int(bc.a_off[1] - bc.a_off[0])
    for alpha, beta in ((0.0, 2.0), (1.25, 0.0), (0.7, 1.3)):
        A, B, Cs = H.to_gpu(bc.A), H.to_gpu(bc.B), H.to_gpu(bc.C)
        if alpha == 0.0:
            A = torch.full_like(A, float("nan"))           # must not be read
        if beta == 0.0:
            Cs = torch.where(Cs == float(W.GAP_FILL), Cs, torch.full_like(Cs, float("nan")))   # C_old must not be read
        G.mg_sgemm_strided_batched(bc.layout, bc.ta, bc.tb, 16, 16, 16, alpha, A, 16, stride, B, 16, stride, beta, Cs,
                                   16, stride, bc.batch)
        torch.cuda.synchronize()
        mats, _ = H.batched_outputs(bc, Cs.cpu().numpy())
        c_ref, d_ref = oracle.sgemm_strided_batched(bc.layout, bc.ta, bc.tb, 16, 16, 16, alpha, bc.A, 16, stride, bc.B,
                                                    16, stride, beta, bc.C, 16, stride, bc.batch)
        assert H.rel_error(mats, c_ref, d_ref) <= H.TOL["f32"]


# ------------------------------------------------------------------ group 5: odd and skinny

@pytest.mark.parametrize("index", range(len(W.CONFIG5_SHAPES)))
@pytest.mark.parametrize("integer", [False, True])
def test_config5(G, oracle, index, integer):
    case = W.config5(index, integer)
    announce(case.name, "int" if integer else "rand")
    H.check_case(case, oracle, sampled=(case.m * case.n * case.k > 3 * 2 ** 30), seed=index)


@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
@pytest.mark.parametrize("shape", [(1, 1, 1), (1, 300, 257), (300, 1, 257), (129, 130, 131), (279, 32, 100),
                                   (32, 32, 32), (65, 63, 17), (2, 3, 1000)])
def test_small_and_skinny_shapes_exact(G, oracle, layout, ta, tb, shape):
    m, n, k = shape
    case = W.skinny_case(m, n, k, case=m * 7 + n * 3 + k, integer=True, layout=layout, ta=ta, tb=tb,
                         alpha=2.0, beta=-1.0)
    announce(case.name, layout, ta, tb)
    H.check_case(case, oracle)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_unaligned_base_pointers(G, oracle, dtype):
    """operands that start 1..3 elements into an allocation (no 16-byte alignment anywhere)"""
    for (m, n, k), offs in (((256, 256, 128), (1, 2, 3)), ((130, 70, 90), (3, 1, 1)), ((512, 256, 256), (0, 4, 0))):
        for layout, ta, tb in ((C, N, N), (C, T, N), (R, N, T)):
            if dtype == "f32":
                case = W.make_case(
                    f"unal_{m}x{n}x{k}", "f32", layout, ta, tb,
                    W.small_ints(W.rng_for(6, m), (m, k)), W.small_ints(W.rng_for(6, n), (k, n)),
                    W.small_ints(W.rng_for(6, k), (m, n)), 1.0, 1.0, exact=True)
            else:
                case = W.hgemm_case(m, n, k, case=m, layout=layout, ta=ta, tb=tb, beta=1.0)
            announce(case.name, dtype, layout, ta, tb, offs)
            H.check_case(case, oracle, offset_elems=offs)


# ------------------------------------------------------------------ special scalars and empty problems

@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_alpha_zero_ignores_nan_in_a_b(G, oracle, dtype):
    m, n, k = 70, 50, 40
    t = np.float32 if dtype == "f32" else np.float16
    Cm = W.small_ints(W.rng_for(7, 1), (m, n), dtype=t)
    case = W.make_case("alpha0", dtype, C, N, T, np.full((m, k), np.nan, t), np.full((k, n), np.inf, t), Cm,
                       0.0, 0.5, exact=True)
    H.check_case(case, oracle)
    case = W.make_case("alpha0beta0", dtype, R, T, N, np.full((m, k), np.nan, t), np.full((k, n), np.nan, t),
                       np.full((m, n), np.nan, t), 0.0, 0.0, exact=True)
    H.check_case(case, oracle)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_beta_zero_ignores_nan_in_c(G, oracle, dtype):
    for m, n, k in ((70, 50, 40), (256, 256, 256), (1, 200, 300)):
        t = np.float32 if dtype == "f32" else np.float16
        g = W.rng_for(7, 2)
        case = W.make_case("beta0", dtype, C, N, N, W.small_ints(g, (m, k), 2, t), W.small_ints(g, (k, n), 2, t),
                           np.full((m, n), np.nan, t), 1.0, 0.0, exact=True)
        announce(case.name, dtype, m, n, k)
        H.check_case(case, oracle)


def test_k_zero_and_empty(G, oracle):
    Cm = W.small_ints(W.rng_for(7, 3), (33, 20))
    case = W.make_case("k0", "f32", C, N, N, np.zeros((33, 0), np.float32), np.zeros((0, 20), np.float32), Cm,
                       3.0, 2.0, exact=True)
    H.check_case(case, oracle)
    import torch
    buf = torch.zeros(64, device="cuda")
    assert G.mg_sgemm(C, N, N, 0, 5, 5, 1.0, buf, 1, buf, 5, 0.0, buf, 1) == 0
    assert G.mg_sgemm(C, N, N, 5, 0, 5, 1.0, buf, 5, buf, 5, 0.0, buf, 5) == 0
    assert torch.all(buf == 0)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
def test_one_or_two_beyond_a_tile_multiple(G, oracle, dtype, layout, ta, tb):
    """shapes one or two rows / columns beyond a multiple of 64 (the 129 = 128 + 1 pattern of the irregular
    workload group): nearly empty last tiles; exact on integers, padding untouched"""
    for (m, n, k) in ((129, 320, 256), (320, 130, 300), (257, 258, 260), (65, 600, 512)):
        if dtype == "f32":
            g = W.rng_for(9, m + n)
            case = W.make_case(f"strip_{m}x{n}x{k}", "f32", layout, ta, tb, W.small_ints(g, (m, k)), W.small_ints(g, (k, n)),
                               W.small_ints(g, (m, n)), 1.5, 0.5, lda=W.tight_ld(layout, ta, m, k) + 3,
                               ldb=W.tight_ld(layout, tb, k, n) + 1, ldc=W.tight_ld(layout, N, m, n) + 2, exact=True)
        else:
            case = W.hgemm_case(m, n, k, case=m + n, layout=layout, ta=ta, tb=tb, alpha=1.0, beta=1.0, integer=True)
        announce(case.name, layout, ta, tb)
        H.check_case(case, oracle)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("ta,tb", [(N, N), (T, N), (N, T), (T, T)])
def test_bounds_checked_k_loop_ends(G, oracle, dtype, ta, tb):
    """the bounds-checked tile kernels choose per K-tile how the staging registers are reloaded (the fast flavour's
    loads, checked loads for the partial last K-tile, none for the last two tiles): sums of zero to six whole K-tiles
    with and without a partial one, on the smallest bounds-checked tile (forced), rows on dword boundaries and (FP16)
    at odd elements, ragged m and n, also cut into two slices; exact on integers"""
    import torch
    bk = 32 if dtype == "f32" else 64
    tag = ("smfma_64x64x32_w2x2" if dtype == "f32" else "hmfma_64x64x64_w2x2")
    contig = {(N, N): "mk", (T, N): "kk", (N, T): "mn", (T, T): "kn"}[(ta, tb)]
    ws = torch.empty(8 << 20, dtype=torch.uint8, device="cuda")
    m, n = 150, 70
    try:
        for whole in range(0, 7):
            for rest in (0, 7, bk - 1):
                k = whole * bk + rest
                if k == 0:
                    continue
                for odd in ((0,) if dtype == "f32" else (0, 1)):
                    for split in ((1, 2) if whole >= 4 else (1,)):
                        # an even k keeps FP16 rows along k on dwords; `odd` moves them off
                        kk = k + (k % 2 if dtype == "f16" else 0)
                        lds = dict(lda=W.tight_ld(C, ta, m, kk) + 2 + odd, ldb=W.tight_ld(C, tb, kk, n) + 2 + odd,
                                   ldc=W.tight_ld(C, N, m, n) + 1)
                        if dtype == "f32":
                            g = W.rng_for(11, 100 * whole + rest)
                            case = W.make_case(f"kends_{m}x{n}x{kk}", "f32", C, ta, tb, W.small_ints(g, (m, kk)),
                                               W.small_ints(g, (kk, n)), W.small_ints(g, (m, n)), 1.0, 1.0, exact=True, **lds)
                        else:
                            case = W.hgemm_case(m, n, kk, case=100 * whole + rest, layout=C, ta=ta, tb=tb, alpha=1.0, beta=1.0,
                                                integer=True, **lds)
                        G.mg_override_config(G.kernel_id(f"{tag}_{contig}_edge"), split)
                        announce(case.name, "split", split, "ld +", 2 + odd, ta, tb)
                        H.check_case(case, oracle, workspace=ws)
    finally:
        G.mg_clear_override()


# ------------------------------------------------------------------ fringe rows / columns beside the tiles

def _fringe_of(layout, m, n):
    """16 * rows + columns that the column-major view of an m x n problem leaves to the fringe work-groups"""
    def extra(d):
        return d % 64 if d >= 64 and 1 <= d % 64 <= 4 else 0
    vm, vn = (m, n) if layout == C else (n, m)
    return (16 * extra(vm) + extra(vn)) if vm >= 64 and vn >= 64 else 0


@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
def test_fringe_rows_and_columns(G, oracle, layout, ta, tb):
    """FP32 problems that are 1 to 4 rows and / or columns more than a multiple of 64: those rows and columns are
    computed by the work-groups appended to the tile grid (matrix-vector products, both of their forms), the tiles
    cover the rest.  Every bounds-checked FP32 tile, unsplit and with a split sum (raw partial sums from both kinds
    of work-group); fringe on one side, on both, of every width; outputs that end inside a work-group's share; sums
    that end inside a 16-byte piece; bit-exact on integers, padding untouched, and one random case per shape."""
    import torch
    code = G.MG_F32
    edge = [t for t in G.kernel_table() if t["dtype"] == code and t["family"] == G.MG_FAMILY_MFMA and t["name"].endswith("_edge")]
    shapes = ((129, 193, 70), (65, 260, 301), (258, 67, 129), (131, 132, 64), (300, 65, 1003), (68, 64, 33), (1027, 129, 518),
              (64, 577, 96))
    ran = 0
    ws = torch.empty(32 << 20, dtype=torch.uint8, device="cuda")
    try:
        G.mg_override_fringe(G.MG_FRINGE_ON)
        for (m, n, k) in shapes:
            cases = [W.skinny_case(m, n, k, case=31, integer=True, layout=layout, ta=ta, tb=tb, alpha=1.5, beta=0.5),
                     W.skinny_case(m, n, k, case=32, integer=False, layout=layout, ta=ta, tb=tb, alpha=-0.75, beta=1.25)]
            for t in edge:
                for split in (1, 3):
                    G.mg_override_config(t["kernel_id"], split)
                    cfg = G.mg_config()
                    q = G.lib().mg_query_selected(code, layout, ta, tb, m, n, k, cases[0].lda, cases[0].ldb, cases[0].ldc,
                                                  1.5, 0.5, 256, ctypes.byref(cfg))
                    if q != 0:
                        continue                     # this tile does not take this operand order, or the split is too fine
                    assert cfg.fringe == _fringe_of(layout, m, n) != 0
                    for case in cases[: 1 if t["tile_m"] * t["tile_n"] > 128 * 64 else 2]:
                        announce("fringe", t["name"], "split", split, case.name, layout, ta, tb, "exact" if case.exact else "random")
                        H.check_case(case, oracle, workspace=ws)
                        ran += 1
        # beta == 0 with NaN in C: the fringe work-groups must not read C either
        G.mg_clear_override()
        G.mg_override_fringe(G.MG_FRINGE_ON)
        case = W.skinny_case(130, 195, 80, case=33, integer=True, layout=layout, ta=ta, tb=tb, alpha=2.0, beta=0.0)
        mask = ~W.padding_mask(layout, case.m, case.n, case.ldc, case.C.size)
        case.C[mask] = np.nan
        announce("fringe beta 0", case.name, layout, ta, tb)
        H.check_case(case, oracle, workspace=ws)
    finally:
        G.mg_clear_override()
    assert ran >= 2 * len(shapes)


def test_fringe_automatic_equals_tiled(G, oracle):
    """automatic mode on a shape of the irregular workload group's kind: the selected route leaves a fringe, and
    its result agrees with the oracle and (on integers, bit for bit) with the all-tiles route"""
    case = W.skinny_case(1025, 129, 1030, case=34, integer=True)
    sel = G.mg_query_selected(G.MG_F32, case.layout, case.ta, case.tb, case.m, case.n, case.k, case.lda, case.ldb, case.ldc,
                              case.alpha, case.beta)
    assert sel["fringe"] == 17, sel
    announce("fringe auto", case.name, sel["name"], sel["split_k"])
    H.check_case(case, oracle)
    _, with_fringe = H.run_gpu(case)
    try:
        G.mg_override_fringe(G.MG_FRINGE_OFF)
        assert G.mg_query_selected(G.MG_F32, case.layout, case.ta, case.tb, case.m, case.n, case.k, case.lda, case.ldb,
                                   case.ldc, case.alpha, case.beta)["fringe"] == 0
        _, tiled = H.run_gpu(case)
    finally:
        G.mg_clear_override()
    assert np.array_equal(H.bits(with_fringe), H.bits(tiled))


@pytest.mark.parametrize("ta,tb", [(N, N), (T, T)])
def test_partial_tiles_whose_operand_ends_beyond_two_gib(G, oracle, ta, tb):
    """a partial tile of the bounds-checked FP32 flavour limits its buffer descriptor to the end of the matrix; with a
    leading dimension of 66000 and a sum of 8200 terms the operand along its rows ends 2.16 GB behind the tile's first
    element, more than a descriptor's 2^31 - 1 bytes: the limit must saturate, not wrap (rows beyond the matrix and
    the padding hold NaN)"""
    m, n, k, ld = 70, 70, 8200, 66000
    g = W.rng_for(9, 4242)
    case = W.make_case(f"wide_ld_{m}x{n}x{k}", "f32", C, ta, tb, W.small_ints(g, (m, k), 2), W.small_ints(g, (k, n), 2),
                       W.small_ints(g, (m, n)), 1.0, 1.0, lda=ld if ta == N else None, ldb=ld if tb == T else None, exact=True)
    announce(case.name, ta, tb, "bytes of the wide operand:", (case.A if ta == N else case.B).nbytes)
    H.check_case(case, oracle)


# ------------------------------------------------------------------ every compiled configuration is result-neutral

def _probe_cases(dtype):
    """small problems that together make every compiled kernel legal at least once"""
    cases = []
    for layout, ta, tb in ((C, N, N), (C, T, N), (C, N, T), (C, T, T), (R, N, N)):
        if dtype == "f32":
            for (m, n, k) in ((512, 512, 256), (260, 250, 100)):
                g = W.rng_for(8, m + k)
                cases.append(W.make_case(f"probe_f32_{m}x{n}x{k}", "f32", layout, ta, tb, W.small_ints(g, (m, k)),
                                         W.small_ints(g, (k, n)), W.small_ints(g, (m, n)), 1.5, 0.5, exact=True))
            cases.append(W.skinny_case(1, 512, 768, case=1, integer=True, layout=layout, ta=ta, tb=tb))
            cases.append(W.skinny_case(512, 1, 768, case=2, integer=True, layout=layout, ta=ta, tb=tb))
        else:
            for (m, n, k) in ((512, 512, 256), (260, 250, 100)):
                cases.append(W.hgemm_case(m, n, k, case=m + k, layout=layout, ta=ta, tb=tb, beta=1.0, integer=True))
            cases.append(W.hgemm_case(512, 512, 256, case=3, layout=layout, ta=ta, tb=tb, beta=0.5))
            cases.append(W.hgemm_case(1, 512, 768, case=4, layout=layout, ta=ta, tb=tb, beta=1.0, integer=True))
            cases.append(W.hgemm_case(512, 1, 768, case=5, layout=layout, ta=ta, tb=tb, beta=1.0, integer=True))
    return cases


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_every_kernel_configuration_gives_parity(G, oracle, dtype):
    import torch
    code = G.MG_F32 if dtype == "f32" else G.MG_F16
    # (not here: the convolution kernels, tests/test_gpu_conv.py, and the flavour for padded operands with the caller's
    # own C, which only the indirect route can call: test_indirect_route_for_ragged_half_problems)
    kernels = [t for t in G.kernel_table() if t["dtype"] == code and t["family"] not in
               (G.MG_FAMILY_BATCHED, G.MG_FAMILY_SCALE, G.MG_FAMILY_CONV) and
               not t["name"].startswith(("hpp16c_", "hdma16c_"))]
    ran = {t["name"]: 0 for t in kernels}
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    try:
        for case in _probe_cases(dtype):
            for t in kernels:
                for split in (1, 2, 3):
                    G.mg_override_config(t["kernel_id"], split)
                    # legality is asked first so that an illegal combination is skipped, not launched
                    cfg = G.mg_config()
                    q = G.lib().mg_query_selected(code, case.layout, case.ta, case.tb, case.m, case.n, case.k,
                                                  case.lda, case.ldb, case.ldc, case.alpha, case.beta, 256,
                                                  ctypes.byref(cfg))
                    if q != 0:
                        continue
                    announce(t["name"], "split", split, case.name, case.layout, case.ta, case.tb)
                    H.check_case(case, oracle, workspace=ws)
                    ran[t["name"]] += 1
    finally:
        G.mg_clear_override()
    never = [name for name, count in ran.items() if count == 0]
    assert not never, f"kernels never exercised: {never}"


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_shared_sum_kernels_over_several_chunks(G, oracle, dtype):
    """the kernels whose eight wavefronts share the sum of one 32 x 32 block: K ranges of one to seven 1 KB chunks per
    row (the loads of three chunks are in flight at once, so the fourth and later ones reuse registers), ragged in
    every direction, all operand orders; bit-exact on integers (beta = 1), within tolerance on random data"""
    per_chunk = 256 if dtype == "f32" else 512
    orders = {"mk": (N, N), "kk": (T, N), "mn": (N, T), "kn": (T, T)}
    try:
        for order, (ta, tb) in orders.items():
            G.mg_override_config(G.kernel_id(("s" if dtype == "f32" else "h") + "tiny_32x32_" + order), 1)
            for m, n, k in ((64, 96, per_chunk), (45, 70, 3 * per_chunk - 5), (96, 33, 4 * per_chunk + 8), (33, 64, 7 * per_chunk - 1)):
                for integer in (True, False):
                    if dtype == "f32":
                        case = W.skinny_case(m, n, k, case=21, integer=integer, ta=ta, tb=tb, alpha=1.0 if integer else 0.5,
                                             beta=1.0 if integer else -0.75)
                    else:
                        case = W.hgemm_case(m, n, k, case=21, ta=ta, tb=tb, beta=1.0 if integer else 0.5, integer=integer)
                    announce("tiny", dtype, order, case.name, "integer" if integer else "random")
                    H.check_case(case, oracle)
    finally:
        G.mg_clear_override()


@pytest.mark.parametrize("shape", [(256, 256, 64), (256, 512, 128), (768, 256, 448), (512, 512, 1024)])
def test_direct_to_lds_kernels(G, oracle, shape):
    """every direct-to-LDS kernel, all operand orders: one K-tile, an odd number of K-tiles, several tiles of C;
    bit-exact on integers (beta = 1) and within tolerance on random data"""
    m, n, k = shape
    names = [t["name"] for t in G.kernel_table() if t["name"].startswith(("hdma", "hpp")) and
             not t["name"].startswith(("hpp16c_", "hdma16c_"))]              # (those: the indirect route's own)
    assert names
    orders = {"mk": (N, N), "kk": (T, N), "mn": (N, T), "kn": (T, T)}
    try:
        for name in names:
            ta, tb = orders[name.rsplit("_", 1)[1]]
            for integer in (True, False):
                case = W.hgemm_case(m, n, k, case=7, ta=ta, tb=tb, beta=1.0 if integer else 0.0, integer=integer)
                G.mg_override_config(G.kernel_id(name), 1)
                announce(name, case.name, "integer" if integer else "random")
                H.check_case(case, oracle)
    finally:
        G.mg_clear_override()


def test_every_batched_configuration_gives_parity(G, oracle):
    kernels = [t for t in G.kernel_table() if t["family"] == G.MG_FAMILY_BATCHED]
    ran = {t["name"]: 0 for t in kernels}
    try:
        for (s, batch) in ((8, 51), (16, 70), (16, 33), (32, 20), (64, 9), (24, 5)):
            for layout, ta, tb, dtype in [(*v, d) for v in ((C, N, N), (R, N, N), (C, T, T), (C, T, N), (C, N, T))
                                          for d in ("f32", "f16")]:
                bc = W.batched_case(s, s, s, batch, case=s, layout=layout, ta=ta, tb=tb, integer=True, dtype=dtype)
                for t in kernels:
                    if t["dtype"] != (G.MG_F32 if dtype == "f32" else G.MG_F16):
                        continue
                    G.mg_override_batched_config(t["kernel_id"])
                    announce(t["name"], bc.name, layout, ta, tb)
                    try:
                        H.check_batched(bc, oracle, exact=True)
                        ran[t["name"]] += 1
                    except G.MgError as e:
                        assert e.status == -11          # this kernel does not take this shape
    finally:
        G.mg_clear_override()
    never = [name for name, count in ran.items() if count == 0]
    assert not never, f"batched kernels never exercised: {never}"


# ------------------------------------------------------------------ HIP graph capture of the library's launches

def test_calls_can_be_captured_in_a_hip_graph(G, oracle):
    """the library only enqueues kernels (no memset, no allocation), so its calls can be captured; every
    replay, with eager work and synchronisations in between, reproduces the eager result"""
    import torch
    case = W.hgemm_case(512, 384, 256, case=21, beta=0.5)
    bc = W.batched_case(16, 16, 16, 40, case=22)
    A, B, C0 = H.to_gpu(case.A), H.to_gpu(case.B), H.to_gpu(case.C)
    t = {name: H.to_gpu(getattr(bc, name)) for name in ("A", "B", "C", "a_off", "b_off", "c_off", "alphas", "betas")}
    Cb0 = t["C"].clone()
    C = C0.clone()

    def calls():
        G.mg_hgemm(case.layout, case.ta, case.tb, case.m, case.n, case.k, case.alpha, A, case.lda, B, case.ldb,
                   case.beta, C, case.ldc)
        G.mg_sgemm_batched(bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, t["alphas"], t["A"], t["a_off"], bc.lda,
                           t["B"], t["b_off"], bc.ldb, t["betas"], t["C"], t["c_off"], bc.ldc, bc.batch)

    calls()
    torch.cuda.synchronize()
    eager_c, eager_b = C.clone(), t["C"].clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        C.copy_(C0); t["C"].copy_(Cb0)
        calls()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    C.copy_(C0); t["C"].copy_(Cb0)
    with torch.cuda.graph(graph):
        calls()
    for _ in range(3):
        C.copy_(C0); t["C"].copy_(Cb0)
        (A.float().sum() + 1).item()              # unrelated eager work and a synchronisation between replays
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, eager_c) and torch.equal(t["C"], eager_b)


# ------------------------------------------------------------------ indirect route (padded copies) for ragged FP16

@pytest.mark.parametrize("ta,tb", [(N, N), (T, N), (N, T), (T, T)])
def test_indirect_route_for_ragged_half_problems(G, oracle, ta, tb):
    """large FP16 problems that are ragged or have odd leading dimensions run on zero-padded aligned copies in the
    workspace (the paper's Section 3.2 route): checked against the oracle, bit-exact on integers, nothing outside C
    written; without workspace, or with too little, the direct route runs and gives the same result"""
    import torch
    for (m, n, k), layout, beta, integer in (((1025, 2060, 1100), C, 0.0, True), ((1025, 2060, 1100), C, 0.5, False),
                                             ((1100, 2049, 1000), R, 1.0, True), ((2817, 3001, 500), C, 0.5, False),
                                             ((2817, 3001, 500), R, 1.0, True), ((2048, 1024, 1088), C, 0.25, False)):
        # (2817, 3001, 500) pads to 3072 x 3072 x 512, which runs on 256 x 256 direct-to-LDS tiles: their flavour with a
        # bounds-checked epilogue writes the caller's C directly (no copy of C in or out); odd leading dimensions in
        # every operand order, so that all four kernels of that flavour run
        # the last shape is whole tiles with odd leading dimensions: only the alignment breaks the fast path
        lds = {}
        if (m, n, k) == (2048, 1024, 1088):
            lds = dict(lda=W.tight_ld(layout, ta, m, k) + 1, ldb=W.tight_ld(layout, tb, k, n) + 1,
                       ldc=W.tight_ld(layout, N, m, n) + 1)
        if (m, n, k) == (2817, 3001, 500):
            odd = lambda ld: ld + 1 - ld % 2
            lds = dict(lda=odd(W.tight_ld(layout, ta, m, k)), ldb=odd(W.tight_ld(layout, tb, k, n)),
                       ldc=odd(W.tight_ld(layout, N, m, n)))
        case = W.hgemm_case(m, n, k, case=41, layout=layout, ta=ta, tb=tb, alpha=1.0, beta=beta, integer=integer, **lds)
        need = G.mg_gemm_workspace_bytes(G.MG_F16, case.layout, case.ta, case.tb, m, n, k, case.lda, case.ldb, case.ldc)
        assert need >= 2 * (m * k + k * n + m * n), "the query must ask for room for the padded copies"
        announce(case.name, "indirect", layout, ta, tb)
        H.check_case(case, oracle)                                  # workspace from the query: indirect route
        _, padded = H.run_gpu(case)
        for label, ws in (("no workspace", None), ("workspace too small for the copies", torch.empty(need - 256, dtype=torch.uint8, device="cuda"))):
            announce(case.name, label)
            st, direct = H.run_gpu(case, workspace=ws)
            assert st == 0
            H.assert_padding_untouched(case, direct)
            if integer:
                assert np.array_equal(H.bits(direct), H.bits(padded))
            else:
                live = ~W.padding_mask(case.layout, m, n, case.ldc, case.C.size)
                a, b = direct[live].astype(np.float64), padded[live].astype(np.float64)
                assert np.max(np.abs(a - b)) <= 4e-3 * np.max(np.abs(b)), "the two routes differ by more than rounding"


def test_aligned_whole_tile_problems_do_not_ask_for_copies(G):
    assert G.mg_gemm_workspace_bytes(G.MG_F16, C, N, N, 4096, 4096, 4096, 4096, 4096, 4096) == 0
    # too small for the copies to pay; slices of the sum (whole multiples of the FP32 result) are fine
    assert G.mg_gemm_workspace_bytes(G.MG_F32, C, N, N, 1000, 1000, 1000, 1000, 1000, 1000) % (1000 * 1000 * 4) == 0
    assert G.mg_gemm_workspace_bytes(G.MG_F16, C, N, N, 300, 300, 300, 300, 300, 300) == 0            # too small to pay


# ------------------------------------------------------------------ seeded random shapes through automatic selection

@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_random_shapes_on_sampled_entries(G, oracle, dtype):
    """two dozen seeded shapes (skinny, ragged, long and short K, padded and odd leading dimensions, every
    layout and operand order) through automatic selection with the workspace the query asks for: whatever
    tile, split factor or route is chosen, sampled entries must match the oracle and nothing outside C change"""
    g = np.random.default_rng(20251 if dtype == "f32" else 20252)
    for index in range(24):
        m, n = (int(g.choice([96, 129, 256, 700, 1024, 1500, 2049, 3000])) for _ in range(2))
        k = int(g.choice([64, 100, 512, 1000, 2304, 4096]))
        layout = int(g.choice([C, R]))
        ta, tb = int(g.choice([N, T])), int(g.choice([N, T]))
        beta = float(g.choice([0.0, 1.0, -0.5]))
        extra = int(g.choice([0, 0, 1, 8]))
        opA = W.uniform(g, (m, k)) if dtype == "f32" else (g.normal(0.0, k ** -0.5, size=(m, k))).astype(np.float16)
        opB = W.uniform(g, (k, n)) if dtype == "f32" else (g.normal(0.0, k ** -0.5, size=(k, n))).astype(np.float16)
        Cm = W.uniform(g, (m, n)) if dtype == "f32" else (g.normal(0.0, 1.0, size=(m, n))).astype(np.float16)
        case = W.make_case(f"rand{index}_{m}x{n}x{k}", dtype, layout, ta, tb, opA, opB, Cm, 1.0, beta,
                           W.tight_ld(layout, ta, m, k) + extra, W.tight_ld(layout, tb, k, n) + extra,
                           W.tight_ld(layout, N, m, n) + extra)
        announce(case.name, layout, ta, tb, "beta", beta, "ld +", extra)
        H.check_case(case, oracle, sampled=True, seed=index)


@pytest.mark.parametrize("layout,ta,tb", [(C, N, N), (R, T, N), (C, N, T)])
def test_large_ragged_single_problems_run_without_copies(G, oracle, layout, ta, tb):
    """a large ragged FP32 problem (a fringe row, partial last tiles, a ragged sum) needs no workspace: the
    bounds-checked tiles take it as it is (FP32 left the padded-copy route when they became faster than the copies);
    sampled entries against the oracle, padding of C untouched, the same bits with and without a workspace, and the
    same result up to summation order with the fringe switched off"""
    m, n, k = 2049, 2050, 2001
    g = np.random.default_rng(77)
    case = W.make_case(f"s_{m}x{n}x{k}", "f32", layout, ta, tb, W.uniform(g, (m, k)), W.uniform(g, (k, n)),
                       W.uniform(g, (m, n)), 1.0, 0.5, W.tight_ld(layout, ta, m, k) + 1, W.tight_ld(layout, tb, k, n) + 1,
                       W.tight_ld(layout, N, m, n) + 1)
    assert G.mg_gemm_workspace_bytes(G.MG_F32, layout, ta, tb, m, n, k, case.lda, case.ldb, case.ldc) == 0
    H.check_case(case, oracle, sampled=True, seed=5)
    import torch
    _, with_ws = H.run_gpu(case, workspace=torch.empty(64 << 20, dtype=torch.uint8, device="cuda"))
    st, direct = H.run_gpu(case, workspace=None)
    assert st == 0
    H.assert_padding_untouched(case, direct)
    assert np.array_equal(H.bits(with_ws), H.bits(direct))
    try:
        G.mg_override_fringe(G.MG_FRINGE_OFF)
        _, tiled = H.run_gpu(case, workspace=None)
    finally:
        G.mg_clear_override()
    live = ~W.padding_mask(layout, m, n, case.ldc, case.C.size)
    a, b = direct[live].astype(np.float64), tiled[live].astype(np.float64)
    assert np.max(np.abs(a - b)) <= 1e-4 * np.max(np.abs(b))
