"""GPU parity of the stand-alone matrix-vector entry points (the level-2 routine of paper Section 4.2)
against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest

import helpers as H
from paper_1705_05249_amd import gemm as G
from paper_1705_05249_amd import workloads as W

pytestmark = pytest.mark.gpu

R, C, N, T = W.ROW_MAJOR, W.COL_MAJOR, W.NO_TRANS, W.TRANS


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout", [C, R])
@pytest.mark.parametrize("trans", [N, T])
@pytest.mark.parametrize("shape", [(1, 1), (3, 5), (64, 64), (257, 130), (1000, 37), (37, 1000), (1, 300), (300, 1),
                                   (2051, 515)])
def test_every_order_unit_increments(oracle, dtype, layout, trans, shape):
    m, n = shape
    case = W.gemv_case(dtype, layout, trans, m, n, alpha=1.25, beta=-0.5, case=m * 7 + n)
    H.check_gemv(case, oracle)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout,trans", [(C, N), (C, T), (R, N), (R, T)])
@pytest.mark.parametrize("incx,incy,pad", [(2, 1, 0), (1, 3, 1), (5, 4, 3)])
def test_increments_and_padded_lda(oracle, dtype, layout, trans, incx, incy, pad):
    case = W.gemv_case(dtype, layout, trans, 193, 301, incx=incx, incy=incy, alpha=-0.75, beta=1.5, pad=pad,
                       case=incx * 10 + incy)
    H.check_gemv(case, oracle)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout,trans", [(C, N), (C, T), (R, N), (R, T)])
def test_integer_inputs_are_exact(oracle, dtype, layout, trans):
    case = W.gemv_case(dtype, layout, trans, 515, 260, incx=2, incy=2, alpha=2.0, beta=-1.0, integer=True, case=3)
    H.check_gemv(case, oracle)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_scalar_conventions(oracle, dtype):
    """beta == 0: y is overwritten even where it held NaN; alpha == 0: A and x may hold NaN; an empty sum scales y"""
    case = W.gemv_case(dtype, C, N, 70, 45, incy=2, alpha=1.0, beta=0.0, case=11)
    case.y[::2] = np.nan
    H.check_gemv(case, oracle)
    case = W.gemv_case(dtype, R, T, 70, 45, incx=2, alpha=0.0, beta=0.5, case=12)
    case.A[:] = np.nan
    case.x[:] = np.nan
    H.check_gemv(case, oracle)
    case = W.gemv_case(dtype, C, N, 33, 0, alpha=1.0, beta=2.0, case=13)
    H.check_gemv(case, oracle)
    case = W.gemv_case(dtype, C, T, 33, 0, alpha=1.0, beta=2.0, case=14)       # no output at all
    st, out = H.run_gemv(case)
    assert st == 0 and np.array_equal(H.bits(out), H.bits(case.y))


@pytest.mark.parametrize("dtype,shape", [("f32", (4096, 4096)), ("f16", (8192, 4096)), ("f32", (16384, 1024))])
@pytest.mark.parametrize("layout,trans", [(C, N), (C, T)])
def test_large_matrices(oracle, dtype, shape, layout, trans):
    """the sizes the timing runs use"""
    case = W.gemv_case(dtype, layout, trans, *shape, alpha=1.0, beta=1.0, case=21)
    H.check_gemv(case, oracle)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout,trans", [(C, N), (C, T), (R, N), (R, T)])
@pytest.mark.parametrize("shape", [(40, 9000), (9000, 40), (700, 5000), (1, 70000), (70000, 1), (3, 4099)])
@pytest.mark.parametrize("workspace", ["auto", None, 4096])
def test_few_outputs_and_a_long_sum(oracle, dtype, layout, trans, shape, workspace):
    """shapes whose sum is cut into slices when the workspace allows: full, none, and room for a few slices only"""
    import torch
    m, n = shape
    case = W.gemv_case(dtype, layout, trans, m, n, incx=1, incy=2, alpha=0.5, beta=2.0, pad=1, case=m + n)
    ws = torch.empty(workspace, dtype=torch.uint8, device="cuda") if isinstance(workspace, int) else workspace
    H.check_gemv(case, oracle, workspace=ws)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_sliced_sum_of_integers_is_exact(oracle, dtype):
    for layout, trans in ((C, N), (C, T)):
        case = W.gemv_case(dtype, layout, trans, 50, 8200, alpha=1.0, beta=1.0, integer=True, case=5)
        case2 = W.gemv_case(dtype, layout, trans, 8200, 50, alpha=1.0, beta=1.0, integer=True, case=6)
        H.check_gemv(case, oracle)
        H.check_gemv(case2, oracle)


def test_same_result_as_the_gemm_entry_point_with_one_column(oracle):
    """the stand-alone call and the n = 1 GEMM run the same kernel: same bits"""
    import torch
    case = W.gemv_case("f32", C, N, 777, 333, alpha=1.5, beta=0.25, case=31)
    _, out = H.run_gemv(case, workspace=None)
    A, x, y = H.to_gpu(case.A), H.to_gpu(case.x), H.to_gpu(case.y)
    G.mg_sgemm(C, N, N, 777, 1, 333, 1.5, A, case.lda, x, 333, 0.25, y, 777)
    torch.cuda.synchronize()
    assert np.array_equal(H.bits(out), H.bits(y.cpu().numpy()))


def test_benchmark_size(oracle):
    """16384 x 16384 FP32, column-major, both orders: the calls the benchmark times, every output checked
    (one seeded matrix serves both: it is square)"""
    import dataclasses
    case = W.gemv_case("f32", C, N, 16384, 16384, alpha=1.0, beta=0.0, case=41)
    H.check_gemv(case, oracle)
    H.check_gemv(dataclasses.replace(case, trans=T), oracle)
