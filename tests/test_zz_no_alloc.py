"""The entry point that brings its own scratch memory (mg_sgemm_static): same result as mg_sgemm with a caller
workspace of the same size, bit for bit, on two calls in a row on the one array (the second smaller, so that what
the first left behind does not matter), plus the oracle's verdict and the refusal of what does not fit."""
import numpy as np
import pytest

from paper_1705_05249_amd import gemm as G, workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _both_ways(case, oracle):
    import torch
    code = G.MG_F32
    sel = G.mg_query_selected(code, case.layout, case.ta, case.tb, case.m, case.n, case.k, case.lda, case.ldb, case.ldc,
                              case.alpha, case.beta)
    assert sel["split_k"] > 1, f"{case.name}: the case must use the scratch memory ({sel})"
    need = G.mg_gemm_workspace_bytes(code, case.layout, case.ta, case.tb, case.m, case.n, case.k, case.lda, case.ldb, case.ldc)
    assert 0 < need <= G.MG_STATIC_SCRATCH_BYTES
    A, B = H.to_gpu(case.A), H.to_gpu(case.B)
    c_ws, c_static = H.to_gpu(case.C), H.to_gpu(case.C)
    ws = torch.empty(G.MG_STATIC_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
    print("mg_sgemm with workspace:", case.name, flush=True)
    G.mg_sgemm(case.layout, case.ta, case.tb, case.m, case.n, case.k, case.alpha, A, case.lda, B, case.ldb, case.beta,
               c_ws, case.ldc, ws)
    print("mg_sgemm_static:", case.name, flush=True)
    G.mg_sgemm_static(case.layout, case.ta, case.tb, case.m, case.n, case.k, case.alpha, A, case.lda, B, case.ldb,
                      case.beta, c_static, case.ldc)
    torch.cuda.synchronize()
    out_ws, out_static = c_ws.cpu().numpy(), c_static.cpu().numpy()
    assert np.array_equal(H.bits(out_ws), H.bits(out_static)), f"{case.name}: the two entry points differ"
    H.assert_padding_untouched(case, out_static)
    got = W.unpack(out_static, case.layout, case.m, case.n, case.ldc)
    c_ref, d_ref = oracle.gemm(case.dtype, case.layout, case.ta, case.tb, case.m, case.n, case.k, case.alpha, case.A,
                                    case.lda, case.B, case.ldb, case.beta, case.C, case.ldc)
    if case.exact:
        assert np.array_equal(got.astype(np.float64), c_ref), f"{case.name}: not bit-exact"
    else:
        assert H.rel_error(got, c_ref, d_ref) <= H.TOL["f32"]


def test_static_scratch_entry_point_matches_the_workspace_one(oracle):
    G.lib()
    G.mg_clear_override()
    # long sums over few outputs: split into slices whose partial sums go through the scratch memory
    first = W.skinny_case(256, 192, 8192, case=71, beta=0.5)
    second = W.skinny_case(64, 128, 4096, case=72, integer=True, ta=W.NO_TRANS, tb=W.TRANS, beta=1.0)
    _both_ways(first, oracle)
    _both_ways(second, oracle)
    _both_ways(first, oracle)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    G.lib()
    G.mg_clear_override()
    m, n, k = 1536, 1024, 32768          # a long sum in eight slices: 48 MiB of partial sums
    need = G.mg_gemm_workspace_bytes(G.MG_F32, W.COL_MAJOR, W.NO_TRANS, W.NO_TRANS, m, n, k, m, k, m)
    assert need > G.MG_STATIC_SCRATCH_BYTES
    # refused on the host before any pointer is looked at
    st = G.mg_sgemm_static(W.COL_MAJOR, W.NO_TRANS, W.NO_TRANS, m, n, k, 1.0, 4096, m, 4096, k, 0.0, 4096, m, check=False)
    assert st == -10          # MG_ERR_WORKSPACE
    # argument errors are reported as by mg_sgemm
    assert G.mg_sgemm_static(W.COL_MAJOR, W.NO_TRANS, W.NO_TRANS, 8, 8, 8, 1.0, 4096, 7, 4096, 8, 0.0, 4096, 8, check=False) == -5   # MG_ERR_LDA
