"""Pins for the CPU oracle (no GPU needed).

The oracle is checked against things other than itself: a hand-computed example with literal
expected values, closed forms, algebraic identities of matrix multiplication, numpy's FP64
matmul as an independent library routine, and numpy's own binary16 decoding.  Each pin is
chosen so that a plausible slip (dropped beta term, wrong leading dimension, transposed
operand, row/col mix-up, wrong offset array) fails at least one of them.
"""
import os

import numpy as np
import pytest

from paper_1705_05249_amd import workloads as W

R, Cm, N, T = W.ROW_MAJOR, W.COL_MAJOR, W.NO_TRANS, W.TRANS
VARIANTS = [(lay, ta, tb) for lay in (R, Cm) for ta in (N, T) for tb in (N, T)]
GOLD = os.path.join(os.path.dirname(__file__), "golden", "handsized.txt")


def run(oracle, case):
    return oracle.gemm(case.dtype, case.layout, case.ta, case.tb, case.m, case.n, case.k,
                       case.alpha, case.A, case.lda, case.B, case.ldb, case.beta, case.C, case.ldc)


def read_golden():
    blocks, name = {}, None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line[0].isalpha():
            name = line
            blocks[name] = []
        else:
            blocks[name].append([float(x) for x in line.split()])
    return {k: np.array(v) for k, v in blocks.items()}


# ---------------------------------------------------------------- literal hand-sized example

@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
@pytest.mark.parametrize("pad", [0, 3])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_handsized_literal(oracle, layout, ta, tb, pad, dtype):
    g = read_golden()
    opA, opB, C = g["opA"], g["opB"], g["C"]
    m, k = opA.shape
    n = opB.shape[1]
    lda = W.tight_ld(layout, ta, m, k) + pad
    ldb = W.tight_ld(layout, tb, k, n) + 2 * pad
    ldc = W.tight_ld(layout, N, m, n) + 3 * pad
    case = W.make_case("hand", dtype, layout, ta, tb, opA, opB, C, 2.0, -1.0, lda, ldb, ldc)
    c_ref, d_ref = run(oracle, case)
    assert np.array_equal(c_ref, g["expected_C"])
    assert np.array_equal(d_ref, g["expected_D"])


def test_dropping_a_term_would_be_seen():
    """the golden example separates alpha, beta, |.| and the transposes: none of these
    wrong formulas reproduces the expected values"""
    g = read_golden()
    opA, opB, C, exp = g["opA"], g["opB"], g["C"], g["expected_C"]
    assert not np.array_equal(2 * opA @ opB, exp)                    # beta term dropped
    assert not np.array_equal(2 * opA @ opB + C, exp)                # sign of beta
    assert not np.array_equal(opA @ opB - C, exp)                    # alpha dropped
    assert not np.array_equal(2 * np.abs(opA) @ np.abs(opB) + np.abs(C), exp)
    assert np.array_equal(2 * np.abs(opA) @ np.abs(opB) + np.abs(C), g["expected_D"])


# ---------------------------------------------------------------- special values of alpha, beta, k

@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
def test_alpha_zero_gives_beta_c_and_ignores_nan_inputs(oracle, layout, ta, tb):
    g = W.rng_for(90, 1)
    m, n, k = 5, 7, 6
    opA = np.full((m, k), np.nan, dtype=np.float32)
    opB = np.full((k, n), np.inf, dtype=np.float32)
    C = W.uniform(g, (m, n))
    case = W.make_case("a0", "f32", layout, ta, tb, opA, opB, C, 0.0, 0.75)
    c_ref, d_ref = run(oracle, case)
    assert np.array_equal(c_ref, 0.75 * C.astype(np.float64))
    assert np.array_equal(d_ref, 0.75 * np.abs(C.astype(np.float64)))


@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
def test_beta_zero_never_reads_c(oracle, layout, ta, tb):
    g = W.rng_for(90, 2)
    m, n, k = 4, 3, 9
    opA, opB = W.small_ints(g, (m, k)), W.small_ints(g, (k, n))
    C = np.full((m, n), np.nan, dtype=np.float32)
    case = W.make_case("b0", "f32", layout, ta, tb, opA, opB, C, -3.0, 0.0)
    c_ref, d_ref = run(oracle, case)
    assert np.array_equal(c_ref, -3.0 * (opA.astype(np.float64) @ opB.astype(np.float64)))
    assert np.all(np.isfinite(d_ref))


def test_k_zero_and_empty_outputs(oracle):
    C = np.arange(6, dtype=np.float32).reshape(2, 3)
    case = W.make_case("k0", "f32", Cm, N, N, np.zeros((2, 0), np.float32), np.zeros((0, 3), np.float32),
                       C, 5.0, 2.0)
    c_ref, d_ref = run(oracle, case)
    assert np.array_equal(c_ref, 2.0 * C) and np.array_equal(d_ref, 2.0 * C)
    for m, n in ((0, 3), (3, 0)):
        c_ref, d_ref = oracle.gemm("f32", Cm, N, N, m, n, 4, 1.0, np.zeros(16, np.float32), max(1, m),
                                   np.zeros(16, np.float32), 4, 1.0, np.zeros(16, np.float32), max(1, m))
        assert c_ref.shape == (m, n) and d_ref.shape == (m, n)


# ---------------------------------------------------------------- identity / permutation

@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
def test_identity_and_permutation(oracle, layout, ta, tb):
    g = W.rng_for(90, 3)
    m, n = 6, 5
    X = W.uniform(g, (m, n))
    C = W.uniform(g, (m, n))
    perm = g.permutation(m)
    P = np.zeros((m, m), dtype=np.float32)
    P[np.arange(m), perm] = 1.0                         # (P X)(i,:) = X(perm[i],:)
    case = W.make_case("perm", "f32", layout, ta, tb, P, X, C, 1.0, 0.0)
    c_ref, _ = run(oracle, case)
    assert np.array_equal(c_ref, X[perm].astype(np.float64))
    # identity on the right, with alpha and beta
    case = W.make_case("id", "f32", layout, ta, tb, X, np.eye(n, dtype=np.float32), C, 2.0, -0.5)
    c_ref, _ = run(oracle, case)
    assert np.array_equal(c_ref, 2.0 * X.astype(np.float64) - 0.5 * C.astype(np.float64))
    # column permutation on the right: (X Q)(:,j) = X(:, q[j]) when Q[q[j], j] = 1
    q = g.permutation(n)
    Q = np.zeros((n, n), dtype=np.float32)
    Q[q, np.arange(n)] = 1.0
    case = W.make_case("permR", "f32", layout, ta, tb, X, Q, C, 1.0, 0.0)
    c_ref, _ = run(oracle, case)
    assert np.array_equal(c_ref, X[:, q].astype(np.float64))


# ---------------------------------------------------------------- closed forms

@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
def test_closed_forms(oracle, layout, ta, tb):
    m, n, k = 7, 5, 11
    alpha, beta, c0 = 1.5, 0.25, 3.0
    ones = lambda s: np.ones(s, dtype=np.float32)
    case = W.make_case("ones", "f32", layout, ta, tb, ones((m, k)), ones((k, n)), c0 * ones((m, n)), alpha, beta)
    c_ref, d_ref = run(oracle, case)
    assert np.all(c_ref == alpha * k + beta * c0) and np.all(d_ref == alpha * k + beta * c0)
    # rank one: A(i,l) = i+1, B(l,j) = j+1  ->  k (i+1)(j+1)
    i1 = np.arange(1, m + 1, dtype=np.float32)[:, None]
    j1 = np.arange(1, n + 1, dtype=np.float32)[None, :]
    case = W.make_case("rank1", "f32", layout, ta, tb, i1 * ones((m, k)), ones((k, n)) * j1, c0 * ones((m, n)),
                       alpha, beta)
    c_ref, _ = run(oracle, case)
    assert np.array_equal(c_ref, alpha * k * (i1 * j1).astype(np.float64) + beta * c0)
    # A(i,l) = l+1, B = 1  ->  k(k+1)/2 ;  A(i,l) = (-1)^l (l+1)  ->  alternating sum, D keeps k(k+1)/2
    l1 = np.arange(1, k + 1, dtype=np.float32)[None, :]
    case = W.make_case("tri", "f32", layout, ta, tb, ones((m, k)) * l1, ones((k, n)), ones((m, n)), 1.0, 0.0)
    c_ref, _ = run(oracle, case)
    assert np.all(c_ref == k * (k + 1) / 2)
    sign = np.where(np.arange(k) % 2 == 0, 1.0, -1.0).astype(np.float32)[None, :]
    case = W.make_case("alt", "f32", layout, ta, tb, ones((m, k)) * l1 * sign, ones((k, n)), ones((m, n)), 1.0, 0.0)
    c_ref, d_ref = run(oracle, case)
    assert np.all(c_ref == (k + 1) // 2) and np.all(d_ref == k * (k + 1) / 2)     # k odd: 1-2+3-...+k
    # shifted delta: A(i,l) = [l == i+2]  picks row i+2 of B
    kk = m + 2
    S = np.zeros((m, kk), dtype=np.float32)
    S[np.arange(m), np.arange(m) + 2] = 1.0
    Bm = W.uniform(W.rng_for(90, 4), (kk, n))
    case = W.make_case("shift", "f32", layout, ta, tb, S, Bm, ones((m, n)), 1.0, 0.0)
    c_ref, _ = run(oracle, case)
    assert np.array_equal(c_ref, Bm[2:].astype(np.float64))


# ---------------------------------------------------------------- identities between calls

@pytest.mark.parametrize("ta,tb", [(N, N), (N, T), (T, N), (T, T)])
def test_transpose_identity_bitwise(oracle, ta, tb):
    """op(A)op(B) = (op(B)^T op(A)^T)^T : swapping operands and flipping both ops gives the transpose"""
    g = W.rng_for(90, 5)
    m, n, k = 9, 6, 13
    opA, opB, C = W.uniform(g, (m, k)), W.uniform(g, (k, n)), W.uniform(g, (m, n))
    c1, d1 = run(oracle, W.make_case("t1", "f32", Cm, ta, tb, opA, opB, C, 1.25, -0.5, m + k + 1, n + k + 2, m + 3))
    flip = lambda t: T if t == N else N
    # second call: op'(A') = op(B)^T (n x k), op'(B') = op(A)^T (k x m), C' = C^T
    c2, d2 = run(oracle, W.make_case("t2", "f32", Cm, flip(tb), flip(ta), opB.T.copy(), opA.T.copy(), C.T.copy(),
                                    1.25, -0.5))
    assert np.array_equal(c1, c2.T) and np.array_equal(d1, d2.T)


@pytest.mark.parametrize("ta,tb", [(N, N), (N, T), (T, N), (T, T)])
def test_row_and_column_major_agree_bitwise(oracle, ta, tb):
    g = W.rng_for(90, 6)
    m, n, k = 8, 11, 5
    opA, opB, C = W.uniform(g, (m, k)), W.uniform(g, (k, n)), W.uniform(g, (m, n))
    outs = [run(oracle, W.make_case("rc", "f32", lay, ta, tb, opA, opB, C, 0.5, 2.0, 14, 15, 16)) for lay in (R, Cm)]
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])


def test_linearity_in_alpha_beta(oracle):
    g = W.rng_for(90, 7)
    m, n, k = 6, 6, 10
    opA, opB, C = W.small_ints(g, (m, k)), W.small_ints(g, (k, n)), W.small_ints(g, (m, n))
    base, _ = run(oracle, W.make_case("l0", "f32", Cm, N, T, opA, opB, C, 1.0, 0.0))
    full, _ = run(oracle, W.make_case("l1", "f32", Cm, N, T, opA, opB, C, 1.5, 0.5))
    assert np.array_equal(full, 1.5 * base + 0.5 * C.astype(np.float64))


# ---------------------------------------------------------------- library routine on random inputs

@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
@pytest.mark.parametrize("shape", [(33, 17, 64), (1, 40, 129), (130, 1, 77), (64, 64, 1)])
def test_against_numpy_fp64(oracle, layout, ta, tb, shape):
    m, n, k = shape
    g = W.rng_for(90, 8)
    opA, opB, C = W.uniform(g, (m, k)), W.uniform(g, (k, n)), W.uniform(g, (m, n))
    lda = W.tight_ld(layout, ta, m, k) + 5
    ldb = W.tight_ld(layout, tb, k, n) + 1
    ldc = W.tight_ld(layout, N, m, n) + 2
    c_ref, d_ref = run(oracle, W.make_case("np", "f32", layout, ta, tb, opA, opB, C, 1.3, -0.7, lda, ldb, ldc))
    a64, b64, c64 = (x.astype(np.float64) for x in (opA, opB, C))
    want = 1.3 * (a64 @ b64) - 0.7 * c64
    den = 1.3 * (np.abs(a64) @ np.abs(b64)) + 0.7 * np.abs(c64)
    assert np.max(np.abs(c_ref - want) / den) <= (k + 4) * 2.0 ** -53
    assert np.max(np.abs(d_ref - den) / den) <= (k + 4) * 2.0 ** -53


def test_config1_integer_case_is_exact_and_matches_numpy(oracle):
    case = W.config1(integer=True)
    c_ref, _ = run(oracle, case)
    A = W.unpack(case.A, Cm, 256, 256, 256).astype(np.float64)
    B = W.unpack(case.B, Cm, 256, 256, 256).astype(np.float64)
    C = W.unpack(case.C, Cm, 256, 256, 256).astype(np.float64)
    assert np.array_equal(c_ref, 1.5 * (A @ B) + 0.5 * C)          # all integers / halves: exact in any order
    assert np.array_equal(c_ref, c_ref.astype(np.float32).astype(np.float64))   # representable in FP32


# ---------------------------------------------------------------- FP16 storage

def test_half_decoding_all_bit_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    mine = oracle.half_to_double(bits)
    ref = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(mine), nan)
    assert np.array_equal(mine[~nan], ref[~nan])
    assert np.array_equal(np.signbit(mine[~nan]), np.signbit(ref[~nan]))
    # a few values fixed by the format itself
    for pattern, value in ((0x3C00, 1.0), (0xC000, -2.0), (0x7BFF, 65504.0), (0x0001, 2.0 ** -24),
                           (0x0400, 2.0 ** -14), (0x3555, 0.333251953125)):
        assert oracle.half_to_double(np.array([pattern], dtype=np.uint16))[0] == value


@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
def test_fp16_against_numpy_fp64(oracle, layout, ta, tb):
    case = W.hgemm_case(21, 34, 150, case=77, layout=layout, ta=ta, tb=tb, alpha=0.5, beta=2.0)
    c_ref, d_ref = run(oracle, case)
    m, n, k = case.m, case.n, case.k
    rA, cA = W.stored_extents(ta, m, k)
    rB, cB = W.stored_extents(tb, k, n)
    SA = W.unpack(case.A, layout, rA, cA, case.lda).astype(np.float64)
    SB = W.unpack(case.B, layout, rB, cB, case.ldb).astype(np.float64)
    C = W.unpack(case.C, layout, m, n, case.ldc).astype(np.float64)
    a = SA if ta == N else SA.T
    b = SB if tb == N else SB.T
    want = 0.5 * (a @ b) + 2.0 * C
    den = 0.5 * (np.abs(a) @ np.abs(b)) + 2.0 * np.abs(C)
    assert np.max(np.abs(c_ref - want) / den) <= (k + 4) * 2.0 ** -53
    assert np.max(np.abs(d_ref - den) / den) <= (k + 4) * 2.0 ** -53


def test_fp16_subnormal_inputs_are_honoured(oracle):
    m = n = k = 4
    A = np.full((m, k), 2.0 ** -24, dtype=np.float16)      # smallest subnormal
    B = np.full((k, n), 1024.0, dtype=np.float16)
    c_ref, _ = run(oracle, W.make_case("sub", "f16", Cm, N, N, A, B, np.zeros((m, n), np.float16), 1.0, 0.0))
    assert np.all(c_ref == k * 2.0 ** -14)


# ---------------------------------------------------------------- sampled entries

def test_entries_equal_full(oracle):
    case = W.skinny_case(37, 29, 53, case=11)
    c_ref, d_ref = run(oracle, case)
    rows, cols = W.sample_entries(case.m, case.n, seed=5, rows=4, cols=4, tile=16, scattered=50)
    ce, de = oracle.gemm_entries(case.dtype, case.layout, case.ta, case.tb, case.m, case.n, case.k, case.alpha,
                                 case.A, case.lda, case.B, case.ldb, case.beta, case.C, case.ldc, rows, cols)
    assert np.array_equal(ce, c_ref[rows, cols]) and np.array_equal(de, d_ref[rows, cols])
    h = W.hgemm_case(19, 23, 40, case=3, ta=T, tb=T, beta=1.0)
    c_ref, d_ref = run(oracle, h)
    rows, cols = W.sample_entries(h.m, h.n, seed=6, rows=3, cols=3, tile=8, scattered=20)
    ce, de = oracle.gemm_entries("f16", h.layout, h.ta, h.tb, h.m, h.n, h.k, h.alpha, h.A, h.lda, h.B, h.ldb,
                                 h.beta, h.C, h.ldc, rows, cols)
    assert np.array_equal(ce, c_ref[rows, cols]) and np.array_equal(de, d_ref[rows, cols])


# ---------------------------------------------------------------- batched form

def run_batched(oracle, bc):
    return oracle.sgemm_batched(bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, bc.alphas, bc.A, bc.a_off, bc.lda,
                                bc.B, bc.b_off, bc.ldb, bc.betas, bc.C, bc.c_off, bc.ldc)


@pytest.mark.parametrize("layout,ta,tb", VARIANTS)
def test_batched_equals_numpy_per_instance(oracle, layout, ta, tb):
    """per-instance offsets, alpha and beta are honoured: each instance equals numpy's FP64
    product of the data found at that instance's own offsets (offsets shuffled, different per buffer)"""
    bc = W.batched_case(5, 7, 6, 9, case=1, layout=layout, ta=ta, tb=tb, shuffle_offsets=True)
    c_ref, d_ref = run_batched(oracle, bc)
    for i in range(bc.batch):
        rA, cA = W.stored_extents(ta, bc.m, bc.k)
        rB, cB = W.stored_extents(tb, bc.k, bc.n)
        SA = W.unpack(bc.A[bc.a_off[i]:], layout, rA, cA, bc.lda).astype(np.float64)
        SB = W.unpack(bc.B[bc.b_off[i]:], layout, rB, cB, bc.ldb).astype(np.float64)
        C = W.unpack(bc.C[bc.c_off[i]:], layout, bc.m, bc.n, bc.ldc).astype(np.float64)
        a = SA if ta == N else SA.T
        b = SB if tb == N else SB.T
        al, be = float(bc.alphas[i]), float(bc.betas[i])
        want = al * (a @ b) + be * C
        den = al * (np.abs(a) @ np.abs(b)) + be * np.abs(C)
        assert np.max(np.abs(c_ref[i] - want) / den) <= 16 * 2.0 ** -53
        assert np.max(np.abs(d_ref[i] - den) / den) <= 16 * 2.0 ** -53


def test_batched_equals_loop_of_singles_bitwise(oracle):
    bc = W.batched_case(8, 8, 8, 12, case=2, shuffle_offsets=True)
    c_ref, d_ref = run_batched(oracle, bc)
    for i in range(bc.batch):
        c1, d1 = oracle.gemm("f32", bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, float(bc.alphas[i]),
                             bc.A[bc.a_off[i]:], bc.lda, bc.B[bc.b_off[i]:], bc.ldb, float(bc.betas[i]),
                             bc.C[bc.c_off[i]:], bc.ldc)
        assert np.array_equal(c_ref[i], c1) and np.array_equal(d_ref[i], d1)


def test_half_batched_equals_loop_of_singles_bitwise(oracle):
    """FP16 storage: the batched oracle is the FP16 single-call oracle per instance (offsets in elements of
    the 2-byte type, FP32 scalars), bit for bit"""
    for layout, ta, tb in ((Cm, N, N), (R, T, N), (Cm, T, T)):
        bc = W.batched_case(7, 5, 9, 11, case=3, layout=layout, ta=ta, tb=tb, shuffle_offsets=True, dtype="f16")
        assert bc.A.dtype == np.float16
        c_ref, d_ref = oracle.gemm_batched("f16", bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, bc.alphas, bc.A, bc.a_off,
                                           bc.lda, bc.B, bc.b_off, bc.ldb, bc.betas, bc.C, bc.c_off, bc.ldc)
        for i in range(bc.batch):
            c1, d1 = oracle.gemm("f16", bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, float(bc.alphas[i]),
                                 bc.A[bc.a_off[i]:], bc.lda, bc.B[bc.b_off[i]:], bc.ldb, float(bc.betas[i]),
                                 bc.C[bc.c_off[i]:], bc.ldc)
            assert np.array_equal(c_ref[i], c1) and np.array_equal(d_ref[i], d1)
        # and an instance against numpy on the widened data
        rA, cA = W.stored_extents(ta, bc.m, bc.k)
        rB, cB = W.stored_extents(tb, bc.k, bc.n)
        i = 4
        SA = W.unpack(bc.A[bc.a_off[i]:], layout, rA, cA, bc.lda).astype(np.float64)
        SB = W.unpack(bc.B[bc.b_off[i]:], layout, rB, cB, bc.ldb).astype(np.float64)
        C0 = W.unpack(bc.C[bc.c_off[i]:], layout, bc.m, bc.n, bc.ldc).astype(np.float64)
        a = SA if ta == N else SA.T
        b = SB if tb == N else SB.T
        want = float(bc.alphas[i]) * (a @ b) + float(bc.betas[i]) * C0
        assert np.max(np.abs(c_ref[i] - want)) <= 1e-13


def test_batched_distinct_offset_arrays(oracle):
    """A, B and C use their own offset arrays (a mix-up between them changes the result)"""
    g = W.rng_for(90, 9)
    s, batch = 3, 4
    mats = [[W.small_ints(g, (s, s)) for _ in range(batch)] for _ in range(3)]
    orders = [g.permutation(batch) for _ in range(3)]
    bufs, offs = [], []
    for which in range(3):
        buf = np.full(batch * (s * s + 2), np.nan, dtype=np.float32)
        off = orders[which].astype(np.int64) * (s * s + 2)
        for i in range(batch):
            buf[off[i]: off[i] + s * s] = W.pack(mats[which][i], Cm, N)
        bufs.append(buf)
        offs.append(off)
    alphas = np.array([1, 2, 3, 4], dtype=np.float32)
    betas = np.array([-1, 0.5, 0, 2], dtype=np.float32)
    bufs[2][np.isnan(bufs[2])] = 0
    c_ref, _ = oracle.sgemm_batched(Cm, N, N, s, s, s, alphas, bufs[0], offs[0], s, bufs[1], offs[1], s,
                                    betas, bufs[2], offs[2], s)
    for i in range(batch):
        want = float(alphas[i]) * (mats[0][i].astype(np.float64) @ mats[1][i].astype(np.float64)) \
            + float(betas[i]) * mats[2][i].astype(np.float64)
        assert np.array_equal(c_ref[i], want)


def test_strided_batched_is_the_generic_one_with_regular_offsets(oracle):
    """pins the strided wrapper: per instance it equals numpy's product of the data found at b*stride"""
    g = W.rng_for(90, 12)
    m, n, k, batch = 4, 3, 5, 6
    sa, sb, sc = m * k + 2, k * n + 1, m * n + 4
    A = W.small_ints(g, batch * sa); B = W.small_ints(g, batch * sb); C0 = W.small_ints(g, batch * sc)
    c_ref, d_ref = oracle.sgemm_strided_batched(Cm, N, T, m, n, k, 1.5, A, m, sa, B, n, sb, -0.5, C0, m, sc, batch)
    for b in range(batch):
        a = W.unpack(A[b * sa:], Cm, m, k, m).astype(np.float64)
        bt = W.unpack(B[b * sb:], Cm, n, k, n).astype(np.float64)          # stored n x k, op = transpose
        c = W.unpack(C0[b * sc:], Cm, m, n, m).astype(np.float64)
        assert np.array_equal(c_ref[b], 1.5 * (a @ bt.T) - 0.5 * c)
        assert np.array_equal(d_ref[b], 1.5 * (np.abs(a) @ np.abs(bt.T)) + 0.5 * np.abs(c))


# ---------------------------------------------------------------- input generator sanity

def test_padded_ld_reading():
    assert [W.padded_ld(x) for x in (999, 4095, 4096, 64, 1, 129, 1000, 4097, 8192)] == \
        [1001, 4097, 4097, 65, 9, 137, 1001, 4105, 8193]


def test_pack_unpack_roundtrip_and_padding_mask():
    g = W.rng_for(90, 10)
    X = W.uniform(g, (5, 3))
    for lay in (R, Cm):
        ld = W.tight_ld(lay, N, 5, 3) + 4
        buf = W.pack(X, lay, N, ld)
        assert np.array_equal(W.unpack(buf, lay, 5, 3, ld), X)
        mask = W.padding_mask(lay, 5, 3, ld, buf.size)
        assert mask.sum() == buf.size - 15 and np.all(np.isnan(buf[mask])) and not np.any(np.isnan(buf[~mask]))
        bt = W.pack(X, lay, T, None)
        assert np.array_equal(W.unpack(bt, lay, 3, 5, W.tight_ld(lay, T, 5, 3)), X.T)


def test_config_shapes_follow_the_recipe():
    c = W.config5(0)
    assert (c.m, c.n, c.k, c.lda, c.ldb, c.ldc, c.ta, c.tb) == (1000, 1001, 999, 1001, 1001, 1001, T, N)
    b = W.config4(16, 1000)
    assert b.A.size == 1000 * (256 + 7) and b.a_off[3] == 3 * 263 and b.alphas.min() >= 0.5 and b.betas.max() <= 2.0
    h = W.config3(0)
    assert h.A.dtype == np.float16 and (h.m, h.n, h.k, h.lda, h.ldb, h.ldc) == (64, 12544, 147, 64, 147, 64)
    assert abs(float(np.std(h.B.astype(np.float64))) - 147 ** -0.5) < 2e-3


# ---------------------------------------------------------------- matrix-vector product

@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout", [Cm, R])
@pytest.mark.parametrize("trans", [N, T])
def test_gemv_against_numpy_and_the_gemm_oracle(oracle, dtype, layout, trans):
    """y = alpha op(A) x + beta y with strided x and y: numpy on the widened data, and the GEMM oracle on the
    same problem written as an n = 1 product (bit for bit: same summation order)"""
    m, n, lda, incx, incy = 7, 5, 9, 3, 2
    g = np.random.default_rng(31)
    np_t = np.float32 if dtype == "f32" else np.float16
    Am = g.uniform(-1, 1, size=(m, n)).astype(np_t)
    A = W.pack(Am, layout, N, lda)
    rows, length = (m, n) if trans == N else (n, m)
    xs = g.uniform(-1, 1, size=length).astype(np_t)
    ys = g.uniform(-1, 1, size=rows).astype(np_t)
    x = np.full((length - 1) * incx + 1, np.nan, np_t); x[::incx] = xs
    y = np.full((rows - 1) * incy + 1, np.nan, np_t); y[::incy] = ys
    y_ref, d_ref = oracle.gemv(dtype, layout, trans, m, n, -1.5, A, lda, x, incx, 0.75, y, incy)
    op = Am.astype(np.float64) if trans == N else Am.astype(np.float64).T
    want = -1.5 * (op @ xs.astype(np.float64)) + 0.75 * ys.astype(np.float64)
    den = 1.5 * (np.abs(op) @ np.abs(xs.astype(np.float64))) + 0.75 * np.abs(ys.astype(np.float64))
    assert np.max(np.abs(y_ref - want)) <= 1e-14 and np.max(np.abs(d_ref - den)) <= 1e-14
    c_ref, dd = oracle.gemm(dtype, layout, trans, N, rows, 1, length, -1.5, A, lda,
                            W.pack(xs.reshape(length, 1), layout, N), W.tight_ld(layout, N, length, 1), 0.75,
                            W.pack(ys.reshape(rows, 1), layout, N), W.tight_ld(layout, N, rows, 1))
    assert np.array_equal(c_ref[:, 0], y_ref) and np.array_equal(dd[:, 0], d_ref)


def test_gemv_conventions(oracle):
    A = np.full(12, np.nan, np.float32)
    y = np.arange(1, 4, dtype=np.float32)
    y_ref, d_ref = oracle.gemv("f32", Cm, N, 3, 4, 0.0, A, 3, np.full(4, np.nan, np.float32), 1, 2.0, y, 1)
    assert np.array_equal(y_ref, 2.0 * y) and np.array_equal(d_ref, 2.0 * y)          # alpha == 0: A, x not read
    A = np.ones(12, np.float32)
    y_ref, d_ref = oracle.gemv("f32", Cm, N, 3, 4, 1.0, A, 3, np.ones(4, np.float32), 1, 0.0, np.full(3, np.nan, np.float32), 1)
    assert np.array_equal(y_ref, np.full(3, 4.0)) and np.array_equal(d_ref, np.full(3, 4.0))   # beta == 0: y not read
