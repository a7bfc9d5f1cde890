"""Seeded synthetic inputs shaped like the paper's GEMM workloads.

This module only draws random numbers and lays them out in BLAS storage (flat buffer +
leading dimension, row/column-major, optional transposition, optional padding).  It holds
none of the GEMM arithmetic and is the one module that both the GPU tests/benchmark and the
CPU oracle's tests may share.  numpy only; never touches the GPU library.

The five workload groups:
  1  one 256^3 FP32 problem, once with uniform[-1,1] entries and once with small integers
     (every partial sum exactly representable -> bit-exact comparison)
  2  square FP32 problems in all 8 storage variants (row/col-major x op(A) x op(B)),
     like the power-of-two SGEMM curves of the paper's cross-device figure
  3  FP16 problems: im2col-shaped convolution GEMMs and one large square (the paper's
     half-precision experiment and its convolution-as-GEMM motivation)
  4  batched small FP32 GEMMs packed in single buffers at per-instance offsets with
     per-instance alpha/beta (the paper's generic batched GEMM experiment)
  5  odd-sized and skinny FP32 problems with padded leading dimensions (the paper's
     "multiples of an odd number" curves, e.g. multiples of 129)
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

ROW_MAJOR, COL_MAJOR = 101, 102
NO_TRANS, TRANS = 111, 112

SEED_BASE = 170505249


def rng_for(config: int, case: int) -> np.random.Generator:
    return np.random.default_rng(SEED_BASE + 1000 * config + case)


# ----------------------------------------------------------------------------- layout helpers

def stored_extents(trans: int, rows: int, cols: int):
    """extents (r, c) of the matrix as stored, for a logical op(X) of rows x cols"""
    return (rows, cols) if trans == NO_TRANS else (cols, rows)


def tight_ld(layout: int, trans: int, rows: int, cols: int) -> int:
    r, c = stored_extents(trans, rows, cols)
    return max(1, r if layout == COL_MAJOR else c)


def storage_len(layout: int, trans: int, rows: int, cols: int, ld: int) -> int:
    r, c = stored_extents(trans, rows, cols)
    if r == 0 or c == 0:
        return 0
    return (c - 1) * ld + r if layout == COL_MAJOR else (r - 1) * ld + c


def pack(logical: np.ndarray, layout: int, trans: int, ld: Optional[int] = None,
         fill=np.nan, tail: int = 0) -> np.ndarray:
    """Flat storage of a logical op(X): element op(X)(i,l) goes where BLAS expects it.
    Positions not covered by the matrix (ld padding, `tail` extra elements) hold `fill`."""
    rows, cols = logical.shape
    stored = logical if trans == NO_TRANS else logical.T
    r, c = stored.shape
    if ld is None:
        ld = tight_ld(layout, trans, rows, cols)
    major, minor = (c, r) if layout == COL_MAJOR else (r, c)
    assert ld >= max(1, minor), "leading dimension too small"
    buf = np.full(major * ld + tail, fill, dtype=logical.dtype)
    view = buf[: major * ld].reshape(major, ld)[:, :minor]
    view[...] = stored.T if layout == COL_MAJOR else stored
    return buf


def unpack(buf: np.ndarray, layout: int, rows: int, cols: int, ld: int) -> np.ndarray:
    """(rows, cols) copy of a non-transposed matrix held in flat storage"""
    major, minor = (cols, rows) if layout == COL_MAJOR else (rows, cols)
    if major == 0 or minor == 0:
        return np.zeros((rows, cols), dtype=buf.dtype)
    need = (major - 1) * ld + minor
    flat = np.empty(major * ld, dtype=buf.dtype)
    flat[:need] = buf[:need]
    flat[need:] = 0
    view = flat.reshape(major, ld)[:, :minor]
    return np.ascontiguousarray(view.T if layout == COL_MAJOR else view)


def padding_mask(layout: int, rows: int, cols: int, ld: int, total: int) -> np.ndarray:
    """boolean mask over a flat buffer of length `total`: True where NO matrix element lives"""
    mask = np.ones(total, dtype=bool)
    major, minor = (cols, rows) if layout == COL_MAJOR else (rows, cols)
    if major and minor:
        idx = (np.arange(major, dtype=np.int64)[:, None] * ld + np.arange(minor, dtype=np.int64)[None, :])
        mask[idx.reshape(-1)] = False
    return mask


# ----------------------------------------------------------------------------- problem records

@dataclass
class GemmCase:
    name: str
    dtype: str            # 'f32' or 'f16' (storage type; accumulation is FP32 on the GPU)
    layout: int
    ta: int
    tb: int
    m: int
    n: int
    k: int
    alpha: float
    beta: float
    A: np.ndarray         # flat storage
    lda: int
    B: np.ndarray
    ldb: int
    C: np.ndarray
    ldc: int
    exact: bool = False   # integer-valued inputs: result must match bit for bit

    @property
    def flops(self) -> float:
        return 2.0 * self.m * self.n * self.k

    @property
    def algorithmic_bytes(self) -> float:
        e = 4 if self.dtype == "f32" else 2
        c_reads = 1 if self.beta != 0 else 0
        return e * (self.m * self.k + self.k * self.n + (1 + c_reads) * self.m * self.n)


@dataclass
class BatchedCase:
    name: str
    layout: int
    ta: int
    tb: int
    m: int
    n: int
    k: int
    alphas: np.ndarray
    betas: np.ndarray
    A: np.ndarray
    a_off: np.ndarray
    lda: int
    B: np.ndarray
    b_off: np.ndarray
    ldb: int
    C: np.ndarray
    c_off: np.ndarray
    ldc: int
    batch: int = field(default=0)
    dtype: str = "f32"

    @property
    def flops(self) -> float:
        return 2.0 * self.m * self.n * self.k * self.batch

    @property
    def algorithmic_bytes(self) -> float:
        # A, B, C_old read + C written, two FP32 scalars, three int64 offsets
        e = 4.0 if self.dtype == "f32" else 2.0
        return self.batch * (e * (self.m * self.k + self.k * self.n + 2 * self.m * self.n) + 8 + 24)


def _np_dtype(dtype: str):
    return np.float32 if dtype == "f32" else np.float16


def make_case(name, dtype, layout, ta, tb, opA, opB, Cmat, alpha, beta,
              lda=None, ldb=None, ldc=None, exact=False, fill=np.nan) -> GemmCase:
    """Pack logical op(A) (m x k), op(B) (k x n), C (m x n) into the requested storage."""
    m, k = opA.shape
    k2, n = opB.shape
    assert k == k2 and Cmat.shape == (m, n)
    t = _np_dtype(dtype)
    opA, opB, Cmat = opA.astype(t, copy=False), opB.astype(t, copy=False), Cmat.astype(t, copy=False)
    lda = lda or tight_ld(layout, ta, m, k)
    ldb = ldb or tight_ld(layout, tb, k, n)
    ldc = ldc or tight_ld(layout, NO_TRANS, m, n)
    return GemmCase(name, dtype, layout, ta, tb, m, n, k, float(alpha), float(beta),
                    pack(opA, layout, ta, lda, fill), lda,
                    pack(opB, layout, tb, ldb, fill), ldb,
                    pack(Cmat, layout, NO_TRANS, ldc, fill), ldc, exact)


def uniform(rng, shape, lo=-1.0, hi=1.0, dtype=np.float32):
    return rng.uniform(lo, hi, size=shape).astype(dtype)


def small_ints(rng, shape, lim=4, dtype=np.float32):
    return rng.integers(-lim, lim + 1, size=shape).astype(dtype)


# ----------------------------------------------------------------------------- group 1

def config1(integer: bool) -> GemmCase:
    """256^3 FP32, column-major, N/N, tight ld, alpha=1.5, beta=0.5"""
    g = rng_for(1, 1 if integer else 0)
    gen = small_ints if integer else uniform
    s = 256
    return make_case("c1_int" if integer else "c1_uniform", "f32", COL_MAJOR, NO_TRANS, NO_TRANS,
                     gen(g, (s, s)), gen(g, (s, s)), gen(g, (s, s)), 1.5, 0.5, exact=integer)


# ----------------------------------------------------------------------------- group 2

CONFIG2_SIZES = (1024, 2048, 4096, 8192)
CONFIG2_BETAS = (0.0, 0.7)


def config2_logical(size: int):
    """the logical op(A), op(B), C of one square size; every storage variant packs these"""
    g = rng_for(2, size)
    return uniform(g, (size, size)), uniform(g, (size, size)), uniform(g, (size, size))


def config2_variant(size, layout, ta, tb, beta, logical=None) -> GemmCase:
    opA, opB, Cm = logical if logical is not None else config2_logical(size)
    tag = f"c2_n{size}_{'R' if layout == ROW_MAJOR else 'C'}{'T' if ta == TRANS else 'N'}{'T' if tb == TRANS else 'N'}_b{beta}"
    return make_case(tag, "f32", layout, ta, tb, opA, opB, Cm, 1.0, beta)


def config2_like(size, layout, ta, tb, beta, seed_case=0, integer=False) -> GemmCase:
    """same structure as group 2 at an arbitrary (small) square size, for the oracle-sized tests"""
    g = rng_for(2, 100000 + seed_case)
    gen = small_ints if integer else uniform
    return make_case(f"c2like_n{size}", "f32", layout, ta, tb, gen(g, (size, size)), gen(g, (size, size)),
                     gen(g, (size, size)), 1.0, beta, exact=integer)


# ----------------------------------------------------------------------------- convolutions

@dataclass
class ConvCase:
    """one image, dense row-major arrays: im (C,H,W), weights (F,C,KH,KW), out (F,OH,OW) holding the old values"""
    name: str
    dtype: str
    channels: int
    height: int
    width: int
    kernel: tuple
    pad: tuple
    stride: tuple
    dilation: tuple
    filters: int
    alpha: float
    beta: float
    im: np.ndarray
    weights: np.ndarray
    out: np.ndarray
    exact: bool = False

    @property
    def out_hw(self):
        return tuple(conv_out_extent(s, k, p, st, d) for s, k, p, st, d in
                     zip((self.height, self.width), self.kernel, self.pad, self.stride, self.dilation))

    @property
    def k(self):
        return self.channels * self.kernel[0] * self.kernel[1]


def conv_out_extent(size, kernel, pad, stride, dilation) -> int:
    span = size + 2 * pad - dilation * (kernel - 1) - 1
    return 0 if span < 0 else span // stride + 1


# the layers whose im2col GEMMs are the FP16 shapes of group 3: (C, H, W, kernel, pad, stride, filters)
CONV_LAYERS = ((3, 224, 224, 7, 3, 2, 64), (64, 56, 56, 3, 1, 1, 128), (128, 28, 28, 3, 1, 1, 256),
               (256, 14, 14, 3, 1, 1, 512))


def conv_case(dtype, channels, height, width, kernel, pad, stride, dilation, filters, alpha=1.0, beta=0.0, case=0,
              integer=False, name=None) -> ConvCase:
    """entries N(0, K^-1/2) like group 3 (or small integers for bit-exact checks)"""
    g = rng_for(6, case)
    np_t = np.float32 if dtype == "f32" else np.float16
    oh = conv_out_extent(height, kernel[0], pad[0], stride[0], dilation[0])
    ow = conv_out_extent(width, kernel[1], pad[1], stride[1], dilation[1])
    shapes = ((channels, height, width), (filters, channels, kernel[0], kernel[1]), (filters, oh, ow))
    if integer:
        im, w, out = (small_ints(g, s, 2, np_t) for s in shapes)
    else:
        sigma = float(channels * kernel[0] * kernel[1]) ** -0.5
        im, w, out = (g.normal(0.0, sigma, size=s).astype(np.float32).astype(np_t) for s in shapes)
    return ConvCase(name or f"conv_{dtype}_{channels}x{height}x{width}_k{kernel[0]}x{kernel[1]}_f{filters}", dtype,
                    channels, height, width, tuple(kernel), tuple(pad), tuple(stride), tuple(dilation), filters, alpha,
                    beta, im, w, out, integer)


def conv_layer(index, dtype="f16", integer=False, beta=0.0) -> ConvCase:
    c, h, w, k, p, s, f = CONV_LAYERS[index]
    return conv_case(dtype, c, h, w, (k, k), (p, p), (s, s), (1, 1), f, 1.0, beta, case=index, integer=integer,
                     name=f"layer{index}_{dtype}")


# ----------------------------------------------------------------------------- group 3

CONFIG3_SHAPES = ((64, 12544, 147), (128, 3136, 576), (256, 784, 1152), (512, 196, 2304), (4096, 4096, 4096))


def config3(index: int, integer: bool = False) -> GemmCase:
    """FP16 storage, column-major N/N, alpha=1, beta=0, entries N(0, sigma=K^-1/2) rounded to FP16"""
    m, n, k = CONFIG3_SHAPES[index]
    return hgemm_case(m, n, k, case=index, integer=integer, name=f"c3_{m}x{n}x{k}")


def hgemm_case(m, n, k, case=0, layout=COL_MAJOR, ta=NO_TRANS, tb=NO_TRANS, alpha=1.0, beta=0.0,
               integer=False, name=None, lda=None, ldb=None, ldc=None) -> GemmCase:
    g = rng_for(3, case)
    if integer:
        # entries in [-2,2]: |sum| <= 4k, exact in FP32; exact in the FP16 output while <= 2048
        opA, opB, Cm = (small_ints(g, s, 2, np.float16) for s in ((m, k), (k, n), (m, n)))
    else:
        sigma = float(k) ** -0.5 if k else 1.0
        opA = g.normal(0.0, sigma, size=(m, k)).astype(np.float32).astype(np.float16)
        opB = g.normal(0.0, sigma, size=(k, n)).astype(np.float32).astype(np.float16)
        Cm = g.normal(0.0, sigma, size=(m, n)).astype(np.float32).astype(np.float16)
    return make_case(name or f"h_{m}x{n}x{k}", "f16", layout, ta, tb, opA, opB, Cm, alpha, beta,
                     lda, ldb, ldc, exact=integer)


# ----------------------------------------------------------------------------- group 4

CONFIG4_SIZES = (8, 16, 32, 64)
CONFIG4_BATCHES = (1000, 10000)
GAP = 7          # elements between consecutive instances in each buffer
GAP_FILL = np.float32(-12345.0)   # sentinel kept in the gaps of C (NaN would not compare equal)


def batched_case(s_m, s_n, s_k, batch, case=0, layout=COL_MAJOR, ta=NO_TRANS, tb=NO_TRANS,
                 integer=False, lda=None, ldb=None, ldc=None, gap=GAP, name=None,
                 shuffle_offsets=False, dtype="f32") -> BatchedCase:
    """`batch` independent GEMMs in single A/B/C buffers; instance i starts at i*(size+gap);
    alpha_i, beta_i ~ U[0.5, 2]; entries U[-1,1] (or small integers with alpha,beta in {0.5,1,1.5,2})"""
    g = rng_for(4, case)
    lda = lda or tight_ld(layout, ta, s_m, s_k)
    ldb = ldb or tight_ld(layout, tb, s_k, s_n)
    ldc = ldc or tight_ld(layout, NO_TRANS, s_m, s_n)
    la = storage_len(layout, ta, s_m, s_k, lda)
    lb = storage_len(layout, tb, s_k, s_n, ldb)
    lc = storage_len(layout, NO_TRANS, s_m, s_n, ldc)
    order = g.permutation(batch) if shuffle_offsets else np.arange(batch)
    a_off = (order * (la + gap)).astype(np.int64)
    b_off = (order * (lb + gap)).astype(np.int64)
    c_off = (order * (lc + gap)).astype(np.int64)
    np_t = _np_dtype(dtype)
    A = np.full(batch * (la + gap), np.nan, dtype=np_t)
    B = np.full(batch * (lb + gap), np.nan, dtype=np_t)
    C = np.full(batch * (lc + gap), GAP_FILL, dtype=np_t)
    if integer and dtype == "f16":
        # entries in [-2,2]: with alpha, beta <= 2 every result stays an exactly representable FP16 number
        gen = lambda rng, shape: small_ints(rng, shape, 2, np_t)
    else:
        gen = (lambda rng, shape: small_ints(rng, shape, 4, np_t)) if integer else \
              (lambda rng, shape: uniform(rng, shape, dtype=np.float32).astype(np_t))
    for i in range(batch):
        opA, opB, Cm = gen(g, (s_m, s_k)), gen(g, (s_k, s_n)), gen(g, (s_m, s_n))
        A[a_off[i]: a_off[i] + la] = pack(opA, layout, ta, lda)[:la]
        B[b_off[i]: b_off[i] + lb] = pack(opB, layout, tb, ldb)[:lb]
        C[c_off[i]: c_off[i] + lc] = pack(Cm, layout, NO_TRANS, ldc, fill=GAP_FILL)[:lc]
    if integer:
        alphas = g.choice(np.array([0.5, 1.0, 1.5, 2.0], dtype=np.float32), size=batch)
        betas = g.choice(np.array([0.5, 1.0, 1.5, 2.0], dtype=np.float32), size=batch)
    else:
        alphas = g.uniform(0.5, 2.0, size=batch).astype(np.float32)
        betas = g.uniform(0.5, 2.0, size=batch).astype(np.float32)
    return BatchedCase(name or f"c4_{dtype}_s{s_m}x{s_n}x{s_k}_b{batch}", layout, ta, tb, s_m, s_n, s_k,
                       alphas, betas, A, a_off, lda, B, b_off, ldb, C, c_off, ldc, batch, dtype)


def config4(size: int, batch: int) -> BatchedCase:
    return batched_case(size, size, size, batch, case=size * 100000 + batch, name=f"c4_s{size}_b{batch}")


def config4_fast(size: int, batch: int, dtype: str = "f32") -> BatchedCase:
    """same layout and distributions as config4, drawn with whole-array calls (for the
    benchmark, where 10000 per-instance draws would dominate set-up time)"""
    g = rng_for(4, size * 100000 + batch + 7)
    per = size * size
    stride = per + GAP
    off = (np.arange(batch, dtype=np.int64) * stride)
    bufs = []
    for fill in (np.nan, np.nan, GAP_FILL):
        buf = np.full((batch, stride), fill, dtype=_np_dtype(dtype))
        buf[:, :per] = g.uniform(-1.0, 1.0, size=(batch, per)).astype(np.float32).astype(_np_dtype(dtype))
        bufs.append(buf.reshape(-1))
    alphas = g.uniform(0.5, 2.0, size=batch).astype(np.float32)
    betas = g.uniform(0.5, 2.0, size=batch).astype(np.float32)
    return BatchedCase(f"c4_s{size}_b{batch}" + ("" if dtype == "f32" else "_f16"), COL_MAJOR, NO_TRANS, NO_TRANS, size,
                       size, size, alphas, betas, bufs[0], off.copy(), size, bufs[1], off.copy(), size,
                       bufs[2], off.copy(), size, batch, dtype)


# ----------------------------------------------------------------------------- group 5

CONFIG5_SHAPES = ((1000, 1001, 999), (4097, 129, 4095), (129, 4097, 4095),
                  (1, 4096, 4096), (4096, 1, 4096), (8192, 8192, 64))


def padded_ld(extent: int) -> int:
    """next multiple of 8, plus 1"""
    return 8 * ((extent + 7) // 8) + 1


def config5(index: int, integer: bool = False) -> GemmCase:
    """FP32 column-major, op(A)=A^T, op(B)=B, padded leading dimensions, alpha=beta=1"""
    m, n, k = CONFIG5_SHAPES[index]
    return skinny_case(m, n, k, case=index, integer=integer, name=f"c5_{m}x{n}x{k}")


def skinny_case(m, n, k, case=0, integer=False, name=None, layout=COL_MAJOR, ta=TRANS, tb=NO_TRANS,
                alpha=1.0, beta=1.0) -> GemmCase:
    g = rng_for(5, case)
    gen = small_ints if integer else uniform
    if integer and k > 1024:
        gen = lambda gg, s: small_ints(gg, s, 2)      # keep |sum| < 2^24
    opA, opB, Cm = gen(g, (m, k)), gen(g, (k, n)), gen(g, (m, n))
    ra = tight_ld(layout, ta, m, k)
    rb = tight_ld(layout, tb, k, n)
    rc = tight_ld(layout, NO_TRANS, m, n)
    return make_case(name or f"sk_{m}x{n}x{k}", "f32", layout, ta, tb, opA, opB, Cm, alpha, beta,
                     padded_ld(ra), padded_ld(rb), padded_ld(rc), exact=integer)


# ----------------------------------------------------------------------------- matrix-vector cases

@dataclass
class GemvCase:
    """One GEMV call: y = alpha op(A) x + beta y.  A is m x n as stored; x, y are flat buffers with increments
    (the slots between the elements hold a sentinel that must survive the call)."""
    name: str
    dtype: str
    layout: int
    trans: int
    m: int
    n: int
    alpha: float
    beta: float
    A: np.ndarray
    lda: int
    x: np.ndarray
    incx: int
    y: np.ndarray
    incy: int
    exact: bool = False

    @property
    def outputs(self) -> int:
        return self.m if self.trans == NO_TRANS else self.n

    @property
    def length(self) -> int:
        return self.n if self.trans == NO_TRANS else self.m


def gemv_case(dtype, layout, trans, m, n, incx=1, incy=1, alpha=1.0, beta=0.0, case=0, integer=False, pad=0,
              name=None) -> GemvCase:
    g = rng_for(6, case)
    np_t = _np_dtype(dtype)
    gen = small_ints if integer else uniform
    if integer and (max(m, n) > 1024 or dtype == "f16"):
        gen = lambda gg, s, dtype=np.float32: small_ints(gg, s, 2, dtype=dtype)   # results stay exactly representable
    Am = gen(g, (m, n), dtype=np_t)
    lda = tight_ld(layout, NO_TRANS, m, n) + pad
    A = pack(Am, layout, NO_TRANS, lda)
    rows, length = (m, n) if trans == NO_TRANS else (n, m)
    x = np.full(max((length - 1) * incx + 1, 1), GAP_FILL, dtype=np_t)
    y = np.full(max((rows - 1) * incy + 1, 1), GAP_FILL, dtype=np_t)
    if length:
        x[::incx] = gen(g, (length,), dtype=np_t)
    if rows:
        y[::incy] = gen(g, (rows,), dtype=np_t)
    return GemvCase(name or f"gemv_{dtype}_{m}x{n}", dtype, layout, trans, m, n, alpha, beta, A, lda, x, incx, y,
                    incy, exact=integer)


# ----------------------------------------------------------------------------- level-3 derivative cases

UPPER, LOWER = 121, 122
NON_UNIT, UNIT = 131, 132
LEFT, RIGHT = 141, 142


@dataclass
class Level3Case:
    """One SYMM ('symm'), SYRK ('syrk') or TRMM ('trmm') call in BLAS storage.  Whatever the routine must not
    read holds NaN: the unreferenced triangle of a symmetric or triangular A, the diagonal of a unit-triangular
    A, and (SYRK) the triangle of C that is not updated.  Padding holds NaN (inputs) or a sentinel (output)."""
    name: str
    routine: str
    dtype: str
    layout: int
    side: int
    uplo: int
    trans: int
    diag: int
    m: int
    n: int
    k: int
    alpha: float
    beta: float
    A: np.ndarray
    lda: int
    B: Optional[np.ndarray]
    ldb: int
    C: Optional[np.ndarray]
    ldc: int
    exact: bool = False


def _blank_triangle(mat, uplo, unit=False):
    out = mat.copy()
    i, j = np.indices(mat.shape)
    out[(i > j) if uplo == UPPER else (i < j)] = np.nan
    if unit:
        out[i == j] = np.nan
    return out


def level3_case(routine, dtype, layout, m, n, k=0, side=LEFT, uplo=UPPER, trans=NO_TRANS, diag=NON_UNIT, alpha=1.0,
                beta=0.0, pad=(0, 0, 0), case=0, integer=False) -> Level3Case:
    g = rng_for(7, case)
    np_t = _np_dtype(dtype)
    lim = 1 if dtype == "f16" or max(m, n, k) > 512 else 2          # integer results stay exactly representable
    gen = (lambda shape: small_ints(g, shape, lim, dtype=np_t)) if integer else (lambda shape: uniform(g, shape, dtype=np_t))

    def store(mat, extra, fill):
        ld = tight_ld(layout, NO_TRANS, *mat.shape) + extra
        return pack(mat, layout, NO_TRANS, ld, fill=fill), ld

    B = C = None
    ldb = ldc = 1
    if routine == "symm":
        ka = m if side == LEFT else n
        A, lda = store(_blank_triangle(gen((ka, ka)), uplo), pad[0], np.nan)
        B, ldb = store(gen((m, n)), pad[1], np.nan)
        C, ldc = store(gen((m, n)), pad[2], GAP_FILL)
    elif routine == "syrk":
        A, lda = store(gen((n, k) if trans == NO_TRANS else (k, n)), pad[0], np.nan)
        C, ldc = store(_blank_triangle(gen((n, n)), uplo), pad[2], GAP_FILL)
        m = n
    elif routine == "trmm":
        ka = m if side == LEFT else n
        A, lda = store(_blank_triangle(gen((ka, ka)), uplo, unit=diag == UNIT), pad[0], np.nan)
        B, ldb = store(gen((m, n)), pad[1], GAP_FILL)
    else:
        raise ValueError(routine)
    name = f"{routine}_{dtype}_{m}x{n}" + (f"x{k}" if routine == "syrk" else "")
    return Level3Case(name, routine, dtype, layout, side, uplo, trans, diag, m, n, k, alpha, beta, A, lda, B, ldb, C, ldc,
                      exact=integer)


# ----------------------------------------------------------------------------- sampling plan

def sample_entries(m: int, n: int, seed: int, rows: int = 16, cols: int = 16, tile: int = 128,
                   scattered: int = 4096):
    """Output positions for the sampled oracle on large problems: a few complete rows and
    columns (first, last, next to tile boundaries, random) plus scattered single entries."""
    g = np.random.default_rng(seed)
    def pick(extent, count):
        fixed = {0, extent - 1}
        # both sides of tile boundaries spread over the whole extent (the first, the last, evenly between), not
        # only the first few: a mistake in the mapping of late tiles (rasterisation, XCD walk) must be seen too
        bounds = np.arange(tile, extent, tile)
        if bounds.size:
            want = max(1, (count // 2 - 2) // 2)
            chosen = bounds[np.unique(np.linspace(0, bounds.size - 1, min(want, bounds.size)).round().astype(int))]
            for b in chosen:
                fixed.update((int(b) - 1, int(b)))
        rest = g.integers(0, extent, size=max(0, count - len(fixed)))
        return np.unique(np.concatenate([np.fromiter(fixed, dtype=np.int64), rest.astype(np.int64)]))
    ri, cj = pick(m, min(rows, m)), pick(n, min(cols, n))
    r1 = np.repeat(ri, n); c1 = np.tile(np.arange(n, dtype=np.int64), ri.size)
    c2 = np.repeat(cj, m); r2 = np.tile(np.arange(m, dtype=np.int64), cj.size)
    r3 = g.integers(0, m, size=scattered).astype(np.int64)
    c3 = g.integers(0, n, size=scattered).astype(np.int64)
    return np.concatenate([r1, r2, r3]), np.concatenate([c1, c2, c3])
