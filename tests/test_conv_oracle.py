"""Pins of the IM2COL / convolution oracle against things other than itself: a hand-computed example,
closed forms, invariants, a library routine on the special case it covers, and the GEMM oracle."""
import os

import numpy as np
import pytest
from scipy import signal

from oracle import conv_oracle as CO
from oracle import gemm_oracle as GO

HERE = os.path.dirname(os.path.abspath(__file__))


def rnd(shape, seed):
    return np.random.default_rng(seed).uniform(-1, 1, size=shape).astype(np.float32)


def test_out_extent_closed_forms():
    assert CO.out_extent(224, 7, 3, 2, 1) == 112       # first layer of the usual ImageNet residual network
    assert CO.out_extent(56, 3, 1, 1, 1) == 56         # "same" 3x3
    assert CO.out_extent(5, 3, 0, 1, 1) == 3
    assert CO.out_extent(5, 3, 0, 2, 1) == 2
    assert CO.out_extent(7, 3, 0, 1, 2) == 3           # dilated 3-tap spans 5
    assert CO.out_extent(2, 5, 0, 1, 1) == 0           # kernel larger than the image


def read_golden():
    """hand-computed example: see tests/golden/conv_handsized.txt"""
    blocks, cur = {}, None
    for line in open(os.path.join(HERE, "golden", "conv_handsized.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        if line.endswith(":"):
            cur = line[:-1]
            blocks[cur] = []
        else:
            blocks[cur].extend(float(x) for x in line.split())
    return blocks


def test_hand_computed_example():
    g = read_golden()
    im = np.array(g["im"], np.float32)               # 2 channels x 3 x 4
    w = np.array(g["weights"], np.float32)            # 2 filters x 2 channels x 2 x 2
    old = np.array(g["out_old"], np.float32)
    col = CO.im2col("f32", 2, 3, 4, (2, 2), (0, 1), (1, 2), (1, 1), im)
    assert col.shape == (8, 6)
    assert np.array_equal(col.reshape(-1), np.array(g["col"]))
    ref, den = CO.conv2d("f32", 2, 3, 4, (2, 2), (0, 1), (1, 2), (1, 1), 2, 2.0, im, w, -1.0, old)
    assert np.array_equal(ref.reshape(-1), np.array(g["out"]))
    assert np.array_equal(den.reshape(-1), np.array(g["den"]))


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_delta_filter_shifts_the_image(dtype):
    """a filter that is 1 at tap (kh, kw) of channel c and 0 elsewhere copies that channel, shifted, zero-filled"""
    C, H, W = 3, 6, 7
    im = rnd((C, H, W), 1)
    if dtype == "f16":
        im = im.astype(np.float16)
    for (c, kh, kw) in ((0, 0, 0), (1, 1, 2), (2, 2, 1)):
        w = np.zeros((1, C, 3, 3), im.dtype)
        w[0, c, kh, kw] = 1
        ref, den = CO.conv2d(dtype, C, H, W, (3, 3), (1, 1), (1, 1), (1, 1), 1, 1.0, im, w, 0.0, np.zeros(0, im.dtype))
        want = np.zeros((H, W))
        for oh in range(H):
            for ow in range(W):
                ih, iw = oh - 1 + kh, ow - 1 + kw
                if 0 <= ih < H and 0 <= iw < W:
                    want[oh, ow] = float(im[c, ih, iw])
        assert np.array_equal(ref[0], want)
        assert np.array_equal(den[0], np.abs(want))


def test_all_ones_filter_gives_box_sums():
    """integer image, all-ones 3x3 filter over 2 channels, no padding: sums over 3x3 windows via prefix sums"""
    C, H, W = 2, 8, 9
    im = np.random.default_rng(2).integers(-4, 5, size=(C, H, W)).astype(np.float32)
    w = np.ones((1, C, 3, 3), np.float32)
    ref, _ = CO.conv2d("f32", C, H, W, (3, 3), (0, 0), (1, 1), (1, 1), 1, 1.0, im, w, 0.0, np.zeros(0, np.float32))
    s = np.zeros((H + 1, W + 1))
    s[1:, 1:] = im.astype(np.float64).sum(axis=0).cumsum(axis=0).cumsum(axis=1)
    want = s[3:, 3:] - s[:-3, 3:] - s[3:, :-3] + s[:-3, :-3]
    assert np.array_equal(ref[0], want)


def test_library_special_case_single_channel():
    """one channel, one filter, stride 1, no dilation: scipy's 2-D cross-correlation ('valid' and zero-padded)"""
    H, W = 11, 13
    im, w = rnd((1, H, W), 3), rnd((1, 1, 4, 3), 4)
    ref, _ = CO.conv2d("f32", 1, H, W, (4, 3), (0, 0), (1, 1), (1, 1), 1, 1.0, im, w, 0.0, np.zeros(0, np.float32))
    want = signal.correlate2d(im[0].astype(np.float64), w[0, 0].astype(np.float64), mode="valid")
    assert ref.shape[1:] == want.shape and np.max(np.abs(ref[0] - want)) < 1e-14
    ref, _ = CO.conv2d("f32", 1, H, W, (4, 3), (2, 1), (1, 1), (1, 1), 1, 1.0, im, w, 0.0, np.zeros(0, np.float32))
    padded = np.zeros((H + 4, W + 2))
    padded[2:-2, 1:-1] = im[0]
    want = signal.correlate2d(padded, w[0, 0].astype(np.float64), mode="valid")
    assert ref.shape[1:] == want.shape and np.max(np.abs(ref[0] - want)) < 1e-14


def test_stride_subsamples_and_dilation_spreads_taps():
    C, H, W, F = 2, 10, 12, 3
    im, w = rnd((C, H, W), 5), rnd((F, C, 3, 3), 6)
    none = np.zeros(0, np.float32)
    full, _ = CO.conv2d("f32", C, H, W, (3, 3), (1, 1), (1, 1), (1, 1), F, 1.0, im, w, 0.0, none)
    strided, _ = CO.conv2d("f32", C, H, W, (3, 3), (1, 1), (2, 3), (1, 1), F, 1.0, im, w, 0.0, none)
    assert np.array_equal(strided, full[:, ::2, ::3])
    # dilation 2 == a 5x5 filter with the taps spread and zeros between
    spread = np.zeros((F, C, 5, 5), np.float32)
    spread[:, :, ::2, ::2] = w
    dil, _ = CO.conv2d("f32", C, H, W, (3, 3), (2, 2), (1, 1), (2, 2), F, 1.0, im, w, 0.0, none)
    ref5, _ = CO.conv2d("f32", C, H, W, (5, 5), (2, 2), (1, 1), (1, 1), F, 1.0, im, spread, 0.0, none)
    assert np.array_equal(dil, ref5)


def test_alpha_beta_conventions_and_linearity():
    C, H, W, F = 2, 5, 6, 2
    im, w, old = rnd((C, H, W), 7), rnd((F, C, 3, 3), 8), rnd((F, H, W), 9)
    args = ("f32", C, H, W, (3, 3), (1, 1), (1, 1), (1, 1), F)
    base, dbase = CO.conv2d(*args, 1.0, im, w, 0.0, np.full_like(old, np.nan))     # beta == 0: out is not read
    assert np.all(np.isfinite(base))
    poisoned = np.full_like(im, np.nan)
    ref, den = CO.conv2d(*args, 0.0, poisoned, np.full_like(w, np.nan), 0.5, old)  # alpha == 0: inputs are not read
    assert np.array_equal(ref, 0.5 * old.astype(np.float64)) and np.array_equal(den, 0.5 * np.abs(old.astype(np.float64)))
    ref, den = CO.conv2d(*args, -1.5, im, w, 0.25, old)
    assert np.allclose(ref, -1.5 * base + 0.25 * old, rtol=0, atol=1e-15)
    assert np.allclose(den, 1.5 * dbase + 0.25 * np.abs(old), rtol=0, atol=1e-15)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_im2col_times_weights_is_the_convolution(dtype):
    """out = w (F x K) * col (K x OH*OW), row-major: the GEMM oracle on the IM2COL oracle's matrix gives the
    direct convolution bit for bit (same summation order over (c, kh, kw))"""
    C, H, W, F = 3, 9, 8, 4
    kernel, pad, stride, dil = (3, 2), (1, 0), (2, 1), (1, 2)
    im, w = rnd((C, H, W), 10), rnd((F, C, *kernel), 11)
    if dtype == "f16":
        im, w = im.astype(np.float16), w.astype(np.float16)
    col = CO.im2col(dtype, C, H, W, kernel, pad, stride, dil, im)
    K, N = col.shape
    ref, den = CO.conv2d(dtype, C, H, W, kernel, pad, stride, dil, F, 1.0, im, w, 0.0, np.zeros(0, im.dtype))
    colT = col.astype(im.dtype)            # exact: every entry is an input value or zero
    wmat = w.reshape(F, K)
    c_ref, d_ref = GO.gemm(dtype, GO.ROW_MAJOR, GO.NO_TRANS, GO.NO_TRANS, F, N, K, 1.0, wmat, K, colT, N, 0.0,
                           np.zeros(F * N, wmat.dtype), N)
    assert np.array_equal(c_ref, ref.reshape(F, N)) and np.array_equal(d_ref, den.reshape(F, N))


def test_im2col_is_a_gather_of_the_padded_image():
    """every column-matrix entry equals the zero-padded image at the index the definition names (numpy
    fancy indexing as an independent way to write the same gather)"""
    C, H, W = 2, 7, 5
    kernel, pad, stride, dil = (3, 3), (2, 1), (2, 1), (1, 2)
    im = rnd((C, H, W), 12)
    col = CO.im2col("f32", C, H, W, kernel, pad, stride, dil, im)
    big = np.zeros((C, H + 2 * pad[0], W + 2 * pad[1]))
    big[:, pad[0]:pad[0] + H, pad[1]:pad[1] + W] = im
    OH, OW = CO.out_extent(H, 3, 2, 2, 1), CO.out_extent(W, 3, 1, 1, 2)
    assert col.shape == (C * 9, OH * OW)
    c, kh, kw = np.unravel_index(np.arange(C * 9), (C, 3, 3))
    oh, ow = np.unravel_index(np.arange(OH * OW), (OH, OW))
    want = big[c[:, None], (oh * 2)[None, :] + kh[:, None] * 1, (ow * 1)[None, :] + kw[:, None] * 2]
    assert np.array_equal(col, want)
