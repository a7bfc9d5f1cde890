"""ctypes front-end of the C oracle in conv_oracle.c  --  TEST INFRASTRUCTURE ONLY.

Takes numpy host arrays in dense row-major "CHW" / "FCHW" order and returns FP64 arrays: the
column matrix of IM2COL, or the convolution result and its error denominator
D = |alpha| sum |w||x| + |beta||out_old|.  Definition followed: the IM2COL routine and the
convolution-as-GEMM remark of the paper (Section 3.1 routine table, Section 1), read as the usual
neural-network cross-correlation with zero padding, stride and dilation.  No arithmetic happens
in this file.
"""
import ctypes

import numpy as np

from . import gemm_oracle as _g

_ready = False


def _lib():
    global _ready
    L = _g.lib()
    if not _ready:
        i64, dbl, vp, ci = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_int
        L.oracle_conv_out_extent.argtypes = [i64] * 5
        L.oracle_conv_out_extent.restype = i64
        L.oracle_im2col.argtypes = [ci] + [i64] * 11 + [vp, vp]
        L.oracle_im2col.restype = None
        L.oracle_conv2d.argtypes = [ci] + [i64] * 12 + [dbl, vp, vp, dbl, vp, vp, vp]
        L.oracle_conv2d.restype = None
        _ready = True
    return L


def _flat(a, dtype, count, what):
    a = np.ascontiguousarray(a).reshape(-1)
    want = np.float32 if dtype == "f32" else np.uint16
    if a.dtype == np.float16 and dtype == "f16":
        a = a.view(np.uint16)
    if a.dtype != want:
        raise TypeError(f"{what}: expected {want}, got {a.dtype}")
    if a.size < count:
        raise ValueError(f"{what}: {a.size} elements, need {count}")
    return a


def out_extent(size, kernel, pad, stride, dilation) -> int:
    return int(_lib().oracle_conv_out_extent(size, kernel, pad, stride, dilation))


def im2col(dtype, channels, height, width, kernel, pad, stride, dilation, im):
    """(K, OH*OW) float64; kernel, pad, stride, dilation are (h, w) pairs"""
    oh, ow = out_extent(height, kernel[0], pad[0], stride[0], dilation[0]), out_extent(width, kernel[1], pad[1], stride[1], dilation[1])
    im = _flat(im, dtype, channels * height * width, "im")
    col = np.empty((channels * kernel[0] * kernel[1], oh * ow), np.float64)
    _lib().oracle_im2col(int(dtype == "f16"), channels, height, width, kernel[0], kernel[1], pad[0], pad[1], stride[0],
                         stride[1], dilation[0], dilation[1], ctypes.c_void_p(im.ctypes.data),
                         ctypes.c_void_p(col.ctypes.data))
    return col


def conv2d(dtype, channels, height, width, kernel, pad, stride, dilation, filters, alpha, im, weights, beta, out_old):
    """(ref, den), each (filters, OH, OW) float64"""
    oh, ow = out_extent(height, kernel[0], pad[0], stride[0], dilation[0]), out_extent(width, kernel[1], pad[1], stride[1], dilation[1])
    im = _flat(im, dtype, 0 if alpha == 0 else channels * height * width, "im")
    weights = _flat(weights, dtype, 0 if alpha == 0 else filters * channels * kernel[0] * kernel[1], "weights")
    out_old = _flat(out_old, dtype, 0 if beta == 0 else filters * oh * ow, "out")
    ref = np.empty((filters, oh, ow), np.float64)
    den = np.empty((filters, oh, ow), np.float64)
    _lib().oracle_conv2d(int(dtype == "f16"), channels, height, width, kernel[0], kernel[1], pad[0], pad[1], stride[0],
                         stride[1], dilation[0], dilation[1], filters, float(alpha), ctypes.c_void_p(im.ctypes.data),
                         ctypes.c_void_p(weights.ctypes.data), float(beta), ctypes.c_void_p(out_old.ctypes.data),
                         ctypes.c_void_p(ref.ctypes.data), ctypes.c_void_p(den.ctypes.data))
    return ref, den
