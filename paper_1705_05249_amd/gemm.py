"""Thin ctypes binding of libmg_gemm.so: same names and argument order as include/mg_gemm.h.

Argument marshalling only -- every step of the computation runs in the HIP kernels.  Matrix
arguments may be torch tensors on the GPU (their data_ptr() is passed) or raw integer device
addresses.  The stream defaults to torch's current HIP stream.  If the shared library has not
been built the import of this module's functions raises: there is no CPU fallback.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmg_gemm.so")

MG_ROW_MAJOR, MG_COL_MAJOR = 101, 102
MG_NO_TRANS, MG_TRANS, MG_CONJ_TRANS = 111, 112, 113
MG_F32, MG_F16 = 0, 1
MG_UPPER, MG_LOWER = 121, 122
MG_NON_UNIT, MG_UNIT = 131, 132
MG_LEFT, MG_RIGHT = 141, 142
MG_OK = 0
MG_FAMILY_DIRECT, MG_FAMILY_MFMA, MG_FAMILY_GEMV, MG_FAMILY_SCALE, MG_FAMILY_BATCHED, MG_FAMILY_CONV = 0, 1, 2, 3, 4, 5

EXPORTS = ("mg_sgemm", "mg_hgemm", "mg_sgemm_static", "mg_sgemv", "mg_hgemv", "mg_gemv_workspace_bytes",
           "mg_ssymm", "mg_hsymm", "mg_ssyrk", "mg_hsyrk", "mg_strmm", "mg_htrmm", "mg_symm_workspace_bytes",
           "mg_syrk_workspace_bytes", "mg_trmm_workspace_bytes", "mg_sgemm_batched", "mg_sgemm_strided_batched", "mg_hgemm_batched",
           "mg_hgemm_strided_batched", "mg_gemm_workspace_bytes",
           "mg_sim2col", "mg_him2col", "mg_sconv2d", "mg_hconv2d", "mg_conv2d_workspace_bytes", "mg_conv2d_out_extent",
           "mg_kernel_count",
           "mg_kernel_info", "mg_kernel_name", "mg_query_selected", "mg_override_config",
           "mg_override_batched_config", "mg_override_fringe", "mg_clear_override", "mg_lds_store_offset", "mg_lds_read_offset", "mg_lds_f32_store_offset", "mg_lds_f32_read_offset",
           "mg_probe_empty_launch", "mg_probe_mfma_only", "mg_probe_hgemm_stamps",
           "mg_status_string", "mg_version")


class mg_config(ctypes.Structure):
    _fields_ = [(name, ctypes.c_int32) for name in
                ("kernel_id", "family", "dtype", "tile_m", "tile_n", "tile_k", "waves_m", "waves_n",
                 "split_k", "threads", "lds_bytes", "fringe")]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


class MgError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def lib():
    """The loaded shared library (loads it on first use; raises if it was never built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first "
                               "(python -c 'import __graft_entry__ as g; g.build()')")
        # PyTorch ships its own copy of the HIP runtime.  A process must talk to one runtime only (kernels are
        # registered with the runtime the library was loaded against, streams and pointers come from torch's),
        # so torch's copy is loaded first and the library binds to it.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        i32, i64, f32, vp, sz = ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
        gemm_args = [i32, i32, i32, i64, i64, i64, f32, vp, i64, vp, i64, f32, vp, i64, vp, sz, vp]
        L.mg_sgemm.argtypes = gemm_args
        L.mg_sgemm.restype = i32
        L.mg_hgemm.argtypes = gemm_args
        L.mg_hgemm.restype = i32
        L.mg_sgemm_static.argtypes = gemm_args[:14] + [vp]
        L.mg_sgemm_static.restype = i32
        gemv_args = [i32, i32, i64, i64, f32, vp, i64, vp, i64, f32, vp, i64, vp, sz, vp]
        L.mg_sgemv.argtypes = gemv_args
        L.mg_sgemv.restype = i32
        L.mg_hgemv.argtypes = gemv_args
        L.mg_hgemv.restype = i32
        L.mg_gemv_workspace_bytes.argtypes = [i32, i32, i32, i64, i64, i64]
        L.mg_gemv_workspace_bytes.restype = sz
        symm_args = [i32, i32, i32, i64, i64, f32, vp, i64, vp, i64, f32, vp, i64, vp, sz, vp]
        syrk_args = [i32, i32, i32, i64, i64, f32, vp, i64, f32, vp, i64, vp, sz, vp]
        trmm_args = [i32, i32, i32, i32, i32, i64, i64, f32, vp, i64, vp, i64, vp, sz, vp]
        for name, args in (("mg_ssymm", symm_args), ("mg_hsymm", symm_args), ("mg_ssyrk", syrk_args),
                           ("mg_hsyrk", syrk_args), ("mg_strmm", trmm_args), ("mg_htrmm", trmm_args)):
            getattr(L, name).argtypes = args
            getattr(L, name).restype = i32
        L.mg_symm_workspace_bytes.argtypes = [i32, i32, i32, i64, i64]
        L.mg_symm_workspace_bytes.restype = sz
        L.mg_syrk_workspace_bytes.argtypes = [i32, i32, i32, i64, i64]
        L.mg_syrk_workspace_bytes.restype = sz
        L.mg_trmm_workspace_bytes.argtypes = [i32, i32, i32, i32, i64, i64]
        L.mg_trmm_workspace_bytes.restype = sz
        L.mg_sgemm_batched.argtypes = [i32, i32, i32, i64, i64, i64, vp, vp, vp, i64, vp, vp, i64, vp, vp, vp, i64,
                                       i64, vp]
        L.mg_sgemm_batched.restype = i32
        L.mg_sgemm_strided_batched.argtypes = [i32, i32, i32, i64, i64, i64, f32, vp, i64, i64, vp, i64, i64, f32, vp,
                                               i64, i64, i64, vp]
        L.mg_sgemm_strided_batched.restype = i32
        L.mg_hgemm_batched.argtypes = L.mg_sgemm_batched.argtypes
        L.mg_hgemm_batched.restype = i32
        L.mg_hgemm_strided_batched.argtypes = L.mg_sgemm_strided_batched.argtypes
        L.mg_hgemm_strided_batched.restype = i32
        L.mg_gemm_workspace_bytes.argtypes = [i32, i32, i32, i32, i64, i64, i64, i64, i64, i64]
        L.mg_gemm_workspace_bytes.restype = sz
        geometry = [i64] * 11
        L.mg_sim2col.argtypes = geometry + [vp, vp, vp]
        L.mg_sim2col.restype = i32
        L.mg_him2col.argtypes = geometry + [vp, vp, vp]
        L.mg_him2col.restype = i32
        conv_args = geometry + [i64, f32, vp, vp, f32, vp, vp, sz, vp]
        L.mg_sconv2d.argtypes = conv_args
        L.mg_sconv2d.restype = i32
        L.mg_hconv2d.argtypes = conv_args
        L.mg_hconv2d.restype = i32
        L.mg_conv2d_workspace_bytes.argtypes = [i32] + geometry + [i64]
        L.mg_conv2d_workspace_bytes.restype = sz
        L.mg_conv2d_out_extent.argtypes = [i64] * 5
        L.mg_conv2d_out_extent.restype = i64
        L.mg_kernel_count.argtypes = []
        L.mg_kernel_count.restype = ctypes.c_int32
        L.mg_kernel_info.argtypes = [ctypes.c_int32, ctypes.POINTER(mg_config)]
        L.mg_kernel_info.restype = i32
        L.mg_kernel_name.argtypes = [ctypes.c_int32]
        L.mg_kernel_name.restype = ctypes.c_char_p
        L.mg_query_selected.argtypes = [i32, i32, i32, i32, i64, i64, i64, i64, i64, i64, f32, f32, i64,
                                        ctypes.POINTER(mg_config)]
        L.mg_query_selected.restype = i32
        L.mg_override_config.argtypes = [ctypes.c_int32, ctypes.c_int32]
        L.mg_override_config.restype = i32
        L.mg_override_batched_config.argtypes = [ctypes.c_int32]
        L.mg_override_batched_config.restype = i32
        L.mg_override_fringe.argtypes = [ctypes.c_int32]
        L.mg_override_fringe.restype = i32
        L.mg_clear_override.argtypes = []
        L.mg_clear_override.restype = None
        L.mg_lds_store_offset.argtypes = [ctypes.c_int32] * 5
        L.mg_lds_store_offset.restype = ctypes.c_int32
        L.mg_lds_read_offset.argtypes = [ctypes.c_int32] * 8
        L.mg_lds_read_offset.restype = ctypes.c_int32
        L.mg_lds_f32_store_offset.argtypes = [ctypes.c_int32] * 4
        L.mg_lds_f32_store_offset.restype = ctypes.c_int32
        L.mg_lds_f32_read_offset.argtypes = [ctypes.c_int32] * 7
        L.mg_lds_f32_read_offset.restype = ctypes.c_int32
        L.mg_probe_empty_launch.argtypes = [vp]
        L.mg_probe_empty_launch.restype = i32
        L.mg_probe_mfma_only.argtypes = [ctypes.c_int32, vp, vp]
        L.mg_probe_mfma_only.restype = i32
        L.mg_probe_hgemm_stamps.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, vp]
        L.mg_probe_hgemm_stamps.restype = i32
        L.mg_status_string.argtypes = [i32]
        L.mg_status_string.restype = ctypes.c_char_p
        L.mg_version.argtypes = []
        L.mg_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _addr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()          # torch tensor


def _stream(stream):
    if stream is not None:
        return _addr(stream) if not hasattr(stream, "cuda_stream") else stream.cuda_stream
    import torch
    return torch.cuda.current_stream().cuda_stream


def _ws(workspace):
    if workspace is None:
        return None, 0
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def status_string(status: int) -> str:
    return lib().mg_status_string(status).decode()


def mg_sgemm(layout, trans_a, trans_b, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, workspace=None, stream=None,
             check=True) -> int:
    ws, ws_bytes = _ws(workspace)
    st = lib().mg_sgemm(layout, trans_a, trans_b, m, n, k, alpha, _addr(A), lda, _addr(B), ldb, beta, _addr(C),
                        ldc, ws, ws_bytes, _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, "mg_sgemm")
    return st


MG_STATIC_SCRATCH_BYTES = 16 << 20
MG_FRINGE_AUTO, MG_FRINGE_OFF, MG_FRINGE_ON = 0, 1, 2


def mg_sgemm_static(layout, trans_a, trans_b, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream=None, check=True) -> int:
    st = lib().mg_sgemm_static(layout, trans_a, trans_b, m, n, k, alpha, _addr(A), lda, _addr(B), ldb, beta, _addr(C),
                               ldc, _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, "mg_sgemm_static")
    return st


def mg_hgemm(layout, trans_a, trans_b, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, workspace=None, stream=None,
             check=True) -> int:
    ws, ws_bytes = _ws(workspace)
    st = lib().mg_hgemm(layout, trans_a, trans_b, m, n, k, alpha, _addr(A), lda, _addr(B), ldb, beta, _addr(C),
                        ldc, ws, ws_bytes, _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, "mg_hgemm")
    return st


def mg_sgemv(layout, trans_a, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None,
             check=True) -> int:
    ws, ws_bytes = _ws(workspace)
    st = lib().mg_sgemv(layout, trans_a, m, n, alpha, _addr(A), lda, _addr(x), incx, beta, _addr(y), incy, ws, ws_bytes,
                        _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, "mg_sgemv")
    return st


def mg_hgemv(layout, trans_a, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace=None, stream=None,
             check=True) -> int:
    ws, ws_bytes = _ws(workspace)
    st = lib().mg_hgemv(layout, trans_a, m, n, alpha, _addr(A), lda, _addr(x), incx, beta, _addr(y), incy, ws, ws_bytes,
                        _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, "mg_hgemv")
    return st


def _symm(name, layout, side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc, workspace, stream, check):
    ws, ws_bytes = _ws(workspace)
    st = getattr(lib(), name)(layout, side, uplo, m, n, alpha, _addr(A), lda, _addr(B), ldb, beta, _addr(C), ldc, ws,
                              ws_bytes, _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, name)
    return st


def mg_ssymm(layout, side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc, workspace=None, stream=None, check=True) -> int:
    return _symm("mg_ssymm", layout, side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc, workspace, stream, check)


def mg_hsymm(layout, side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc, workspace=None, stream=None, check=True) -> int:
    return _symm("mg_hsymm", layout, side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc, workspace, stream, check)


def _syrk(name, layout, uplo, trans, n, k, alpha, A, lda, beta, C, ldc, workspace, stream, check):
    ws, ws_bytes = _ws(workspace)
    st = getattr(lib(), name)(layout, uplo, trans, n, k, alpha, _addr(A), lda, beta, _addr(C), ldc, ws, ws_bytes,
                              _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, name)
    return st


def mg_ssyrk(layout, uplo, trans, n, k, alpha, A, lda, beta, C, ldc, workspace=None, stream=None, check=True) -> int:
    return _syrk("mg_ssyrk", layout, uplo, trans, n, k, alpha, A, lda, beta, C, ldc, workspace, stream, check)


def mg_hsyrk(layout, uplo, trans, n, k, alpha, A, lda, beta, C, ldc, workspace=None, stream=None, check=True) -> int:
    return _syrk("mg_hsyrk", layout, uplo, trans, n, k, alpha, A, lda, beta, C, ldc, workspace, stream, check)


def _trmm(name, layout, side, uplo, trans_a, diag, m, n, alpha, A, lda, B, ldb, workspace, stream, check):
    ws, ws_bytes = _ws(workspace)
    st = getattr(lib(), name)(layout, side, uplo, trans_a, diag, m, n, alpha, _addr(A), lda, _addr(B), ldb, ws, ws_bytes,
                              _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, name)
    return st


def mg_strmm(layout, side, uplo, trans_a, diag, m, n, alpha, A, lda, B, ldb, workspace=None, stream=None, check=True) -> int:
    return _trmm("mg_strmm", layout, side, uplo, trans_a, diag, m, n, alpha, A, lda, B, ldb, workspace, stream, check)


def mg_htrmm(layout, side, uplo, trans_a, diag, m, n, alpha, A, lda, B, ldb, workspace=None, stream=None, check=True) -> int:
    return _trmm("mg_htrmm", layout, side, uplo, trans_a, diag, m, n, alpha, A, lda, B, ldb, workspace, stream, check)


def mg_symm_workspace_bytes(dtype, layout, side, m, n) -> int:
    return lib().mg_symm_workspace_bytes(dtype, layout, side, m, n)


def mg_syrk_workspace_bytes(dtype, layout, trans, n, k) -> int:
    return lib().mg_syrk_workspace_bytes(dtype, layout, trans, n, k)


def mg_trmm_workspace_bytes(dtype, layout, side, trans_a, m, n) -> int:
    return lib().mg_trmm_workspace_bytes(dtype, layout, side, trans_a, m, n)


def mg_gemv_workspace_bytes(dtype, layout, trans_a, m, n, lda) -> int:
    return lib().mg_gemv_workspace_bytes(dtype, layout, trans_a, m, n, lda)


def mg_sgemm_batched(layout, trans_a, trans_b, m, n, k, alphas, A, a_offsets, lda, B, b_offsets, ldb, betas, C,
                     c_offsets, ldc, batch_count, stream=None, check=True) -> int:
    st = lib().mg_sgemm_batched(layout, trans_a, trans_b, m, n, k, _addr(alphas), _addr(A), _addr(a_offsets), lda,
                                _addr(B), _addr(b_offsets), ldb, _addr(betas), _addr(C), _addr(c_offsets), ldc,
                                batch_count, _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, "mg_sgemm_batched")
    return st


def mg_hgemm_batched(layout, trans_a, trans_b, m, n, k, alphas, A, a_offsets, lda, B, b_offsets, ldb, betas, C,
                     c_offsets, ldc, batch_count, stream=None, check=True) -> int:
    st = lib().mg_hgemm_batched(layout, trans_a, trans_b, m, n, k, _addr(alphas), _addr(A), _addr(a_offsets), lda,
                                _addr(B), _addr(b_offsets), ldb, _addr(betas), _addr(C), _addr(c_offsets), ldc,
                                batch_count, _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, "mg_hgemm_batched")
    return st


def mg_hgemm_strided_batched(layout, trans_a, trans_b, m, n, k, alpha, A, lda, stride_a, B, ldb, stride_b, beta, C,
                             ldc, stride_c, batch_count, stream=None, check=True) -> int:
    st = lib().mg_hgemm_strided_batched(layout, trans_a, trans_b, m, n, k, alpha, _addr(A), lda, stride_a, _addr(B),
                                        ldb, stride_b, beta, _addr(C), ldc, stride_c, batch_count, _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, "mg_hgemm_strided_batched")
    return st


def mg_sgemm_strided_batched(layout, trans_a, trans_b, m, n, k, alpha, A, lda, stride_a, B, ldb, stride_b, beta, C,
                             ldc, stride_c, batch_count, stream=None, check=True) -> int:
    st = lib().mg_sgemm_strided_batched(layout, trans_a, trans_b, m, n, k, alpha, _addr(A), lda, stride_a, _addr(B),
                                        ldb, stride_b, beta, _addr(C), ldc, stride_c, batch_count, _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, "mg_sgemm_strided_batched")
    return st


def _geometry(channels, height, width, kernel, pad, stride, dilation):
    return (channels, height, width, kernel[0], kernel[1], pad[0], pad[1], stride[0], stride[1], dilation[0], dilation[1])


def _im2col(name, channels, height, width, kernel, pad, stride, dilation, im, col, stream, check):
    st = getattr(lib(), name)(*_geometry(channels, height, width, kernel, pad, stride, dilation), _addr(im), _addr(col),
                              _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, name)
    return st


def mg_sim2col(channels, height, width, kernel, pad, stride, dilation, im, col, stream=None, check=True) -> int:
    """kernel, pad, stride, dilation: (h, w) pairs"""
    return _im2col("mg_sim2col", channels, height, width, kernel, pad, stride, dilation, im, col, stream, check)


def mg_him2col(channels, height, width, kernel, pad, stride, dilation, im, col, stream=None, check=True) -> int:
    return _im2col("mg_him2col", channels, height, width, kernel, pad, stride, dilation, im, col, stream, check)


def _conv2d(name, channels, height, width, kernel, pad, stride, dilation, filters, alpha, im, weights, beta, out,
            workspace, stream, check):
    ws, ws_bytes = _ws(workspace)
    st = getattr(lib(), name)(*_geometry(channels, height, width, kernel, pad, stride, dilation), filters, alpha,
                              _addr(im), _addr(weights), beta, _addr(out), ws, ws_bytes, _stream(stream))
    if check and st != MG_OK:
        raise MgError(st, name)
    return st


def mg_sconv2d(channels, height, width, kernel, pad, stride, dilation, filters, alpha, im, weights, beta, out,
               workspace=None, stream=None, check=True) -> int:
    return _conv2d("mg_sconv2d", channels, height, width, kernel, pad, stride, dilation, filters, alpha, im, weights,
                   beta, out, workspace, stream, check)


def mg_hconv2d(channels, height, width, kernel, pad, stride, dilation, filters, alpha, im, weights, beta, out,
               workspace=None, stream=None, check=True) -> int:
    return _conv2d("mg_hconv2d", channels, height, width, kernel, pad, stride, dilation, filters, alpha, im, weights,
                   beta, out, workspace, stream, check)


def mg_conv2d_workspace_bytes(dtype, channels, height, width, kernel, pad, stride, dilation, filters) -> int:
    return int(lib().mg_conv2d_workspace_bytes(dtype, *_geometry(channels, height, width, kernel, pad, stride, dilation),
                                               filters))


def mg_conv2d_out_extent(size, kernel, pad, stride, dilation) -> int:
    return int(lib().mg_conv2d_out_extent(size, kernel, pad, stride, dilation))


def mg_gemm_workspace_bytes(dtype, layout, trans_a, trans_b, m, n, k, lda, ldb, ldc) -> int:
    return int(lib().mg_gemm_workspace_bytes(dtype, layout, trans_a, trans_b, m, n, k, lda, ldb, ldc))


def mg_kernel_count() -> int:
    return int(lib().mg_kernel_count())


def mg_kernel_info(kernel_id: int) -> dict:
    cfg = mg_config()
    st = lib().mg_kernel_info(kernel_id, ctypes.byref(cfg))
    if st != MG_OK:
        raise MgError(st, "mg_kernel_info")
    d = cfg.as_dict()
    d["name"] = mg_kernel_name(kernel_id)
    return d


def mg_kernel_name(kernel_id: int) -> str:
    return lib().mg_kernel_name(kernel_id).decode()


def mg_lds_store_offset(k_contiguous, fragment_rows, tile_rows, row, k) -> int:
    return lib().mg_lds_store_offset(int(bool(k_contiguous)), fragment_rows, tile_rows, row, k)


def mg_lds_read_offset(k_contiguous, fragment_rows, tile_rows, wave_row, lane, fragment, k_step, half=0) -> int:
    return lib().mg_lds_read_offset(int(bool(k_contiguous)), fragment_rows, tile_rows, wave_row, lane, fragment, k_step, half)


def mg_lds_f32_store_offset(k_contiguous, tile_rows, row, k) -> int:
    return lib().mg_lds_f32_store_offset(int(bool(k_contiguous)), tile_rows, row, k)


def mg_lds_f32_read_offset(k_contiguous, tile_rows, wave_row, lane, fragment, k_step, element=0) -> int:
    return lib().mg_lds_f32_read_offset(int(bool(k_contiguous)), tile_rows, wave_row, lane, fragment, k_step, element)


def _checked(st, where, check):
    if check and st != MG_OK:
        raise MgError(st, where)
    return st


def mg_probe_empty_launch(stream=None, check=True) -> int:
    return _checked(lib().mg_probe_empty_launch(_stream(stream)), "mg_probe_empty_launch", check)


def mg_probe_mfma_only(rounds, sink, stream=None, check=True) -> int:
    return _checked(lib().mg_probe_mfma_only(rounds, _addr(sink), _stream(stream)), "mg_probe_mfma_only", check)


def mg_probe_hgemm_stamps(m, n, k, A, lda, B, ldb, C, ldc, stamps, stream=None, check=True) -> int:
    return _checked(lib().mg_probe_hgemm_stamps(m, n, k, _addr(A), lda, _addr(B), ldb, _addr(C), ldc, _addr(stamps),
                                                _stream(stream)), "mg_probe_hgemm_stamps", check)


def mg_query_selected(dtype, layout, trans_a, trans_b, m, n, k, lda, ldb, ldc, alpha=1.0, beta=0.0,
                      pointer_alignment=256) -> dict:
    cfg = mg_config()
    st = lib().mg_query_selected(dtype, layout, trans_a, trans_b, m, n, k, lda, ldb, ldc, alpha, beta,
                                 pointer_alignment, ctypes.byref(cfg))
    if st != MG_OK:
        raise MgError(st, "mg_query_selected")
    d = cfg.as_dict()
    d["name"] = mg_kernel_name(cfg.kernel_id)
    return d


def mg_override_config(kernel_id: int, split_k: int = 1, check=True) -> int:
    st = lib().mg_override_config(kernel_id, split_k)
    if check and st != MG_OK:
        raise MgError(st, "mg_override_config")
    return st


def mg_override_batched_config(kernel_id: int, check=True) -> int:
    st = lib().mg_override_batched_config(kernel_id)
    if check and st != MG_OK:
        raise MgError(st, "mg_override_batched_config")
    return st


def mg_override_fringe(mode: int, check=True) -> int:
    st = lib().mg_override_fringe(mode)
    if check and st != MG_OK:
        raise MgError(st, "mg_override_fringe")
    return st


def mg_clear_override() -> None:
    lib().mg_clear_override()


def mg_version() -> str:
    return lib().mg_version().decode()


def kernel_table():
    return [mg_kernel_info(i) for i in range(mg_kernel_count())]


def kernel_id(name: str) -> int:
    for i in range(mg_kernel_count()):
        if mg_kernel_name(i) == name:
            return i
    raise KeyError(name)
