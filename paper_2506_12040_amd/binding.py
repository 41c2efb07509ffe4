"""Thin ctypes binding of libbtc_hip.so: same names as include/btc.h, argument
marshalling only.  Tensors are torch CUDA(HIP) tensors used purely as device
buffers; every step of the computation runs in the library's kernels.  There
is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG, "libbtc_hip.so")

BTC_OK = 0
BTC_ERR_NULL, BTC_ERR_SHAPE, BTC_ERR_UNSUPPORTED, BTC_ERR_ALIGN = -1, -2, -3, -4
BTC_ERR_INDEX_RANGE, BTC_ERR_HIP, BTC_ERR_WORKSPACE = -5, -6, -7
BTC_F16, BTC_BF16, BTC_F32 = 0, 1, 2
(BTC_ENGINE_AUTO, BTC_ENGINE_EXPAND, BTC_ENGINE_LUT, BTC_ENGINE_MFMA_ONE, BTC_ENGINE_MFMA, BTC_ENGINE_TILED,
 BTC_ENGINE_GENERIC, BTC_ENGINE_FP4, BTC_ENGINE_CODE) = range(9)


class btc_shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("out", "in_", "v", "K", "b", "nchunks", "words_per_row")]


class BtcError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {status_str(status)} ({status})")
        self.status = status


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Load the built library; raise if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run paper_2506_12040_amd.build.build() "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        sp = ctypes.POINTER(btc_shape)
        L.btc_shape_init.restype = ctypes.c_int
        L.btc_shape_init.argtypes = [sp, i32, i32, i32, i32]
        L.btc_packed_bytes.restype = sz
        L.btc_packed_bytes.argtypes = [sp]
        L.btc_workspace_bytes.restype = sz
        L.btc_workspace_bytes.argtypes = [sp, i32, ctypes.c_int]
        L.btc_pack.restype = ctypes.c_int
        L.btc_pack.argtypes = [vp, sp, vp, vp, vp, sz]
        L.btc_unpack.restype = ctypes.c_int
        L.btc_unpack.argtypes = [vp, sp, vp, vp]
        L.btc_gemv.restype = ctypes.c_int
        L.btc_gemv.argtypes = [vp, sp, vp, vp, vp, vp, vp, i32, vp, ctypes.c_int, vp, sz]
        L.btc_gemv_static.restype = ctypes.c_int
        L.btc_gemv_static.argtypes = [vp, sp, vp, vp, vp, vp, vp, i32, vp, ctypes.c_int]
        L.btc_gemv_engine.restype = ctypes.c_int
        L.btc_gemv_engine.argtypes = [vp, sp, vp, vp, vp, vp, vp, i32, vp, ctypes.c_int, vp, sz, i32]
        L.btc_gemm.restype = ctypes.c_int
        L.btc_gemm.argtypes = [vp, sp, vp, vp, vp, vp, vp, ctypes.c_int, i32, vp, ctypes.c_int, vp, sz]
        L.btc_transform.restype = ctypes.c_int
        L.btc_transform.argtypes = [vp, vp, ctypes.c_int, i32, i32, i32, vp, vp, vp, vp, ctypes.c_int]
        L.btc_assign.restype = ctypes.c_int
        L.btc_assign.argtypes = [vp, vp, ctypes.c_int64, i32, vp, i32, vp, vp]
        L.btc_update_workspace_bytes.restype = sz
        L.btc_update_workspace_bytes.argtypes = [i32, i32]
        L.btc_update.restype = ctypes.c_int
        L.btc_update.argtypes = [vp, vp, vp, ctypes.c_int64, i32, vp, i32, vp, sz]
        L.btc_quantize_rows.restype = ctypes.c_int
        L.btc_quantize_rows.argtypes = [vp, vp, ctypes.c_int, i32, i32, i32, vp, vp, vp, vp]
        L.btc_aq_workspace_bytes.restype = sz
        L.btc_aq_workspace_bytes.argtypes = [sp, i32]
        L.btc_weight_rowsums.restype = ctypes.c_int
        L.btc_weight_rowsums.argtypes = [vp, sp, vp, vp, vp, vp, vp, vp, sz]
        L.btc_gemm_aq.restype = ctypes.c_int
        L.btc_gemm_aq.argtypes = [vp, sp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, ctypes.c_int, vp, sz]
        L.btc_transform_prepared_bytes.restype = ctypes.c_size_t
        L.btc_transform_prepared_bytes.argtypes = [i32, i32]
        L.btc_transform_prepare.restype = ctypes.c_int
        L.btc_transform_prepare.argtypes = [vp, i32, i32, vp, vp, vp, ctypes.c_size_t]
        L.btc_gemv_transformed_workspace_bytes.restype = ctypes.c_size_t
        L.btc_gemv_transformed_workspace_bytes.argtypes = [sp]
        L.btc_gemv_transformed.restype = ctypes.c_int
        L.btc_gemv_transformed.argtypes = [vp, sp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp,
                                           ctypes.c_size_t]
        L.btc_gemv_transformed_multi.restype = ctypes.c_int
        L.btc_gemv_transformed_multi.argtypes = [vp, sp, i32, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp,
                                                 ctypes.c_int, vp, ctypes.c_size_t]
        L.btc_gemv_multi.restype = ctypes.c_int
        L.btc_gemv_multi.argtypes = [vp, sp, i32, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, ctypes.c_size_t]
        L.btc_gemv_multi_shapes.restype = ctypes.c_int
        L.btc_gemv_multi_shapes.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, ctypes.c_size_t]
        L.btc_gemv_groups.restype = ctypes.c_int
        L.btc_gemv_groups.argtypes = [vp, sp, vp, vp, vp, vp, vp, i32, vp, vp, ctypes.c_int]
        L.btc_status_str.restype = ctypes.c_char_p
        L.btc_status_str.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def status_str(status: int) -> str:
    return lib().btc_status_str(int(status)).decode()


def _ptr(t) -> ctypes.c_void_p:
    """Device (or host) address of a torch tensor, a raw int address, or None."""
    if t is None:
        return ctypes.c_void_p(0)
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _nbytes(t) -> int:
    return 0 if t is None or isinstance(t, int) else t.numel() * t.element_size()


def _check(status: int, what: str) -> None:
    if status != BTC_OK:
        raise BtcError(status, what)


def btc_shape_init(out: int, n_in: int, v: int, K: int) -> btc_shape:
    s = btc_shape()
    _check(lib().btc_shape_init(ctypes.byref(s), out, n_in, v, K), "btc_shape_init")
    return s


def btc_packed_bytes(s: btc_shape) -> int:
    return lib().btc_packed_bytes(ctypes.byref(s))


def btc_workspace_bytes(s: btc_shape, rows: int, is_gemm: bool) -> int:
    return lib().btc_workspace_bytes(ctypes.byref(s), rows, int(is_gemm))


def btc_pack(s: btc_shape, idx, packed, workspace, stream=None, workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().btc_pack(_stream(stream), ctypes.byref(s), _ptr(idx), _ptr(packed), _ptr(workspace), wb),
           "btc_pack")


def btc_unpack(s: btc_shape, packed, idx, stream=None) -> None:
    _check(lib().btc_unpack(_stream(stream), ctypes.byref(s), _ptr(packed), _ptr(idx)), "btc_unpack")


def btc_gemv(s: btc_shape, packed, codebook, alpha, mu, x, batch: int, y, y_dtype: int,
             workspace=None, stream=None, workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().btc_gemv(_stream(stream), ctypes.byref(s), _ptr(packed), _ptr(codebook), _ptr(alpha), _ptr(mu),
                          _ptr(x), batch, _ptr(y), y_dtype, _ptr(workspace), wb), "btc_gemv")


def btc_gemv_static(s: btc_shape, packed, codebook, alpha, mu, x, batch: int, y, y_dtype: int, stream=None) -> None:
    _check(lib().btc_gemv_static(_stream(stream), ctypes.byref(s), _ptr(packed), _ptr(codebook), _ptr(alpha), _ptr(mu),
                                 _ptr(x), batch, _ptr(y), y_dtype), "btc_gemv_static")


def btc_gemv_engine(s: btc_shape, packed, codebook, alpha, mu, x, batch: int, y, y_dtype: int, engine: int,
                    workspace=None, stream=None, workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().btc_gemv_engine(_stream(stream), ctypes.byref(s), _ptr(packed), _ptr(codebook), _ptr(alpha), _ptr(mu),
                                 _ptr(x), batch, _ptr(y), y_dtype, _ptr(workspace), wb, engine), "btc_gemv_engine")


def btc_gemm(s: btc_shape, packed, codebook, alpha, mu, X, x_dtype: int, M: int, Y, y_dtype: int,
             workspace=None, stream=None, workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().btc_gemm(_stream(stream), ctypes.byref(s), _ptr(packed), _ptr(codebook), _ptr(alpha), _ptr(mu),
                          _ptr(X), x_dtype, M, _ptr(Y), y_dtype, _ptr(workspace), wb), "btc_gemm")


def btc_transform(X, x_dtype: int, M: int, n1: int, n2: int, sign_bits, P1, P2, Y, y_dtype: int, stream=None) -> None:
    _check(lib().btc_transform(_stream(stream), _ptr(X), x_dtype, M, n1, n2, _ptr(sign_bits), _ptr(P1), _ptr(P2),
                               _ptr(Y), y_dtype), "btc_transform")


def btc_quantize_rows(X, x_dtype: int, M: int, n: int, bits: int, Q, lo, step, qsum=None, stream=None) -> None:
    _check(lib().btc_quantize_rows(_stream(stream), _ptr(X), x_dtype, M, n, bits, _ptr(Q), _ptr(lo), _ptr(step),
                                   _ptr(qsum)), "btc_quantize_rows")


def btc_aq_workspace_bytes(s: BtcShape, M: int) -> int:
    return lib().btc_aq_workspace_bytes(ctypes.byref(s), M)


def btc_weight_rowsums(s: BtcShape, packed, codebook, alpha, mu, wsum, workspace, stream=None) -> None:
    _check(lib().btc_weight_rowsums(_stream(stream), ctypes.byref(s), _ptr(packed), _ptr(codebook), _ptr(alpha),
                                    _ptr(mu), _ptr(wsum), _ptr(workspace), _nbytes(workspace)), "btc_weight_rowsums")


def btc_gemm_aq(s: BtcShape, packed, codebook, alpha, mu, wsum, Q, lo, step, M: int, Y, y_dtype: int, workspace,
                stream=None) -> None:
    _check(lib().btc_gemm_aq(_stream(stream), ctypes.byref(s), _ptr(packed), _ptr(codebook), _ptr(alpha), _ptr(mu),
                             _ptr(wsum), _ptr(Q), _ptr(lo), _ptr(step), M, _ptr(Y), y_dtype, _ptr(workspace),
                             _nbytes(workspace)), "btc_gemm_aq")


def btc_transform_prepared_bytes(n1: int, n2: int) -> int:
    return lib().btc_transform_prepared_bytes(n1, n2)


def btc_transform_prepare(n1: int, n2: int, P1, P2, prepared, stream=None) -> None:
    _check(lib().btc_transform_prepare(_stream(stream), n1, n2, _ptr(P1), _ptr(P2), _ptr(prepared), _nbytes(prepared)),
           "btc_transform_prepare")


def btc_gemv_transformed_workspace_bytes(s: BtcShape) -> int:
    return lib().btc_gemv_transformed_workspace_bytes(ctypes.byref(s))


def btc_gemv_transformed(s: BtcShape, packed, codebook, alpha, mu, x, n1: int, n2: int, sign_bits, P1, P2, prepared, y,
                         y_dtype: int, workspace=None, xt_out=None, stream=None) -> None:
    _check(lib().btc_gemv_transformed(_stream(stream), ctypes.byref(s), _ptr(packed), _ptr(codebook), _ptr(alpha),
                                      _ptr(mu), _ptr(x), n1, n2, _ptr(sign_bits), _ptr(P1), _ptr(P2), _ptr(prepared),
                                      _ptr(xt_out), _ptr(y), y_dtype, _ptr(workspace), _nbytes(workspace)),
           "btc_gemv_transformed")


def _ptr_array(ts):
    return (ctypes.c_void_p * len(ts))(*[_ptr(t).value for t in ts])


def btc_gemv_multi(s: BtcShape, packed, codebook, alpha, mu, x, y, y_dtype: int, workspace=None, stream=None) -> None:
    """packed, codebook, alpha, mu, y: sequences of the same length (1..4), one entry per matrix."""
    _check(lib().btc_gemv_multi(_stream(stream), ctypes.byref(s), len(packed), _ptr_array(packed), _ptr_array(codebook),
                                _ptr_array(alpha), _ptr_array(mu), _ptr(x), _ptr_array(y), y_dtype, _ptr(workspace),
                                _nbytes(workspace)), "btc_gemv_multi")


def btc_gemv_multi_shapes(shapes, packed, codebook, alpha, mu, x, y, y_dtype: int, workspace=None, stream=None) -> None:
    """shapes, packed, codebook, alpha, mu, y: sequences of the same length (1..4), one entry per matrix; the shapes
    agree in everything but the number of rows."""
    arr = (ctypes.POINTER(btc_shape) * len(shapes))(*[ctypes.pointer(s) for s in shapes])
    _check(lib().btc_gemv_multi_shapes(_stream(stream), arr, len(shapes), _ptr_array(packed), _ptr_array(codebook),
                                       _ptr_array(alpha), _ptr_array(mu), _ptr(x), _ptr_array(y), y_dtype,
                                       _ptr(workspace), _nbytes(workspace)), "btc_gemv_multi_shapes")


def btc_gemv_transformed_multi(s: BtcShape, packed, codebook, alpha, mu, x, n1: int, n2: int, sign_bits, P1, P2, prepared,
                               y, y_dtype: int, workspace=None, xt_out=None, stream=None) -> None:
    """packed, codebook, alpha, mu, y: sequences of the same length (1..4), one entry per matrix."""
    _check(lib().btc_gemv_transformed_multi(_stream(stream), ctypes.byref(s), len(packed), _ptr_array(packed),
                                            _ptr_array(codebook), _ptr_array(alpha), _ptr_array(mu), _ptr(x), n1, n2,
                                            _ptr(sign_bits), _ptr(P1), _ptr(P2), _ptr(prepared), _ptr(xt_out),
                                            _ptr_array(y), y_dtype, _ptr(workspace), _nbytes(workspace)),
           "btc_gemv_transformed_multi")


def btc_gemv_groups(s: BtcShape, packed, codebook, alpha, mu, group_map, ngroups: int, x, y, y_dtype: int,
                    stream=None) -> None:
    _check(lib().btc_gemv_groups(_stream(stream), ctypes.byref(s), _ptr(packed), _ptr(codebook), _ptr(alpha), _ptr(mu),
                                 _ptr(group_map), ngroups, _ptr(x), _ptr(y), y_dtype), "btc_gemv_groups")


def btc_assign(vectors, N: int, v: int, codebook, K: int, z, dist2=None, stream=None) -> None:
    _check(lib().btc_assign(_stream(stream), _ptr(vectors), N, v, _ptr(codebook), K, _ptr(z), _ptr(dist2)),
           "btc_assign")


def btc_update_workspace_bytes(v: int, K: int) -> int:
    return lib().btc_update_workspace_bytes(v, K)


def btc_update(vectors, z, N: int, v: int, codebook, K: int, workspace, stream=None,
               workspace_bytes: Optional[int] = None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    _check(lib().btc_update(_stream(stream), _ptr(vectors), _ptr(z), N, v, _ptr(codebook), K, _ptr(workspace), wb),
           "btc_update")
