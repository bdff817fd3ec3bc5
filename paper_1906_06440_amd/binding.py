"""ctypes binding of libbrg.so: same names and argument order as include/brg.h.

Tensors are torch tensors on a ROCm device (PyTorch is used for device memory
and streams only).  Each function enqueues on torch's current stream and raises
``BrgError`` on a non-zero status.  No computation happens in Python.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

__all__ = [
    "BrgError", "lib_path", "load", "status_name", "last_error", "version",
    "F32", "BF16", "ACT_NONE", "ACT_RELU", "ACT_SIGMOID", "ACT_TANH",
    "OK", "EINVAL", "EALIGN", "EUNSUPPORTED", "EHIP",
    "ConvDesc", "FcDesc", "LstmDesc",
    "brg_gemm", "brg_gemm_strided", "brg_conv_ws_bytes", "brg_conv_fwd", "brg_conv_bwd_data", "brg_conv_bwd_wgt",
    "brg_conv_bwd_wgt_ws_bytes", "brg_fc_fwd", "brg_fc_bwd", "brg_fc_bwd_chain", "brg_lstm_fwd", "brg_lstm_bwd",
    "brg_lstm_bwd_ws_bytes", "brg_lstm_bwd_ws_bytes_dtype", "brg_conv_bwd_wgt_noalloc", "brg_tuning_reload", "CONV_BWD_WGT_NOALLOC_MAX_BYTES", "EXPORTS",
]

F32, BF16 = 0, 1
ACT_NONE, ACT_RELU, ACT_SIGMOID, ACT_TANH = 0, 1, 2, 3
OK, EINVAL, EALIGN, EUNSUPPORTED, EHIP = 0, 1, 2, 3, 4
_STATUS = {0: "BRG_OK", 1: "BRG_EINVAL", 2: "BRG_EALIGN", 3: "BRG_EUNSUPPORTED", 4: "BRG_EHIP"}

EXPORTS = [
    "brg_last_error", "brg_version", "brg_gemm", "brg_gemm_strided", "brg_conv_ws_bytes", "brg_conv_fwd",
    "brg_conv_bwd_data", "brg_conv_bwd_wgt", "brg_conv_bwd_wgt_ws_bytes", "brg_fc_fwd", "brg_fc_bwd", "brg_fc_bwd_chain",
    "brg_lstm_fwd", "brg_lstm_bwd", "brg_lstm_bwd_ws_bytes", "brg_lstm_bwd_ws_bytes_dtype", "brg_conv_bwd_wgt_noalloc", "brg_tuning_reload",
]
CONV_BWD_WGT_NOALLOC_MAX_BYTES = 72 * 1024 * 1024

_HERE = os.path.dirname(os.path.abspath(__file__))


class BrgError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("%s: %s" % (_STATUS.get(status, str(status)), text))
        self.status = status


def lib_path() -> str:
    return os.path.join(_HERE, "libbrg.so")


_lib = None


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int64) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "bc", "bk")]


class FcDesc(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("N", "C", "K", "bn", "bc", "bk")]


class LstmDesc(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("T", "N", "C", "K", "bn", "bc", "bk")]


def load():
    """Load libbrg.so (built beforehand by ``build.build_library``); never builds, never falls back."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError("libbrg.so is not built (%s); run __graft_entry__.build() first" % path)
    lib = C.CDLL(path)
    i64, f32, vp, ci = C.c_int64, C.c_float, C.c_void_p, C.c_int
    lib.brg_last_error.restype = C.c_char_p
    lib.brg_version.restype = C.c_char_p
    lib.brg_gemm.argtypes = [ci, ci, i64, i64, i64, i64, i64, i64, vp, vp, vp, i64, f32, f32, vp, ci, vp]
    lib.brg_gemm_strided.argtypes = [ci, ci, i64, i64, i64, i64, i64, i64, vp, i64, vp, i64, vp, i64,
                                     f32, f32, vp, ci, vp]
    lib.brg_conv_ws_bytes.argtypes = [C.POINTER(ConvDesc), ci]
    lib.brg_conv_fwd.argtypes = [C.POINTER(ConvDesc), ci, ci, vp, vp, vp, vp, ci, vp, vp]
    lib.brg_conv_bwd_data.argtypes = [C.POINTER(ConvDesc), ci, ci, vp, vp, vp, vp, vp]
    lib.brg_conv_bwd_wgt.argtypes = [C.POINTER(ConvDesc), ci, vp, vp, vp, vp, vp]
    lib.brg_conv_bwd_wgt_ws_bytes.argtypes = [C.POINTER(ConvDesc), ci]
    lib.brg_conv_bwd_wgt_noalloc.argtypes = [C.POINTER(ConvDesc), ci, vp, vp, vp, vp]
    lib.brg_tuning_reload.argtypes = []
    lib.brg_tuning_reload.restype = None
    lib.brg_fc_fwd.argtypes = [C.POINTER(FcDesc), ci, ci, vp, vp, vp, ci, vp, vp]
    lib.brg_fc_bwd.argtypes = [C.POINTER(FcDesc), ci, vp, vp, vp, vp, ci, vp, vp, vp, vp, vp]
    lib.brg_fc_bwd_chain.argtypes = [C.POINTER(FcDesc), ci, vp, vp, vp, vp, ci, ci, vp, vp, vp, vp, vp]
    lib.brg_lstm_fwd.argtypes = [C.POINTER(LstmDesc), ci, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.brg_lstm_bwd.argtypes = [C.POINTER(LstmDesc), ci] + [vp] * 18
    lib.brg_lstm_bwd_ws_bytes.argtypes = [C.POINTER(LstmDesc)]
    lib.brg_lstm_bwd_ws_bytes_dtype.argtypes = [C.POINTER(LstmDesc), ci]
    for name in EXPORTS:
        if name not in ("brg_last_error", "brg_version", "brg_conv_ws_bytes", "brg_conv_bwd_wgt_ws_bytes",
                        "brg_lstm_bwd_ws_bytes", "brg_lstm_bwd_ws_bytes_dtype", "brg_tuning_reload"):
            getattr(lib, name).restype = ci
    lib.brg_conv_ws_bytes.restype = i64
    lib.brg_conv_bwd_wgt_ws_bytes.restype = i64
    lib.brg_lstm_bwd_ws_bytes.restype = i64
    lib.brg_lstm_bwd_ws_bytes_dtype.restype = i64
    _lib = lib
    return lib


def status_name(code: int) -> str:
    return _STATUS.get(code, str(code))


def last_error() -> str:
    return load().brg_last_error().decode()


def version() -> str:
    return load().brg_version().decode()


def _ptr(t):
    """Device address of a tensor (None -> NULL); ints pass through (raw addresses)."""
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0
    return C.c_void_p(int(stream))


def _check(status: int):
    if status != OK:
        raise BrgError(status, last_error())


def brg_gemm(dtype, out_dtype, m, n, k, lda, ldb, ldc, A_ptrs, B_ptrs, Cmat, count, alpha=1.0,
             beta=0.0, bias=None, act=ACT_NONE, stream=None):
    """Address-list form; ``A_ptrs``/``B_ptrs`` are int64 device tensors holding device addresses."""
    _check(load().brg_gemm(dtype, out_dtype, m, n, k, lda, ldb, ldc, _ptr(A_ptrs), _ptr(B_ptrs),
                           _ptr(Cmat), count, alpha, beta, _ptr(bias), act, _stream(stream)))


def brg_gemm_strided(dtype, out_dtype, m, n, k, lda, ldb, ldc, A, strideA, B, strideB, Cmat, count,
                     alpha=1.0, beta=0.0, bias=None, act=ACT_NONE, stream=None):
    _check(load().brg_gemm_strided(dtype, out_dtype, m, n, k, lda, ldb, ldc, _ptr(A), strideA, _ptr(B),
                                   strideB, _ptr(Cmat), count, alpha, beta, _ptr(bias), act,
                                   _stream(stream)))


def brg_conv_ws_bytes(desc: ConvDesc, dtype) -> int:
    return int(load().brg_conv_ws_bytes(C.byref(desc), dtype))


def brg_conv_fwd(desc: ConvDesc, dtype, out_dtype, I, Wt, O, bias=None, act=ACT_NONE, ws=None,
                 stream=None):
    _check(load().brg_conv_fwd(C.byref(desc), dtype, out_dtype, _ptr(I), _ptr(Wt), _ptr(O), _ptr(bias),
                               act, _ptr(ws), _stream(stream)))


def brg_conv_bwd_data(desc: ConvDesc, dtype, out_dtype, dO, Wt, dI, ws=None, stream=None):
    _check(load().brg_conv_bwd_data(C.byref(desc), dtype, out_dtype, _ptr(dO), _ptr(Wt), _ptr(dI),
                                    _ptr(ws), _stream(stream)))


def brg_conv_bwd_wgt_ws_bytes(desc: ConvDesc, dtype) -> int:
    return int(load().brg_conv_bwd_wgt_ws_bytes(C.byref(desc), dtype))


def brg_conv_bwd_wgt(desc: ConvDesc, dtype, I, dO, dWt, ws=None, stream=None):
    _check(load().brg_conv_bwd_wgt(C.byref(desc), dtype, _ptr(I), _ptr(dO), _ptr(dWt), _ptr(ws),
                                   _stream(stream)))


def brg_conv_bwd_wgt_noalloc(desc: ConvDesc, dtype, I, dO, dWt, stream=None):
    _check(load().brg_conv_bwd_wgt_noalloc(C.byref(desc), dtype, _ptr(I), _ptr(dO), _ptr(dWt), _stream(stream)))


def brg_tuning_reload():
    """Read the tuning-override environment variables again (they are read once, at the first call)."""
    load().brg_tuning_reload()


def brg_fc_fwd(desc: FcDesc, dtype, out_dtype, X, Wt, bias, act, Y, stream=None):
    _check(load().brg_fc_fwd(C.byref(desc), dtype, out_dtype, _ptr(X), _ptr(Wt), _ptr(bias), act,
                             _ptr(Y), _stream(stream)))


def brg_fc_bwd(desc: FcDesc, dtype, dY, Y, X, Wt, act, dX, dWt, dbias, ws=None, stream=None):
    _check(load().brg_fc_bwd(C.byref(desc), dtype, _ptr(dY), _ptr(Y), _ptr(X), _ptr(Wt), act, _ptr(dX),
                             _ptr(dWt), _ptr(dbias), _ptr(ws), _stream(stream)))


def brg_fc_bwd_chain(desc: FcDesc, dtype, dY, Y, X, Wt, act, act_in, dX, dWt, dbias, ws=None, stream=None):
    _check(load().brg_fc_bwd_chain(C.byref(desc), dtype, _ptr(dY), _ptr(Y), _ptr(X), _ptr(Wt), act, act_in,
                                   _ptr(dX), _ptr(dWt), _ptr(dbias), _ptr(ws), _stream(stream)))


def brg_lstm_fwd(desc: LstmDesc, dtype, x, W4, R4, b4, h0, s0, h, s, gates=None, ws=None, stream=None):
    _check(load().brg_lstm_fwd(C.byref(desc), dtype, _ptr(x), _ptr(W4), _ptr(R4), _ptr(b4), _ptr(h0),
                               _ptr(s0), _ptr(h), _ptr(s), _ptr(gates), _ptr(ws), _stream(stream)))


def brg_lstm_bwd_ws_bytes(desc: LstmDesc) -> int:
    return int(load().brg_lstm_bwd_ws_bytes(C.byref(desc)))


def brg_lstm_bwd_ws_bytes_dtype(desc: LstmDesc, dtype) -> int:
    return int(load().brg_lstm_bwd_ws_bytes_dtype(C.byref(desc), dtype))


def brg_lstm_bwd(desc: LstmDesc, dtype, x, W4, R4, h0, s0, h, s, gates, dh, ds_last, dx, dW4, dR4, db4, dh0, ds0, ws,
                 stream=None):
    _check(load().brg_lstm_bwd(C.byref(desc), dtype, _ptr(x), _ptr(W4), _ptr(R4), _ptr(h0), _ptr(s0), _ptr(h), _ptr(s),
                               _ptr(gates), _ptr(dh), _ptr(ds_last), _ptr(dx), _ptr(dW4), _ptr(dR4), _ptr(db4), _ptr(dh0),
                               _ptr(ds0), _ptr(ws), _stream(stream)))
