"""CPU oracle for the batch-reduce GEMM path -- TEST INFRASTRUCTURE ONLY.

This package wraps ``brg_oracle.c`` (plain C loops in double precision written
from the paper's defining equations) with ctypes.  Only ``tests/``, the smoke
check and the benchmark's ``cpu_baseline`` leg may import it.  It shares no
code with the GPU library and never imports it.

All arrays are C-contiguous ``numpy.float32``; bf16 experiments pass float32
arrays whose values are already bf16-representable.

``lstm_bwd`` (reverse-mode derivative of equations 1-6 of section 3.1) is plain
numpy in float64; it is pinned by ``torch.autograd`` in float64 and by central
differences (``tests/test_oracle_fc_lstm.py``); ``tests/test_gpu_lstm.py`` checks the
GPU backward pass against it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "brg_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

ACT_NONE, ACT_RELU, ACT_SIGMOID, ACT_TANH = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (+OpenMP on the outermost independent loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_round_bf16.restype = C.c_float
        _lib.orc_round_bf16.argtypes = [C.c_float]
        _lib.orc_f32_to_bf16_bits.restype = C.c_uint16
        _lib.orc_f32_to_bf16_bits.argtypes = [C.c_float]
        _lib.orc_bf16_bits_to_f32.restype = C.c_float
        _lib.orc_bf16_bits_to_f32.argtypes = [C.c_uint16]
        _lib.orc_conv_P.restype = C.c_int64
        _lib.orc_conv_Q.restype = C.c_int64
    return _lib


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i64(v):
    return C.c_int64(int(v))


# ------------------------------------------------------------------ bf16 ----
def f32_to_bf16_bits(x: float) -> int:
    return int(lib().orc_f32_to_bf16_bits(C.c_float(x)))


def bf16_bits_to_f32(b: int) -> float:
    return float(lib().orc_bf16_bits_to_f32(C.c_uint16(b)))


def round_bf16(a) -> np.ndarray:
    a = _f32(a)
    out = np.empty_like(a)
    lib().orc_round_bf16_array(_p(a), _p(out), _i64(a.size))
    return out


# ---------------------------------------------------------------- BRGEMM ----
def brgemm(A_blocks, B_blocks, m, n, k, lda, ldb, ldc, C_io, alpha=1.0, beta=0.0,
           bias=None, act=ACT_NONE, out_bf16=False) -> np.ndarray:
    """Address-list form. ``A_blocks``/``B_blocks`` are lists of float32 arrays (any views
    of contiguous float32 storage); ``C_io`` is updated in place and returned."""
    count = len(A_blocks)
    assert len(B_blocks) == count
    keep = [_f32(a) if not (isinstance(a, np.ndarray) and a.dtype == np.float32) else a for a in A_blocks]
    keepb = [_f32(b) if not (isinstance(b, np.ndarray) and b.dtype == np.float32) else b for b in B_blocks]
    ap = (C.c_void_p * max(count, 1))(*[a.ctypes.data for a in keep])
    bp = (C.c_void_p * max(count, 1))(*[b.ctypes.data for b in keepb])
    assert C_io.dtype == np.float32
    b = None if bias is None else _f32(bias)
    lib().orc_brgemm(_i64(m), _i64(n), _i64(k), _i64(lda), _i64(ldb), _i64(ldc), ap, bp,
                     _p(C_io), _i64(count), C.c_double(alpha), C.c_double(beta), _p(b),
                     C.c_int(act), C.c_int(int(out_bf16)))
    return C_io


def brgemm_strided(A, strideA, B, strideB, m, n, k, lda, ldb, ldc, C_io, count, alpha=1.0,
                   beta=0.0, bias=None, act=ACT_NONE, out_bf16=False) -> np.ndarray:
    A = _f32(A)
    B = _f32(B)
    b = None if bias is None else _f32(bias)
    assert C_io.dtype == np.float32
    lib().orc_brgemm_strided(_i64(m), _i64(n), _i64(k), _i64(lda), _i64(ldb), _i64(ldc),
                             _p(A), _i64(strideA), _p(B), _i64(strideB), _p(C_io), _i64(count),
                             C.c_double(alpha), C.c_double(beta), _p(b), C.c_int(act),
                             C.c_int(int(out_bf16)))
    return C_io


# --------------------------------------------------------------- layouts ----
def nchw_to_blocked(x, bc, Cp=None):
    x = _f32(x)
    N, Cc, H, W = x.shape
    Cp = Cp or ((Cc + bc - 1) // bc) * bc
    out = np.empty((N, Cp // bc, H, W, bc), np.float32)
    lib().orc_nchw_to_blocked(_p(x), _p(out), _i64(N), _i64(Cc), _i64(Cp), _i64(H), _i64(W), _i64(bc))
    return out


def blocked_to_nchw(xb, Cc=None):
    xb = _f32(xb)
    N, Cb, H, W, bc = xb.shape
    Cp = Cb * bc
    Cc = Cc or Cp
    out = np.empty((N, Cc, H, W), np.float32)
    lib().orc_blocked_to_nchw(_p(xb), _p(out), _i64(N), _i64(Cc), _i64(Cp), _i64(H), _i64(W), _i64(bc))
    return out


def kcrs_to_blocked(w, bc, bk, Cp=None):
    w = _f32(w)
    K, Cc, R, S = w.shape
    Cp = Cp or ((Cc + bc - 1) // bc) * bc
    out = np.empty((K // bk, Cp // bc, R, S, bc, bk), np.float32)
    lib().orc_kcrs_to_blocked(_p(w), _p(out), _i64(K), _i64(Cc), _i64(Cp), _i64(R), _i64(S), _i64(bc), _i64(bk))
    return out


def blocked_to_kcrs(wb, Cc=None):
    wb = _f32(wb)
    Kb, Cb, R, S, bc, bk = wb.shape
    K, Cp = Kb * bk, Cb * bc
    Cc = Cc or Cp
    out = np.empty((K, Cc, R, S), np.float32)
    lib().orc_blocked_to_kcrs(_p(wb), _p(out), _i64(K), _i64(Cc), _i64(Cp), _i64(R), _i64(S), _i64(bc), _i64(bk))
    return out


def w2_to_blocked(w, bc, bk):
    """[K][C] -> [K_b][C_b][b_c][b_k]"""
    w = _f32(w)
    K, Cc = w.shape
    out = np.empty((K // bk, Cc // bc, bc, bk), np.float32)
    lib().orc_w2_to_blocked(_p(w), _p(out), _i64(K), _i64(Cc), _i64(bc), _i64(bk))
    return out


def blocked_to_w2(wb):
    wb = _f32(wb)
    Kb, Cb, bc, bk = wb.shape
    out = np.empty((Kb * bk, Cb * bc), np.float32)
    lib().orc_blocked_to_w2(_p(wb), _p(out), _i64(Kb * bk), _i64(Cb * bc), _i64(bc), _i64(bk))
    return out


def a2_to_blocked(x, bn, bc):
    """[N][C] -> [N_b][C_b][b_n][b_c]"""
    x = _f32(x)
    N, Cc = x.shape
    out = np.empty((N // bn, Cc // bc, bn, bc), np.float32)
    lib().orc_a2_to_blocked(_p(x), _p(out), _i64(N), _i64(Cc), _i64(bn), _i64(bc))
    return out


def blocked_to_a2(xb):
    xb = _f32(xb)
    Nb, Cb, bn, bc = xb.shape
    out = np.empty((Nb * bn, Cb * bc), np.float32)
    lib().orc_blocked_to_a2(_p(xb), _p(out), _i64(Nb * bn), _i64(Cb * bc), _i64(bn), _i64(bc))
    return out


# ----------------------------------------------------------- convolution ----
class _ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int64) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "bc", "bk")]


@dataclass
class ConvShape:
    """C is the STORED channel count (multiple of bc)."""
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int = 1
    pad: int = 0
    bc: int = 16
    bk: int = 16

    def _c(self):
        return _ConvDesc(self.N, self.C, self.H, self.W, self.K, self.R, self.S, self.stride,
                         self.stride, self.pad, self.pad, self.bc, self.bk)

    @property
    def P(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def i_shape(self):
        return (self.N, self.C // self.bc, self.H, self.W, self.bc)

    @property
    def w_shape(self):
        return (self.K // self.bk, self.C // self.bc, self.R, self.S, self.bc, self.bk)

    @property
    def o_shape(self):
        return (self.N, self.K // self.bk, self.P, self.Q, self.bk)


def conv_fwd(d: ConvShape, I, Wt, bias=None, act=ACT_NONE, out_bf16=False):
    I, Wt = _f32(I), _f32(Wt)
    assert I.shape == d.i_shape and Wt.shape == d.w_shape
    O = np.empty(d.o_shape, np.float32)
    b = None if bias is None else _f32(bias)
    dd = d._c()
    lib().orc_conv_fwd(C.byref(dd), _p(I), _p(Wt), _p(O), _p(b), C.c_int(act), C.c_int(int(out_bf16)))
    return O


def conv_fwd_sample(d: ConvShape, I, Wt, idx4, bias=None, act=ACT_NONE, out_bf16=False):
    """Values of O at the (n, k, oj, oi) rows of ``idx4`` (int64 [S][4])."""
    I, Wt = _f32(I), _f32(Wt)
    idx4 = np.ascontiguousarray(idx4, dtype=np.int64)
    out = np.empty(idx4.shape[0], np.float32)
    b = None if bias is None else _f32(bias)
    dd = d._c()
    lib().orc_conv_fwd_sample(C.byref(dd), _p(I), _p(Wt), _p(b), C.c_int(act), C.c_int(int(out_bf16)),
                              _p(idx4), _i64(idx4.shape[0]), _p(out))
    return out


def conv_bwd_data(d: ConvShape, dO, Wt, out_bf16=False):
    dO, Wt = _f32(dO), _f32(Wt)
    assert dO.shape == d.o_shape and Wt.shape == d.w_shape
    dI = np.empty(d.i_shape, np.float32)
    dd = d._c()
    lib().orc_conv_bwd_data(C.byref(dd), _p(dO), _p(Wt), _p(dI), C.c_int(int(out_bf16)))
    return dI


def conv_bwd_data_sample(d: ConvShape, dO, Wt, idx4, out_bf16=False):
    """Values of dI at the (n, c, h, w) rows of ``idx4``."""
    dO, Wt = _f32(dO), _f32(Wt)
    idx4 = np.ascontiguousarray(idx4, dtype=np.int64)
    out = np.empty(idx4.shape[0], np.float32)
    dd = d._c()
    lib().orc_conv_bwd_data_sample(C.byref(dd), _p(dO), _p(Wt), C.c_int(int(out_bf16)), _p(idx4),
                                   _i64(idx4.shape[0]), _p(out))
    return out


def conv_bwd_wgt(d: ConvShape, I, dO):
    I, dO = _f32(I), _f32(dO)
    assert I.shape == d.i_shape and dO.shape == d.o_shape
    dW = np.empty(d.w_shape, np.float32)
    dd = d._c()
    lib().orc_conv_bwd_wgt(C.byref(dd), _p(I), _p(dO), _p(dW))
    return dW


# ------------------------------------------------------ fully connected ----
class _FcDesc(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("N", "C", "K", "bn", "bc", "bk")]


@dataclass
class FcShape:
    N: int
    C: int
    K: int
    bn: int = 64
    bc: int = 64
    bk: int = 64

    def _c(self):
        return _FcDesc(self.N, self.C, self.K, self.bn, self.bc, self.bk)

    @property
    def x_shape(self):
        return (self.N // self.bn, self.C // self.bc, self.bn, self.bc)

    @property
    def w_shape(self):
        return (self.K // self.bk, self.C // self.bc, self.bc, self.bk)

    @property
    def y_shape(self):
        return (self.N // self.bn, self.K // self.bk, self.bn, self.bk)


def fc_fwd(d: FcShape, X, Wt, bias=None, act=ACT_NONE, out_bf16=False):
    X, Wt = _f32(X), _f32(Wt)
    assert X.shape == d.x_shape and Wt.shape == d.w_shape
    Y = np.empty(d.y_shape, np.float32)
    b = None if bias is None else _f32(bias)
    dd = d._c()
    lib().orc_fc_fwd(C.byref(dd), _p(X), _p(Wt), _p(b), C.c_int(act), _p(Y), C.c_int(int(out_bf16)))
    return Y


def fc_bwd(d: FcShape, dY, Y, X, Wt, act=ACT_NONE, want_dx=True, want_dw=True, want_db=True,
           dx_bf16=False):
    dY, X, Wt = _f32(dY), _f32(X), _f32(Wt)
    Yc = None if Y is None else _f32(Y)
    assert act != ACT_RELU or Yc is not None
    dX = np.empty(d.x_shape, np.float32) if want_dx else None
    dW = np.empty(d.w_shape, np.float32) if want_dw else None
    db = np.empty(d.K, np.float32) if want_db else None
    dd = d._c()
    lib().orc_fc_bwd(C.byref(dd), _p(dY), _p(Yc), _p(X), _p(Wt), C.c_int(act), _p(dX), _p(dW), _p(db),
                     C.c_int(int(dx_bf16)))
    return dX, dW, db


# ------------------------------------------------------------------ LSTM ----
class _LstmDesc(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("T", "N", "C", "K", "bn", "bc", "bk")]


@dataclass
class LstmShape:
    T: int
    N: int
    C: int
    K: int
    bn: int = 16
    bc: int = 64
    bk: int = 64

    def _c(self):
        return _LstmDesc(self.T, self.N, self.C, self.K, self.bn, self.bc, self.bk)

    @property
    def w_shape(self):
        return (4, self.K // self.bk, self.C // self.bc, self.bc, self.bk)

    @property
    def r_shape(self):
        return (4, self.K // self.bk, self.K // self.bk, self.bk, self.bk)


def lstm_fwd(d: LstmShape, x, W4, R4, b4=None, h0=None, s0=None, want_gates=True):
    x, W4, R4 = _f32(x), _f32(W4), _f32(R4)
    assert x.shape == (d.T, d.N, d.C) and W4.shape == d.w_shape and R4.shape == d.r_shape
    b = None if b4 is None else _f32(b4)
    h0c = None if h0 is None else _f32(h0)
    s0c = None if s0 is None else _f32(s0)
    h = np.empty((d.T, d.N, d.K), np.float32)
    s = np.empty((d.T, d.N, d.K), np.float32)
    g = np.empty((4, d.T, d.N, d.K), np.float32) if want_gates else None
    dd = d._c()
    lib().orc_lstm_fwd(C.byref(dd), _p(x), _p(W4), _p(R4), _p(b), _p(h0c), _p(s0c), _p(h), _p(s), _p(g))
    return h, s, g


def lstm_fwd_bf16(d: LstmShape, x, W4, R4, b4=None, h0=None, s0=None):
    """The LSTM layer with bf16 operands (section 2 of the paper: the kernel is agnostic of the compute precision;
    the paper gives no recipe for the recurrence, this is the reading the GPU path documents): x, W4, R4 and h0
    hold bf16-representable values; every step is equations 1-6 in double precision (``lstm_fwd`` with T = 1) on
    the STORED h_{t-1}; h_t is rounded to bf16 (nearest even) once, when it is stored, and that stored value is what
    step t+1 multiplies; the cell state and the gate values are kept in fp32.  Returns h (bf16 values), s, gates."""
    d1 = LstmShape(1, d.N, d.C, d.K, d.bn, d.bc, d.bk)
    x = _f32(x)
    h = np.empty((d.T, d.N, d.K), np.float32)
    s = np.empty((d.T, d.N, d.K), np.float32)
    g = np.empty((4, d.T, d.N, d.K), np.float32)
    hp, sp = h0, s0
    for t in range(d.T):
        ht, st, gt = lstm_fwd(d1, x[t:t + 1], W4, R4, b4, hp, sp)
        h[t] = round_bf16(ht[0])
        s[t] = st[0]
        g[:, t] = gt[:, 0]
        hp, sp = h[t], s[t]
    return h, s, g


def lstm_bwd(d: LstmShape, x, W4, R4, h0, s0, h, s, gates, dh, ds_last=None):
    """Reverse-mode derivative of the LSTM layer in float64 (paper section 3.1: equations 1-6 define the
    forward pass; the paper reports the backward / weight-update pass without listing it, so this is the
    chain rule applied to those equations, step by step from t = T-1 down to 0).

    h, s [T][N][K] and gates [4][T][N][K] (values of i, c, f, o) are the forward results; dh [T][N][K] is the
    gradient of the loss with respect to every output h_t, ds_last [N][K] (optional) the one with respect to the
    final cell state.  Returns dx [T][N][C], dW4, dR4 (blocked like W4, R4), db4 [4][K], dh0, ds0 [N][K]."""
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    W = np.stack([f64(blocked_to_w2(W4[g])) for g in range(4)])       # [4][K][C]
    R = np.stack([f64(blocked_to_w2(R4[g])) for g in range(4)])       # [4][K][K]: z_g = R_g h_{t-1}
    x, h, s, gates, dh = f64(x), f64(h), f64(s), f64(gates), f64(dh)
    zero = np.zeros((d.N, d.K))
    h_init = zero if h0 is None else f64(h0)
    s_init = zero if s0 is None else f64(s0)
    dW, dR, db = np.zeros_like(W), np.zeros_like(R), np.zeros((4, d.K))
    dx = np.zeros((d.T, d.N, d.C))
    dh_next = zero.copy()
    ds_next = zero.copy() if ds_last is None else f64(ds_last)
    for t in range(d.T - 1, -1, -1):
        i, c, f, o = gates[0, t], gates[1, t], gates[2, t], gates[3, t]
        s_prev = s[t - 1] if t > 0 else s_init
        h_prev = h[t - 1] if t > 0 else h_init
        dht = dh[t] + dh_next                        # h_t feeds the output and step t+1
        ts = np.tanh(s[t])
        d_o = dht * ts                               # h_t = o * tanh(s_t)
        dst = dht * o * (1.0 - ts * ts) + ds_next    # s_t feeds h_t and s_{t+1}
        d_i, d_c, d_f = dst * c, dst * i, dst * s_prev   # s_t = f * s_{t-1} + i * c
        ds_next = dst * f
        dz = (d_i * i * (1.0 - i), d_c * (1.0 - c * c), d_f * f * (1.0 - f), d_o * o * (1.0 - o))
        dh_next = np.zeros((d.N, d.K))
        for g in range(4):                           # z_g = W_g x_t + R_g h_{t-1} + b_g
            dW[g] += dz[g].T @ x[t]
            dR[g] += dz[g].T @ h_prev
            db[g] += dz[g].sum(axis=0)
            dx[t] += dz[g] @ W[g]
            dh_next += dz[g] @ R[g]
    dW4 = np.stack([w2_to_blocked(dW[g].astype(np.float32), d.bc, d.bk) for g in range(4)])
    dR4 = np.stack([w2_to_blocked(dR[g].astype(np.float32), d.bk, d.bk) for g in range(4)])
    return dx, dW4, dR4, db, dh_next, ds_next


def rel_fro(got, want) -> float:
    """Relative Frobenius error ||got - want||_F / ||want||_F in float64 (0/0 -> 0).
    Pinned by hand values in tests/test_oracle_metrics.py."""
    g = np.asarray(got, dtype=np.float64).ravel()
    w = np.asarray(want, dtype=np.float64).ravel()
    den = np.linalg.norm(w)
    num = np.linalg.norm(g - w)
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return float(num / den)


def bf16_ulp(x) -> np.ndarray:
    """Spacing of bf16 numbers (8 significant bits) at magnitude |x|: 2**(floor(log2|x|) - 7); 0 at x == 0."""
    a = np.abs(np.asarray(x, dtype=np.float64))
    _, e = np.frexp(a)                       # a = m * 2**e, 0.5 <= m < 1  =>  floor(log2 a) = e - 1
    return np.where(a > 0, np.ldexp(1.0, e - 8), 0.0)


def elem_bound(got, want, out_bf16=False, widen=1.0) -> np.ndarray:
    """Per-element error bound that goes beside the Frobenius norm in the parity tests.

    fp32 result of an fp32-accumulated sum:   1e-5 * widen * (|want| + rms(want))
    bf16 result (one RNE rounding of such a sum): the same plus one bf16 spacing at max(|got|, |want|)
    (the two sides round sums that differ by the fp32 term, so they land on the same or on neighbouring
    bf16 numbers).  ``widen`` > 1 is for reductions much longer than 4096 terms and for results that pass
    through several dependent steps; every use states its reason."""
    w = np.abs(np.asarray(want, dtype=np.float64))
    rms = float(np.sqrt(np.mean(w * w))) if w.size else 0.0
    b = 1e-5 * widen * (w + rms)
    if out_bf16:
        b = b + bf16_ulp(np.maximum(w, np.abs(np.asarray(got, dtype=np.float64))))
    return b


def elem_excess(got, want, out_bf16=False, widen=1.0):
    """(max over elements of |got - want| / elem_bound, flat index of that element); <= 1 passes.
    A non-finite ``got`` gives inf.  0/0 counts as 0."""
    g = np.asarray(got, dtype=np.float64).ravel()
    w = np.asarray(want, dtype=np.float64).ravel()
    if g.size == 0:
        return 0.0, -1
    b = elem_bound(g, w, out_bf16, widen)
    err = np.abs(g - w)
    ratio = np.where(err == 0, 0.0, err / np.where(b > 0, b, np.finfo(np.float64).tiny))
    ratio = np.where(np.isfinite(g), ratio, np.inf)
    j = int(np.argmax(ratio))
    return float(ratio[j]), j
