"""Host-side checks of the C-ABI library: it loads, exports every declared symbol and
rejects bad arguments before touching the GPU (runs without a GPU)."""
import ctypes as C
import os
import re

import pytest

import paper_1906_06440_amd as brg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(brg.lib_path()):
        from paper_1906_06440_amd.build import build_library
        build_library()
    return brg.load()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "brg.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(brg_[a-z_0-9]+)\s*\(", header))
    assert declared == set(brg.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert brg.version().startswith("brg")


A16 = 0x1000  # a fake, 16-byte aligned, non-null "device address": validation must fail first


def test_gemm_argument_validation(lib):
    ok = dict(dtype=0, out=0, m=4, n=4, k=4, lda=4, ldb=4, ldc=4)

    def call(**kw):
        a = dict(ok, **kw)
        return lib.brg_gemm_strided(a["dtype"], a["out"], a["m"], a["n"], a["k"], a["lda"], a["ldb"], a["ldc"],
                                    a.get("A", A16), 16, a.get("B", A16), 16, a.get("C", A16), a.get("count", 1),
                                    1.0, 0.0, a.get("bias", None), a.get("act", 0), None)

    assert call(m=-1) == brg.EINVAL
    assert "negative" in brg.last_error()
    assert call(lda=3) == brg.EINVAL
    assert call(dtype=7) == brg.EINVAL
    assert call(act=9) == brg.EINVAL
    assert call(C=None) == brg.EINVAL
    assert call(A=None) == brg.EINVAL
    assert call(C=A16 + 4) == brg.EALIGN
    assert call(bias=A16 + 8) == brg.EALIGN
    assert call(dtype=0, out=1) == brg.EUNSUPPORTED
    assert call(m=0) == brg.OK          # empty problem: no launch, no GPU needed
    assert lib.brg_gemm(0, 0, 4, 4, 4, 4, 4, 4, None, None, A16, 2, 1.0, 0.0, None, 0, None) == brg.EINVAL


def test_conv_argument_validation(lib):
    def desc(**kw):
        v = dict(N=1, C=16, H=8, W=8, K=16, R=3, S=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1, bc=16, bk=16)
        v.update(kw)
        return brg.ConvDesc(**v)

    def fwd(d, I=A16, W=A16, O=A16):
        return lib.brg_conv_fwd(C.byref(d), 0, 0, I, W, O, None, 0, None, None)

    assert fwd(desc(C=24)) == brg.EINVAL
    assert "blocking" in brg.last_error()
    assert fwd(desc(stride_h=0)) == brg.EINVAL
    assert fwd(desc(H=1, W=1, pad_h=0, pad_w=0)) == brg.EINVAL
    assert fwd(desc(bc=8)) == brg.EUNSUPPORTED
    assert fwd(desc(), I=None) == brg.EINVAL
    assert fwd(desc(), O=A16 + 2) == brg.EALIGN
    assert lib.brg_conv_fwd(None, 0, 0, A16, A16, A16, None, 0, None, None) == brg.EINVAL
    assert lib.brg_conv_bwd_data(C.byref(desc(K=20)), 0, 0, A16, A16, A16, None, None) == brg.EINVAL
    assert lib.brg_conv_bwd_wgt(C.byref(desc()), 5, A16, A16, A16, None, None) == brg.EINVAL


def test_fc_and_lstm_argument_validation(lib):
    d = brg.FcDesc(N=64, C=64, K=64, bn=64, bc=64, bk=64)
    assert lib.brg_fc_fwd(C.byref(brg.FcDesc(N=60, C=64, K=64, bn=64, bc=64, bk=64)), 0, 0, A16, A16, None, 0,
                          A16, None) == brg.EINVAL
    assert lib.brg_fc_fwd(C.byref(d), 0, 0, None, A16, None, 0, A16, None) == brg.EINVAL
    assert lib.brg_fc_bwd(C.byref(d), 0, A16, None, A16, A16, brg.ACT_RELU, A16, None, None, None,
                          None) == brg.EINVAL      # ReLU without Y
    assert lib.brg_fc_bwd(C.byref(d), 0, A16, A16, A16, A16, brg.ACT_TANH, A16, None, None, None,
                          None) == brg.EUNSUPPORTED
    d16 = brg.FcDesc(N=64, C=64, K=64, bn=64, bc=16, bk=16)
    assert lib.brg_fc_bwd(C.byref(d16), 1, A16, A16, A16, A16, brg.ACT_RELU, A16, None, None, A16 + 8,
                          None) == brg.EALIGN      # misaligned workspace
    ld = brg.LstmDesc(T=2, N=4, C=64, K=64, bn=4, bc=64, bk=64)
    assert lib.brg_lstm_fwd(C.byref(ld), 7, A16, A16, A16, None, None, None, A16, A16, None, None,
                            None) == brg.EINVAL       # bad dtype (fp32 and bf16 are both built)
    assert lib.brg_lstm_fwd(C.byref(ld), 1, A16 + 2, A16, A16, None, None, None, A16, A16, None, None,
                            None) == brg.EALIGN
    assert lib.brg_lstm_fwd(C.byref(ld), 1, A16, A16, A16, None, None, None, A16, A16, A16, A16 + 4,
                            None) == brg.EALIGN       # misaligned workspace
    assert lib.brg_lstm_fwd(C.byref(brg.LstmDesc(T=2, N=4, C=60, K=64, bn=4, bc=64, bk=64)), 0, A16, A16, A16,
                            None, None, None, A16, A16, None, None, None) == brg.EINVAL
    assert lib.brg_lstm_fwd(C.byref(ld), 0, A16, A16, A16, None, None, None, None, A16, None, None,
                            None) == brg.EINVAL


def test_lstm_bwd_and_workspace_queries_validation(lib):
    ld = brg.LstmDesc(T=2, N=4, C=64, K=64, bn=4, bc=64, bk=64)
    lib.brg_lstm_bwd_ws_bytes.restype = C.c_int64
    assert lib.brg_lstm_bwd_ws_bytes(C.byref(ld)) == (4 * 2 + 17) * 4 * 64 * 4
    assert lib.brg_lstm_bwd_ws_bytes(None) == 0
    args = [A16] * 9 + [None] + [A16] * 3 + [None] * 3 + [A16, None]       # x .. dh, ds_last, dx dW4 dR4, db4 dh0 ds0, ws, stream
    lib.brg_lstm_bwd_ws_bytes_dtype.restype = C.c_int64
    base = (4 * 2 + 17) * 4 * 64 * 4
    assert lib.brg_lstm_bwd_ws_bytes_dtype(C.byref(ld), 0) == base
    # bf16: + fp32 copies of x [2][4][64], W4 and R4 [4][64][64], h [2][4][64], h0 [4][64]
    assert lib.brg_lstm_bwd_ws_bytes_dtype(C.byref(ld), 1) == base + 4 * (2 * 4 * 64 + 2 * 4 * 64 * 64 + 2 * 4 * 64 + 4 * 64)
    assert lib.brg_lstm_bwd(C.byref(ld), 7, *args) == brg.EINVAL            # bad dtype
    bad = list(args)
    bad[16] = None                                                           # no workspace
    assert lib.brg_lstm_bwd(C.byref(ld), 0, *bad) == brg.EINVAL
    bad = list(args)
    bad[10] = A16 + 4                                                        # misaligned dx
    assert lib.brg_lstm_bwd(C.byref(ld), 0, *bad) == brg.EALIGN
    assert lib.brg_lstm_bwd(C.byref(brg.LstmDesc(T=2, N=4, C=60, K=64, bn=4, bc=64, bk=64)), 0, *args) == brg.EINVAL
    # workspace size of the weight gradient: 0 for layers without a tuned kernel or a single pixel range
    lib.brg_conv_bwd_wgt_ws_bytes.restype = C.c_int64
    cd = brg.ConvDesc(64, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 16, 16)
    assert lib.brg_conv_bwd_wgt_ws_bytes(C.byref(cd), 1) > 0
    assert lib.brg_conv_bwd_wgt_ws_bytes(C.byref(brg.ConvDesc(64, 64, 56, 56, 64, 5, 5, 1, 1, 2, 2, 16, 16)), 1) == 0
    assert lib.brg_conv_bwd_wgt_ws_bytes(None, 1) == 0
