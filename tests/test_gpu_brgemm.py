"""GPU parity: brg_gemm / brg_gemm_strided against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_1906_06440_amd as brg
import workloads as wl
from gpu_util import TOL, as_seen_by_gpu, check, dev, empty, host

pytestmark = pytest.mark.gpu


def _run_strided(A, B, m, n, k, lda, ldb, ldc, count, sa, sb, dtype=brg.F32, out=brg.F32, alpha=1.0,
                 beta=0.0, C0=None, bias=None, act=brg.ACT_NONE):
    dA, dB = dev(A, dtype), dev(B, dtype)
    dC = empty((n, ldc), out) if C0 is None else dev(C0, out)
    dbias = None if bias is None else dev(bias)
    brg.brg_gemm_strided(dtype, out, m, n, k, lda, ldb, ldc, dA, sa, dB, sb, dC, count, alpha, beta, dbias, act)
    torch.cuda.synchronize()
    return host(dC)


def _oracle_strided(A, B, m, n, k, lda, ldb, ldc, count, sa, sb, dtype, out, alpha, beta, C0, bias, act):
    Af, Bf = as_seen_by_gpu(A, dtype), as_seen_by_gpu(B, dtype)
    C = np.zeros((n, ldc), np.float32) if C0 is None else as_seen_by_gpu(C0, out).copy()
    orc.brgemm_strided(Af, sa, Bf, sb, m, n, k, lda, ldb, ldc, C, count, alpha, beta, bias, act, out == brg.BF16)
    return C


def test_config1_fp32_strided_and_pointer_list():
    A, B = wl.cfg1_brgemm()
    want = np.zeros((64, 64), np.float32)
    orc.brgemm(list(A), list(B), 64, 64, 64, 64, 64, 64, want)
    got = _run_strided(A, B, 64, 64, 64, 64, 64, 64, 16, 4096, 4096)
    check(got, want, brg.F32, "cfg1 strided")
    # address-list form, blocks listed in a scrambled order and B taken from another buffer
    dA, dB = dev(A), dev(B)
    perm = np.random.default_rng(1).permutation(16)
    ap = torch.tensor([dA.data_ptr() + int(i) * 4096 * 4 for i in perm], dtype=torch.int64, device="cuda")
    bp = torch.tensor([dB.data_ptr() + int(i) * 4096 * 4 for i in perm], dtype=torch.int64, device="cuda")
    dC = empty((64, 64))
    brg.brg_gemm(brg.F32, brg.F32, 64, 64, 64, 64, 64, 64, ap, bp, dC, 16)
    torch.cuda.synchronize()
    check(host(dC), want, brg.F32, "cfg1 pointer list")
    # bitwise run-to-run determinism (no atomics on the path)
    dC2 = empty((64, 64))
    brg.brg_gemm(brg.F32, brg.F32, 64, 64, 64, 64, 64, 64, ap, bp, dC2, 16)
    torch.cuda.synchronize()
    assert torch.equal(dC, dC2)


def test_all_ones_closed_form():
    A = np.ones((16, 64, 64), np.float32)
    got = _run_strided(A, A, 64, 64, 64, 64, 64, 64, 16, 4096, 4096)
    assert np.all(got == 1024.0)


SHAPES = [  # m n k count lda ldb ldc
    (1, 1, 1, 1, 1, 1, 1), (5, 3, 7, 2, 5, 7, 5), (64, 64, 16, 3, 64, 16, 64), (70, 66, 19, 5, 72, 24, 80),
    (129, 33, 64, 2, 129, 64, 129), (200, 130, 40, 4, 208, 48, 200), (16, 300, 16, 36, 16, 32, 16),
    (64, 64, 64, 1, 64, 64, 64), (31, 257, 3, 9, 40, 4, 36),
    # 64-deep blocks, m and n multiples of 64, chains of 4 and more: the ring kernel with alpha, beta, bias, activation
    (128, 128, 64, 6, 128, 64, 128), (64, 192, 64, 4, 72, 68, 64), (64, 64, 64, 17, 64, 64, 64),
]


@pytest.mark.parametrize("m,n,k,count,lda,ldb,ldc", SHAPES)
@pytest.mark.parametrize("dtype,out", [(brg.F32, brg.F32), (brg.BF16, brg.F32), (brg.BF16, brg.BF16)])
def test_shapes_ragged_tails(m, n, k, count, lda, ldb, ldc, dtype, out):
    rng = np.random.default_rng(m * 7 + n * 3 + k)
    sa, sb = lda * k + 8, ldb * n + 8
    A = (2 * rng.random(count * sa, dtype=np.float32) - 1)
    B = (2 * rng.random(count * sb, dtype=np.float32) - 1)
    C0 = (2 * rng.random((n, ldc), dtype=np.float32) - 1)
    bias = (2 * rng.random(m, dtype=np.float32) - 1)
    for alpha, beta, b, act in [(1.0, 0.0, None, brg.ACT_NONE), (0.5, -1.5, bias, brg.ACT_RELU)]:
        got = _run_strided(A, B, m, n, k, lda, ldb, ldc, count, sa, sb, dtype, out, alpha, beta, C0, b, act)
        want = _oracle_strided(A, B, m, n, k, lda, ldb, ldc, count, sa, sb, dtype, out, alpha, beta, C0, b, act)
        check(got[:, :m], want[:, :m], dtype, f"{m}x{n}x{k}x{count}", out)
        # rows of C between m and ldc are never written
        ref_pad = as_seen_by_gpu(C0, out)[:, m:]
        assert np.array_equal(got[:, m:], ref_pad)


def test_beta0_does_not_read_c_and_count0():
    A, B = wl.cfg1_brgemm(count=2, m=16, n=16, k=16)
    got = _run_strided(A, B, 16, 16, 16, 16, 16, 16, 2, 256, 256, C0=np.full((16, 16), np.nan, np.float32))
    assert np.isfinite(got).all()
    C0 = np.arange(256, dtype=np.float32).reshape(16, 16)
    got = _run_strided(A, B, 16, 16, 16, 16, 16, 16, 0, 256, 256, beta=2.0, C0=C0)
    assert np.array_equal(got, 2 * C0)
    got = _run_strided(A, B, 16, 16, 16, 16, 16, 16, 0, 256, 256, beta=0.0, C0=np.full((16, 16), np.nan, np.float32))
    assert np.all(got == 0)


def test_sigmoid_tanh_epilogue_and_aliasing():
    A, _ = wl.cfg1_brgemm(count=3, m=32, n=32, k=32)
    A *= 0.2
    for act in (brg.ACT_SIGMOID, brg.ACT_TANH):
        got = _run_strided(A, A, 32, 32, 32, 32, 32, 32, 3, 1024, 1024, act=act)   # A aliases B
        want = _oracle_strided(A, A, 32, 32, 32, 32, 32, 32, 3, 1024, 1024, brg.F32, brg.F32, 1.0, 0.0, None, None, act)
        check(got, want, brg.F32, "act %d" % act)


@pytest.mark.parametrize("knob", ["BRG_GEMM_GENERAL", "BRG_NO_RING"])
def test_cfg1_on_the_other_kernels(monkeypatch, knob):
    """The general tile kernel and the double-buffered block kernel on the cfg1 chain."""
    monkeypatch.setenv(knob, "1")
    brg.brg_tuning_reload()
    A, B = wl.cfg1_brgemm()
    want = np.zeros((64, 64), np.float32)
    orc.brgemm(list(A), list(B), 64, 64, 64, 64, 64, 64, want)
    check(_run_strided(A, B, 64, 64, 64, 64, 64, 64, 16, 4096, 4096), want, brg.F32, "cfg1 " + knob)
