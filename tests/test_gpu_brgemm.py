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


def _ptr_list_case(dtype, out, m, n, k, count, lda, ldb, ldc, elem_off, alpha, beta, with_bias, act, seed):
    """Blocks scattered through two big buffers at offsets that are multiples of `elem_off` elements (1 = only
    element alignment), listed in a scrambled order, some blocks listed twice (blocks may repeat and alias)."""
    rng = np.random.default_rng(seed)
    esz = 2 if dtype == brg.BF16 else 4
    span_a, span_b = lda * k + 24, ldb * n + 24
    nblk = count + 3
    Abuf = (2 * rng.random(nblk * span_a + 64, dtype=np.float32) - 1)
    Bbuf = (2 * rng.random(nblk * span_b + 64, dtype=np.float32) - 1)
    pick = rng.integers(0, nblk, count)
    offa = [int(i) * span_a + int(rng.integers(0, 6)) * elem_off for i in pick]
    offb = [int(i) * span_b + int(rng.integers(0, 6)) * elem_off for i in rng.permutation(pick)]
    C0 = (2 * rng.random((n, ldc), dtype=np.float32) - 1)
    bias = (2 * rng.random(m, dtype=np.float32) - 1) if with_bias else None
    dA, dB = dev(Abuf, dtype), dev(Bbuf, dtype)
    ap = torch.tensor([dA.data_ptr() + o * esz for o in offa], dtype=torch.int64, device="cuda")
    bp = torch.tensor([dB.data_ptr() + o * esz for o in offb], dtype=torch.int64, device="cuda")
    dC = empty((n, ldc), out)
    dC.copy_(dev(C0, out))
    brg.brg_gemm(dtype, out, m, n, k, lda, ldb, ldc, ap, bp, dC, count, alpha, beta, None if bias is None else dev(bias), act)
    torch.cuda.synchronize()
    got = host(dC)
    Af, Bf = as_seen_by_gpu(Abuf, dtype), as_seen_by_gpu(Bbuf, dtype)
    want = as_seen_by_gpu(C0, out).copy()
    orc.brgemm([Af[o:] for o in offa], [Bf[o:] for o in offb], m, n, k, lda, ldb, ldc, want, alpha, beta, bias, act,
               out == brg.BF16)
    check(got[:, :m], want[:, :m], dtype, "pointer list %dx%dx%dx%d off %d" % (m, n, k, count, elem_off), out)
    assert np.array_equal(got[:, m:], as_seen_by_gpu(C0, out)[:, m:]), "rows of C between m and ldc are never written"


@pytest.mark.parametrize("dtype,out", [(brg.F32, brg.F32), (brg.BF16, brg.F32), (brg.BF16, brg.BF16)])
@pytest.mark.parametrize("m,n,count,lda,ldb,ldc,elem_off", [
    (64, 64, 16, 64, 64, 64, 8),        # cfg1's shape as an address list, 16-byte aligned blocks: direct loads
    (128, 192, 6, 136, 72, 132, 8),     # several tiles, padded leading dimensions, aligned
    (64, 128, 5, 64, 64, 64, 1),        # blocks with only element alignment: staged through registers
    (128, 64, 7, 129, 67, 128, 1),      # leading dimensions that break row alignment as well
    (64, 64, 2, 64, 64, 64, 8),         # short list (fp32: below the ring depth, general kernel)
])
def test_pointer_list_on_the_staged_kernels(dtype, out, m, n, count, lda, ldb, ldc, elem_off):
    """brg_gemm (the paper's two pointer arrays) with 64-deep blocks, m and n multiples of 64: the staged kernels."""
    _ptr_list_case(dtype, out, m, n, 64, count, lda, ldb, ldc, elem_off, 1.0, 0.0, False, brg.ACT_NONE, seed=m + n + count)
    _ptr_list_case(dtype, out, m, n, 64, count, lda, ldb, ldc, elem_off, 0.75, -0.5, True, brg.ACT_RELU, seed=m + n + count + 1)


@pytest.mark.parametrize("out", [brg.F32, brg.BF16])
@pytest.mark.parametrize("m,n,count,lda,ldb,ldc", [(64, 64, 16, 64, 64, 64), (256, 128, 3, 264, 64, 256), (64, 320, 1, 64, 80, 68),
                                                   (1024, 1024, 16, 1024, 64, 1024)])
def test_bf16_strided_blocks_on_the_bf16_matrix_instruction(out, m, n, count, lda, ldb, ldc):
    """brg_gemm_strided, bf16, 64-deep blocks (the first shape is cfg1's chain in bf16; the last a 1024-cubed GEMM
    as 16 blocks): plain, and with alpha, beta, bias and an activation."""
    k = 64
    rng = np.random.default_rng(m + n + count)
    sa, sb = lda * k + 8, ldb * n + 16
    A = (2 * rng.random(count * sa, dtype=np.float32) - 1)
    B = (2 * rng.random(count * sb, dtype=np.float32) - 1)
    C0 = (2 * rng.random((n, ldc), dtype=np.float32) - 1)
    bias = (2 * rng.random(m, dtype=np.float32) - 1)
    for alpha, beta, b, act in [(1.0, 0.0, None, brg.ACT_NONE), (0.5, -1.5, bias, brg.ACT_TANH)]:
        got = _run_strided(A, B, m, n, k, lda, ldb, ldc, count, sa, sb, brg.BF16, out, alpha, beta, C0, b, act)
        want = _oracle_strided(A, B, m, n, k, lda, ldb, ldc, count, sa, sb, brg.BF16, out, alpha, beta, C0, b, act)
        check(got[:, :m], want[:, :m], brg.BF16, f"bf16 {m}x{n}x{k}x{count}", out)
        assert np.array_equal(got[:, m:], as_seen_by_gpu(C0, out)[:, m:])


# Seeded random calls of the stride form: any m, n, k up to 150 (half of them multiples of 64, where the tuned
# kernels apply), padded leading dimensions, chains of 0..20 blocks, strides that are zero, equal to a block or
# larger, random alpha / beta / bias, none or ReLU (the saturating activations have their own test with pre-activations
# of order one: behind sums of order ten the absolute rounding error of the sum exceeds a bound taken from outputs below one).
@pytest.mark.parametrize("dtype,out", [(brg.F32, brg.F32), (brg.BF16, brg.F32), (brg.BF16, brg.BF16)])
def test_random_strided_calls(dtype, out):
    rng = np.random.default_rng(2024)
    for case in range(40):
        if rng.random() < 0.5:
            m, n, k = 64 * int(rng.integers(1, 3)), 64 * int(rng.integers(1, 3)), 64
        else:
            m, n, k = (int(rng.integers(1, 151)) for _ in range(3))
        count = int(rng.integers(0, 21))
        lda, ldb, ldc = m + 8 * int(rng.integers(0, 3)), k + 8 * int(rng.integers(0, 3)), m + 8 * int(rng.integers(0, 3))
        sa = int(rng.choice([0, lda * k, lda * k + 16]))
        sb = int(rng.choice([0, ldb * n, ldb * n + 24]))
        A = 2 * rng.random(max(1, count) * (lda * k + 16), dtype=np.float32) - 1
        B = 2 * rng.random(max(1, count) * (ldb * n + 24), dtype=np.float32) - 1
        C0 = 2 * rng.random((n, ldc), dtype=np.float32) - 1
        bias = (2 * rng.random(m, dtype=np.float32) - 1) if rng.random() < 0.5 else None
        alpha, beta = float(rng.choice([1.0, 0.5, -2.0])), float(rng.choice([0.0, 1.0, -0.5]))
        act = int(rng.choice([brg.ACT_NONE, brg.ACT_RELU]))
        what = "case %d: %dx%dx%d count %d ld %d,%d,%d strides %d,%d alpha %g beta %g act %d" % (
            case, m, n, k, count, lda, ldb, ldc, sa, sb, alpha, beta, act)
        got = _run_strided(A, B, m, n, k, lda, ldb, ldc, count, sa, sb, dtype, out, alpha, beta, C0, bias, act)
        want = _oracle_strided(A, B, m, n, k, lda, ldb, ldc, count, sa, sb, dtype, out, alpha, beta, C0, bias, act)
        check(got[:, :m], want[:, :m], dtype, what, out)
        assert np.array_equal(got[:, m:], as_seen_by_gpu(C0, out)[:, m:]), what
