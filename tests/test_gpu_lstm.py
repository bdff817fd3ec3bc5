"""GPU parity: LSTM layer forward and backward against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_1906_06440_amd as brg
import workloads as wl
from gpu_util import as_seen_by_gpu, check, dev, empty, host, workspace

pytestmark = pytest.mark.gpu


def _bwd_widen(T):
    """The gate gradients of step t carry the rounding errors of the T - t dependent steps before them (each an
    fp32 GEMM plus element-wise products), and dW, dR, db sum them over all steps: the element-wise bound is
    widened by sqrt(T), the growth of a sum of independent errors."""
    return max(1.0, float(T) ** 0.5)


def gpu_lstm(d, x, W4, R4, b4=None, h0=None, s0=None, want_gates=True, use_ws=True, dtype=brg.F32):
    """dtype BF16: x, W4, R4, h0 and the result h are bf16; bias, cell state and gate values stay fp32."""
    desc = brg.LstmDesc(d.T, d.N, d.C, d.K, d.bn, d.bc, d.bk)
    h, s = empty((d.T, d.N, d.K), dtype), empty((d.T, d.N, d.K))
    g = empty((4, d.T, d.N, d.K)) if want_gates else None
    opt = lambda a, dt=brg.F32: None if a is None else dev(a, dt)
    ws = workspace(64) if use_ws else None   # grid-barrier words (cleared by the library)
    brg.brg_lstm_fwd(desc, dtype, dev(x, dtype), dev(W4, dtype), dev(R4, dtype), opt(b4), opt(h0, dtype), opt(s0), h, s, g, ws)
    torch.cuda.synchronize()
    if ws is not None:   # word 1 of the workspace: the resident kernel gave up waiting
        assert int(ws[:8].view(torch.int32)[1].item()) == 0, "recurrent kernel reported a barrier time-out"
    torch.cuda.synchronize()
    return host(h), host(s), None if g is None else host(g)


@pytest.mark.parametrize("T,N,C,K,bc,bk", [(3, 16, 64, 64, 64, 64), (4, 20, 96, 80, 32, 16), (2, 70, 48, 36, 16, 4),
                                           (5, 64, 128, 192, 64, 64), (1, 3, 8, 8, 8, 8), (6, 32, 192, 256, 64, 64),
                                           (4, 48, 64, 128, 64, 64)])
def test_lstm_small(T, N, C, K, bc, bk):
    x, W4, R4, b4 = wl.cfg4_lstm(T, N, C, K, bc, bk, with_bias=True, seed_extra=T + N)
    W4 *= 4.0
    R4 *= 4.0
    rng = np.random.default_rng(T * N)
    h0, s0 = wl.uniform(rng, (N, K), -0.5, 0.5), wl.uniform(rng, (N, K), -0.5, 0.5)
    d = orc.LstmShape(T, N, C, K, 16, bc, bk)
    for kw in (dict(b4=b4, h0=h0, s0=s0), dict()):
        h, s, g = gpu_lstm(d, x, W4, R4, **kw)
        rh, rs, rg = orc.lstm_fwd(d, x, W4, R4, **kw)
        check(h, rh, brg.F32, "h")
        check(s, rs, brg.F32, "s")
        check(g, rg, brg.F32, "gates")
    # without a gates buffer / without workspace the general per-step path runs: same results within tolerance
    h2, s2, _ = gpu_lstm(d, x, W4, R4, want_gates=False)
    check(h2, rh, brg.F32, "h (no gates buffer)")
    check(s2, rs, brg.F32, "s (no gates buffer)")
    h3, s3, g3 = gpu_lstm(d, x, W4, R4, use_ws=False)
    check(h3, rh, brg.F32, "h (no workspace)")
    check(g3, rg, brg.F32, "gates (no workspace)")


def test_config4_full_size():
    """T=50, N=64, C=K=1024, zero bias and zero initial state."""
    x, W4, R4, _ = wl.cfg4_lstm()
    d = orc.LstmShape(50, 64, 1024, 1024, 16, 64, 64)
    h, s, g = gpu_lstm(d, x, W4, R4)
    rh, rs, rg = orc.lstm_fwd(d, x, W4, R4)
    check(h, rh, brg.F32, "h")
    check(s, rs, brg.F32, "s")
    check(g, rg, brg.F32, "gates")
    assert np.abs(h).max() < 1


@pytest.mark.parametrize("T,N,C,K,bc,bk", [(3, 16, 64, 64, 64, 64), (4, 20, 96, 80, 32, 16), (2, 70, 48, 36, 16, 4),
                                           (1, 3, 8, 8, 8, 8), (6, 32, 192, 256, 64, 64), (10, 64, 128, 128, 64, 64), (3, 128, 64, 320, 64, 64),
                                           (2, 64, 192, 64, 64, 64)])
@pytest.mark.parametrize("full", [True, False])
@pytest.mark.parametrize("dtype", [brg.F32, brg.BF16])
def test_lstm_backward(T, N, C, K, bc, bk, full, dtype):
    """Backward pass on the forward results the GPU stored (so both sides differentiate the same point): all six
    gradients with initial states and a gradient on the final cell state, or only dx / dW / dR from zero states.
    bf16: x, W4, R4, h0 and h are bf16 (h as the bf16 forward pass left it), the pass itself runs in fp32 on
    exactly those values, so the fp32 bound applies."""
    x, W4, R4, b4 = wl.cfg4_lstm(T, N, C, K, bc, bk, with_bias=True, seed_extra=T + N)
    W4 *= 4.0
    R4 *= 4.0
    rng = np.random.default_rng(T * N + 7)
    h0 = wl.uniform(rng, (N, K), -0.5, 0.5) if full else None
    s0 = wl.uniform(rng, (N, K), -0.5, 0.5) if full else None
    dh = wl.uniform(rng, (T, N, K))
    ds_last = wl.uniform(rng, (N, K)) if full else None
    d = orc.LstmShape(T, N, C, K, 16, bc, bk)
    h, s, g = gpu_lstm(d, x, W4, R4, b4=b4, h0=h0, s0=s0, dtype=dtype)
    desc = brg.LstmDesc(T, N, C, K, 16, bc, bk)
    opt = lambda a, dt=brg.F32: None if a is None else dev(a, dt)
    dx, dW4, dR4 = empty((T, N, C)), empty(d.w_shape), empty(d.r_shape)
    db4 = empty((4, K)) if full else None
    dh0 = empty((N, K)) if full else None
    ds0 = empty((N, K)) if full else None
    assert brg.brg_lstm_bwd_ws_bytes_dtype(desc, brg.F32) == brg.brg_lstm_bwd_ws_bytes(desc)
    ws = workspace(brg.brg_lstm_bwd_ws_bytes_dtype(desc, dtype))
    brg.brg_lstm_bwd(desc, dtype, dev(x, dtype), dev(W4, dtype), dev(R4, dtype), opt(h0, dtype), opt(s0), dev(h, dtype), dev(s), dev(g),
                     dev(dh), opt(ds_last), dx, dW4, dR4, db4, dh0, ds0, ws)
    torch.cuda.synchronize()
    x, W4, R4 = (as_seen_by_gpu(v, dtype) for v in (x, W4, R4))
    h0 = None if h0 is None else as_seen_by_gpu(h0, dtype)
    rx, rW, rR, rb, rh0, rs0 = orc.lstm_bwd(d, x, W4, R4, h0, s0, h, s, g, dh, ds_last)
    wd = _bwd_widen(T)
    check(host(dx), rx, brg.F32, "dx", widen=wd)
    check(host(dW4), rW, brg.F32, "dW4", widen=wd)
    check(host(dR4), rR, brg.F32, "dR4", widen=wd)
    if full:
        check(host(db4), rb, brg.F32, "db4", widen=wd)
        check(host(dh0), rh0, brg.F32, "dh0", widen=wd)
        check(host(ds0), rs0, brg.F32, "ds0", widen=wd)


def test_config4_backward_full_size():
    """cfg4 shape (T = 50, N = 64, C = K = 1024): backward from a random dh on the GPU's own forward results."""
    x, W4, R4, _ = wl.cfg4_lstm()
    d = orc.LstmShape(50, 64, 1024, 1024, 16, 64, 64)
    h, s, g = gpu_lstm(d, x, W4, R4)
    rng = np.random.default_rng(50)
    dh = wl.uniform(rng, (50, 64, 1024), -0.1, 0.1)
    desc = brg.LstmDesc(50, 64, 1024, 1024, 16, 64, 64)
    dx, dW4, dR4, db4 = empty((50, 64, 1024)), empty(d.w_shape), empty(d.r_shape), empty((4, 1024))
    ws = workspace(brg.brg_lstm_bwd_ws_bytes(desc))
    brg.brg_lstm_bwd(desc, brg.F32, dev(x), dev(W4), dev(R4), None, None, dev(h), dev(s), dev(g), dev(dh), None,
                     dx, dW4, dR4, db4, None, None, ws)
    torch.cuda.synchronize()
    rx, rW, rR, rb, _, _ = orc.lstm_bwd(d, x, W4, R4, None, None, h, s, g, dh)
    wd = _bwd_widen(50)
    check(host(dx), rx, brg.F32, "dx", widen=wd)
    check(host(dW4), rW, brg.F32, "dW4", widen=wd)
    check(host(dR4), rR, brg.F32, "dR4", widen=wd)
    check(host(db4), rb, brg.F32, "db4", widen=wd)


def test_lstm_resident_kernel_gives_up_loudly(monkeypatch):
    """The resident kernel's step barrier is a bounded wait.  With a limit of zero polls (set from the host) a
    workgroup that has to wait at all gives up: every wave exits normally, word 1 of the workspace is set, and the
    kernel enqueued behind it overwrites h, s and the gates with NaN, so the run cannot pass for a result.  The
    next call with the default limit, on the same workspace, is correct again (the library clears the words)."""
    T, N, C, K = 6, 64, 128, 1024
    x, W4, R4, b4 = wl.cfg4_lstm(T, N, C, K, 64, 64, with_bias=True, seed_extra=3)
    desc = brg.LstmDesc(T, N, C, K, 16, 64, 64)
    h, s, g = empty((T, N, K)), empty((T, N, K)), empty((4, T, N, K))
    ws = workspace(64)
    monkeypatch.setenv("BRG_LSTM_SPIN_LIMIT", "0")
    brg.brg_tuning_reload()
    brg.brg_lstm_fwd(desc, brg.F32, dev(x), dev(W4), dev(R4), dev(b4), None, None, h, s, g, ws)
    torch.cuda.synchronize()
    gave_up = int(ws[:8].view(torch.int32)[1].item()) != 0
    # 256 workgroups never all reach a barrier within zero polls of each other
    assert gave_up, "the wait was expected to give up"
    assert torch.isnan(h).all() and torch.isnan(s).all() and torch.isnan(g).all()
    monkeypatch.delenv("BRG_LSTM_SPIN_LIMIT")
    brg.brg_tuning_reload()
    brg.brg_lstm_fwd(desc, brg.F32, dev(x), dev(W4), dev(R4), dev(b4), None, None, h, s, g, ws)
    torch.cuda.synchronize()
    assert int(ws[:8].view(torch.int32)[1].item()) == 0
    d = orc.LstmShape(T, N, C, K, 16, 64, 64)
    rh, rs, rg = orc.lstm_fwd(d, x, W4, R4, b4)
    check(host(h), rh, brg.F32, "h after a give-up")
    check(host(s), rs, brg.F32, "s after a give-up")


def test_lstm_general_path_forced(monkeypatch):
    """BRG_LSTM_GENERAL: a shape of the resident / batched kernels on one general launch per time step."""
    monkeypatch.setenv("BRG_LSTM_GENERAL", "1")
    brg.brg_tuning_reload()
    T, N, C, K = 4, 64, 128, 128
    x, W4, R4, b4 = wl.cfg4_lstm(T, N, C, K, 64, 64, with_bias=True, seed_extra=21)
    d = orc.LstmShape(T, N, C, K, 16, 64, 64)
    h, s, g = gpu_lstm(d, x, W4, R4, b4=b4)
    rh, rs, rg = orc.lstm_fwd(d, x, W4, R4, b4=b4)
    check(h, rh, brg.F32, "h (general)")
    check(s, rs, brg.F32, "s (general)")
    check(g, rg, brg.F32, "gates (general)")


def _check_bf16_lstm(d, x, W4, R4, b4, h0, s0, h, s, g, what):
    """bf16 layer against the oracle's reading (h_t rounded to bf16 when stored and fed back rounded; fp32 state and
    gates).  (1) Whole sequence at the stated bf16 tolerance.  (2) Step by step from the GPU's OWN stored h_{t-1},
    s_{t-1} -- both sides then round the same sums, so every element must agree to the element-wise bound: a
    one-spacing difference of a stored h_t would otherwise feed every later step."""
    rh, rs, rg = orc.lstm_fwd_bf16(d, x, W4, R4, b4, h0, s0)
    assert orc.rel_fro(h, rh) <= 1e-2 and orc.rel_fro(s, rs) <= 1e-2 and orc.rel_fro(g, rg) <= 1e-2, what
    d1 = orc.LstmShape(1, d.N, d.C, d.K, d.bn, d.bc, d.bk)
    for t in range(d.T):
        hp = h[t - 1] if t else h0
        sp = s[t - 1] if t else s0
        th, ts, tg = orc.lstm_fwd(d1, x[t:t + 1], W4, R4, b4, hp, sp)
        check(h[t], orc.round_bf16(th[0]), brg.BF16, "%s h step %d" % (what, t), brg.BF16)
        check(s[t], ts[0], brg.BF16, "%s s step %d" % (what, t), brg.F32)
        check(g[:, t], tg[:, 0], brg.BF16, "%s gates step %d" % (what, t), brg.F32)


@pytest.mark.parametrize("T,N,C,K,bc,bk", [(3, 16, 64, 64, 64, 64), (4, 20, 96, 80, 32, 16), (5, 64, 128, 192, 64, 64), (1, 3, 8, 8, 8, 8),
                                           (6, 32, 192, 256, 64, 64), (4, 70, 64, 128, 64, 64), (3, 168, 128, 64, 64, 64),
                                           (2, 250, 64, 64, 64, 64)])
def test_lstm_bf16_small(T, N, C, K, bc, bk):
    """bf16 layer: resident kernel (64-wide blocks; one to four batch passes, ragged T*N) and the general path."""
    x, W4, R4, b4 = wl.cfg4_lstm(T, N, C, K, bc, bk, with_bias=True, seed_extra=T + N + 1)
    W4 *= 4.0
    R4 *= 4.0
    rng = np.random.default_rng(T * N + 3)
    h0, s0 = wl.uniform(rng, (N, K), -0.5, 0.5), wl.uniform(rng, (N, K), -0.5, 0.5)
    x, W4, R4, h0 = (as_seen_by_gpu(v, brg.BF16) for v in (x, W4, R4, h0))
    d = orc.LstmShape(T, N, C, K, 16, bc, bk)
    for kw in (dict(b4=b4, h0=h0, s0=s0), dict(b4=None, h0=None, s0=None)):
        h, s, g = gpu_lstm(d, x, W4, R4, dtype=brg.BF16, **kw)
        _check_bf16_lstm(d, x, W4, R4, kw["b4"], kw["h0"], kw["s0"], h, s, g, "bf16 lstm")
    # no workspace: one general launch per time step
    h, s, g = gpu_lstm(d, x, W4, R4, b4=b4, h0=h0, s0=s0, use_ws=False, dtype=brg.BF16)
    _check_bf16_lstm(d, x, W4, R4, b4, h0, s0, h, s, g, "bf16 lstm (general path)")


@pytest.mark.parametrize("T,N,C,K", [(4, 70, 64, 128), (3, 168, 128, 64), (2, 250, 64, 64), (3, 129, 192, 256)])
def test_lstm_fp32_more_than_64_batch_rows_on_the_resident_kernel(T, N, C, K):
    """N > 64: two to four batch passes per step; T*N not a multiple of the projection tile."""
    x, W4, R4, b4 = wl.cfg4_lstm(T, N, C, K, 64, 64, with_bias=True, seed_extra=T + N + 2)
    W4 *= 4.0
    R4 *= 4.0
    rng = np.random.default_rng(T * N + 5)
    h0, s0 = wl.uniform(rng, (N, K), -0.5, 0.5), wl.uniform(rng, (N, K), -0.5, 0.5)
    d = orc.LstmShape(T, N, C, K, 16, 64, 64)
    h, s, g = gpu_lstm(d, x, W4, R4, b4=b4, h0=h0, s0=s0)
    rh, rs, rg = orc.lstm_fwd(d, x, W4, R4, b4=b4, h0=h0, s0=s0)
    check(h, rh, brg.F32, "h")
    check(s, rs, brg.F32, "s")
    check(g, rg, brg.F32, "gates")


@pytest.mark.parametrize("dtype", [brg.F32, brg.BF16])
def test_lstm_paper_minibatch_168(dtype):
    """The minibatch of the paper's LSTM experiment (section 4.1.1: N = 168, C = K = 1024), twelve time steps."""
    T, N = 12, 168
    x, W4, R4, _ = wl.cfg4_lstm(T, N)
    d = orc.LstmShape(T, N, 1024, 1024, 16, 64, 64)
    if dtype == brg.BF16:
        x, W4, R4 = (as_seen_by_gpu(v, brg.BF16) for v in (x, W4, R4))
        h, s, g = gpu_lstm(d, x, W4, R4, dtype=brg.BF16)
        _check_bf16_lstm(d, x, W4, R4, None, None, None, h, s, g, "N=168 bf16")
    else:
        h, s, g = gpu_lstm(d, x, W4, R4)
        rh, rs, rg = orc.lstm_fwd(d, x, W4, R4)
        check(h, rh, brg.F32, "h")
        check(s, rs, brg.F32, "s")
        check(g, rg, brg.F32, "gates")


def test_config4_full_size_bf16():
    """cfg4's shape (T = 50, N = 64, C = K = 1024) with bf16 operands."""
    x, W4, R4, _ = wl.cfg4_lstm()
    x, W4, R4 = (as_seen_by_gpu(v, brg.BF16) for v in (x, W4, R4))
    d = orc.LstmShape(50, 64, 1024, 1024, 16, 64, 64)
    h, s, g = gpu_lstm(d, x, W4, R4, dtype=brg.BF16)
    _check_bf16_lstm(d, x, W4, R4, None, None, None, h, s, g, "cfg4 bf16")


# Seeded random layers: any T, N up to 200, C and K multiples of the block sizes; forward fp32 and bf16 (whatever
# path the call picks: resident kernels for 64-wide blocks and K a multiple of 64, one launch per step otherwise).
@pytest.mark.parametrize("dtype", [brg.F32, brg.BF16])
def test_lstm_random_layers(dtype):
    rng = np.random.default_rng(99)
    for case in range(10):
        if rng.random() < 0.6:
            bc = bk = 64
        else:
            bc, bk = int(rng.choice([8, 16, 32])), int(rng.choice([8, 16, 32]))
        T, N = int(rng.integers(1, 8)), int(rng.integers(1, 200))
        C, K = bc * int(rng.integers(1, 5)), bk * int(rng.integers(1, 6))
        x, W4, R4, b4 = wl.cfg4_lstm(T, N, C, K, bc, bk, with_bias=True, seed_extra=case)
        W4 *= 4.0
        R4 *= 4.0
        h0, s0 = wl.uniform(rng, (N, K), -0.5, 0.5), wl.uniform(rng, (N, K), -0.5, 0.5)
        x, W4, R4, h0 = (as_seen_by_gpu(v, dtype) for v in (x, W4, R4, h0))     # (the oracle is fed what the GPU is fed)
        d = orc.LstmShape(T, N, C, K, 16, bc, bk)
        h, s, g = gpu_lstm(d, x, W4, R4, b4=b4, h0=h0, s0=s0, dtype=dtype)
        what = "T%d N%d C%d K%d blocks %d,%d" % (T, N, C, K, bc, bk)
        if dtype == brg.BF16:
            _check_bf16_lstm(d, x, W4, R4, b4, h0, s0, h, s, g, what)
        else:
            rh, rs, rg = orc.lstm_fwd(d, x, W4, R4, b4, h0, s0)
            check(h, rh, brg.F32, what + " h")
            check(s, rs, brg.F32, what + " s")
            check(g, rg, brg.F32, what + " gates")
