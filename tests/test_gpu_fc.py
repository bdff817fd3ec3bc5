"""GPU parity: fully connected forward / backward against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_1906_06440_amd as brg
import workloads as wl
from gpu_util import as_seen_by_gpu, check, dev, empty, host, workspace

pytestmark = pytest.mark.gpu


def _fwd(d, X, W, b, act, dtype=brg.F32, out=brg.F32):
    desc = brg.FcDesc(d.N, d.C, d.K, d.bn, d.bc, d.bk)
    dY = empty(d.y_shape, out)
    brg.brg_fc_fwd(desc, dtype, out, dev(X, dtype), dev(W, dtype), None if b is None else dev(b), act, dY)
    torch.cuda.synchronize()
    return host(dY)


def _bwd(d, dY, Y, X, W, act, dtype=brg.F32):
    desc = brg.FcDesc(d.N, d.C, d.K, d.bn, d.bc, d.bk)
    dX, dW, db = empty(d.x_shape, dtype), empty(d.w_shape), empty((d.K,))
    brg.brg_fc_bwd(desc, dtype, dev(dY, dtype), None if Y is None else dev(Y, dtype), dev(X, dtype), dev(W, dtype),
                   act, dX, dW, db)
    torch.cuda.synchronize()
    return host(dX), host(dW), host(db)


SHAPES = [(64, 64, 64, 64, 64, 64), (128, 192, 64, 64, 64, 64), (96, 80, 48, 32, 16, 16), (8, 24, 40, 4, 8, 8),
          (130, 70, 90, 65, 35, 45), (256, 128, 320, 64, 64, 64), (256, 128, 192, 64, 16, 16), (192, 96, 64, 32, 16, 16),
          (128, 128, 256, 32, 16, 16), (320, 256, 128, 64, 16, 16), (64, 2048, 1024, 32, 16, 16)]


@pytest.mark.parametrize("N,C,K,bn,bc,bk", SHAPES)
@pytest.mark.parametrize("dtype", [brg.F32, brg.BF16])
def test_fc_fwd_bwd_small(N, C, K, bn, bc, bk, dtype):
    rng = np.random.default_rng(N + C + K)
    d = orc.FcShape(N, C, K, bn, bc, bk)
    X = wl.uniform(rng, d.x_shape)
    W = wl.normal(rng, d.w_shape, (1.0 / C) ** 0.5)
    b = wl.normal(rng, (K,), 0.1)
    dY = wl.uniform(rng, d.y_shape)
    Xs, Ws, dYs = (as_seen_by_gpu(v, dtype) for v in (X, W, dY))
    for act in (brg.ACT_NONE, brg.ACT_RELU):
        Y = _fwd(d, X, W, b, act, dtype, dtype)
        check(Y, orc.fc_fwd(d, Xs, Ws, b, act, dtype == brg.BF16), dtype, "fc fwd")
        # backward is fed the GPU's own stored Y on both sides (ReLU mask must not flip)
        dX, dW, db = _bwd(d, dY, Y, X, W, act, dtype)
        rX, rW, rb = orc.fc_bwd(d, dYs, Y, Xs, Ws, act, dx_bf16=dtype == brg.BF16)
        check(dX, rX, dtype, "fc dX")
        check(dW, rW, dtype, "fc dW", out=brg.F32)
        check(db, rb, dtype, "fc db", out=brg.F32)
    assert (Y == 0).mean() > 0.2      # the ReLU case really masked something


def test_fc_optional_outputs_and_fp32_out_from_bf16():
    rng = np.random.default_rng(5)
    d = orc.FcShape(64, 64, 64)
    X, W = wl.uniform(rng, d.x_shape), wl.normal(rng, d.w_shape, 0.125)
    Y = _fwd(d, X, W, None, brg.ACT_NONE, brg.BF16, brg.F32)
    check(Y, orc.fc_fwd(d, as_seen_by_gpu(X, brg.BF16), as_seen_by_gpu(W, brg.BF16)), brg.BF16, "bf16->fp32", out=brg.F32)
    desc = brg.FcDesc(64, 64, 64, 64, 64, 64)
    dX = empty(d.x_shape, fill=7.0)
    brg.brg_fc_bwd(desc, brg.F32, dev(Y), None, dev(X), dev(W), brg.ACT_NONE, dX, None, None)
    torch.cuda.synchronize()
    rX, _, _ = orc.fc_bwd(d, Y, None, X, W, orc.ACT_NONE, want_dw=False, want_db=False)
    check(host(dX), rX, brg.F32, "dX only")


def _bwd_chain(d, dY, Y, X, W, act, act_in, dtype=brg.F32):
    desc = brg.FcDesc(d.N, d.C, d.K, d.bn, d.bc, d.bk)
    dX, dW, db = empty(d.x_shape, dtype), empty(d.w_shape), empty((d.K,))
    brg.brg_fc_bwd_chain(desc, dtype, dev(dY, dtype), None if Y is None else dev(Y, dtype), dev(X, dtype),
                         dev(W, dtype), act, act_in, dX, dW, db)
    torch.cuda.synchronize()
    return host(dX), host(dW), host(db)


@pytest.mark.parametrize("N,C,K,bn,bc,bk", [(128, 192, 64, 64, 64, 64), (96, 80, 48, 32, 16, 16)])
@pytest.mark.parametrize("dtype", [brg.F32, brg.BF16])
def test_fc_bwd_chain_fuses_producer_relu(N, C, K, bn, bc, bk, dtype):
    """act_in = RELU: the stored dX is dX o [X > 0] (X holds zeros where the producing ReLU clipped)."""
    rng = np.random.default_rng(N + K)
    d = orc.FcShape(N, C, K, bn, bc, bk)
    X = np.maximum(wl.uniform(rng, d.x_shape), 0)          # an input that came out of a ReLU
    W = wl.normal(rng, d.w_shape, (1.0 / C) ** 0.5)
    dY = wl.uniform(rng, d.y_shape)
    Xs, Ws, dYs = (as_seen_by_gpu(v, dtype) for v in (X, W, dY))
    dX, dW, db = _bwd_chain(d, dY, None, X, W, brg.ACT_NONE, brg.ACT_RELU, dtype)
    rX, rW, rb = orc.fc_bwd(d, dYs, None, Xs, Ws, orc.ACT_NONE, dx_bf16=dtype == brg.BF16)
    check(dX, rX * (Xs > 0), dtype, "masked dX")
    check(dW, rW, dtype, "dW", out=brg.F32)
    check(db, rb, dtype, "db", out=brg.F32)
    assert (dX == 0).mean() > 0.3


@pytest.mark.parametrize("N,C,K", [(192, 128, 256), (320, 256, 384), (448, 384, 128)])
@pytest.mark.parametrize("act_in", [brg.ACT_NONE, brg.ACT_RELU])
@pytest.mark.parametrize("act", [brg.ACT_NONE, brg.ACT_RELU])
def test_fc_bwd_128x64_tiles_forced(N, C, K, act_in, act, monkeypatch):
    """The 128 x 64-tile backward kernel (three-stage ring) on shapes below its size threshold: even block
    counts, chains of 3 to 7 blocks, with and without the ReLU mask on dY (register-staged operand) and the
    fused producer mask on dX; the last shape has K/64 = 2, so its by-data chain is too short and the launch
    must fall back to the 64 x 64 kernel."""
    monkeypatch.setenv("BRG_FC_G128", "1")
    brg.brg_tuning_reload()
    rng = np.random.default_rng(N + C + K)
    d = orc.FcShape(N, C, K, 64, 64, 64)
    X = np.maximum(wl.uniform(rng, d.x_shape), 0)
    W = wl.normal(rng, d.w_shape, (1.0 / C) ** 0.5)
    dY = wl.uniform(rng, d.y_shape)
    Y = np.maximum(wl.uniform(rng, d.y_shape), 0) if act == brg.ACT_RELU else None
    dX, dW, db = _bwd_chain(d, dY, Y, X, W, act, act_in, brg.F32)
    rX, rW, rb = orc.fc_bwd(d, dY, Y, X, W, orc.ACT_RELU if act == brg.ACT_RELU else orc.ACT_NONE)
    if act_in == brg.ACT_RELU:
        rX = rX * (X > 0)
    check(dX, rX, brg.F32, "dX")
    check(dW, rW, brg.F32, "dW", out=brg.F32)
    check(db, rb, brg.F32, "db", out=brg.F32)


def test_config3_mlp_full_size():
    """4 layers 1024->1024, minibatch 1024, 64x64x64 blocking: forward chained with bias+ReLU,
    backward chained from a synthetic dY; every layer also checked in isolation on identical inputs."""
    X0, Ws, bs, dYl = wl.cfg3_mlp()
    d = orc.FcShape(1024, 1024, 1024)
    acts_gpu = [X0]
    for l in range(4):
        Y = _fwd(d, acts_gpu[-1], Ws[l], bs[l], brg.ACT_RELU)
        check(Y, orc.fc_fwd(d, acts_gpu[-1], Ws[l], bs[l], orc.ACT_RELU), brg.F32, "layer %d fwd" % l)
        acts_gpu.append(Y)
    g = dYl
    for l in reversed(range(4)):
        dX, dW, db = _bwd(d, g, acts_gpu[l + 1], acts_gpu[l], Ws[l], brg.ACT_RELU)
        rX, rW, rb = orc.fc_bwd(d, g, acts_gpu[l + 1], acts_gpu[l], Ws[l], orc.ACT_RELU)
        check(dX, rX, brg.F32, "layer %d dX" % l)
        check(dW, rW, brg.F32, "layer %d dW" % l, out=brg.F32)
        check(db, rb, brg.F32, "layer %d db" % l, out=brg.F32)
        g = dX
    # the same chain the way the benchmark drives it: the ReLU backward of layer l-1 is fused into the
    # dX epilogue of layer l, so only the last layer masks its incoming gradient
    g = dYl
    for l in reversed(range(4)):
        act = brg.ACT_RELU if l == 3 else brg.ACT_NONE
        act_in = brg.ACT_RELU if l > 0 else brg.ACT_NONE
        Yl = acts_gpu[l + 1] if l == 3 else None
        dX, dW, db = _bwd_chain(d, g, Yl, acts_gpu[l], Ws[l], act, act_in)
        rX, rW, rb = orc.fc_bwd(d, g, Yl, acts_gpu[l], Ws[l], act)
        if l > 0:
            rX = rX * (acts_gpu[l] > 0)
        check(dX, rX, brg.F32, "chain layer %d dZ" % l)
        check(dW, rW, brg.F32, "chain layer %d dW" % l, out=brg.F32)
        check(db, rb, brg.F32, "chain layer %d db" % l, out=brg.F32)
        g = dX


def test_fc_paper_minibatch_1344():
    """The minibatch the paper runs its MLP at (section 4.1.3: 1344 = 21 blocks of 64), C = K = 1024, fp32: forward
    with bias + ReLU, then the fused backward launch with the ReLU mask and the producer mask."""
    X0, Ws, bs, dYl = wl.cfg3_mlp(N=1344, layers=1)
    d = orc.FcShape(1344, 1024, 1024)
    X0 = np.maximum(X0, 0)
    Y = _fwd(d, X0, Ws[0], bs[0], brg.ACT_RELU)
    check(Y, orc.fc_fwd(d, X0, Ws[0], bs[0], orc.ACT_RELU), brg.F32, "fwd")
    dX, dW, db = _bwd_chain(d, dYl, Y, X0, Ws[0], brg.ACT_RELU, brg.ACT_RELU)
    rX, rW, rb = orc.fc_bwd(d, dYl, Y, X0, Ws[0], orc.ACT_RELU)
    check(dX, rX * (X0 > 0), brg.F32, "dX")
    check(dW, rW, brg.F32, "dW", out=brg.F32)
    check(db, rb, brg.F32, "db", out=brg.F32)


def test_fc_bf16_16_blocks_full_size_runs_as_1x1_convolution():
    """bf16, bc = bk = 16, N = C = K = 1024: forward (bias + ReLU) and unmasked backward take the 1x1
    convolution kernels (the blocked layouts coincide), weight and bias gradients the transposing-read kernel."""
    rng = np.random.default_rng(16)
    d = orc.FcShape(1024, 1024, 1024, 64, 16, 16)
    X = wl.uniform(rng, d.x_shape)
    W = wl.normal(rng, d.w_shape, (1.0 / 1024) ** 0.5)
    b = wl.normal(rng, (1024,), 0.1)
    dY = wl.uniform(rng, d.y_shape)
    Xs, Ws, dYs = (as_seen_by_gpu(v, brg.BF16) for v in (X, W, dY))
    Y = _fwd(d, X, W, b, brg.ACT_RELU, brg.BF16, brg.BF16)
    check(Y, orc.fc_fwd(d, Xs, Ws, b, orc.ACT_RELU, out_bf16=True), brg.BF16, "fwd")
    dX, dW, db = _bwd(d, dY, None, X, W, brg.ACT_NONE, brg.BF16)
    rX, rW, rb = orc.fc_bwd(d, dYs, None, Xs, Ws, orc.ACT_NONE, dx_bf16=True)
    check(dX, rX, brg.BF16, "dX")
    check(dW, rW, brg.BF16, "dW", out=brg.F32)
    check(db, rb, brg.BF16, "db", out=brg.F32)


@pytest.mark.parametrize("N,C,K,bn,bc", [(256, 128, 192, 64, 16), (128, 256, 128, 32, 16), (1024, 1024, 1024, 64, 16),
                                         (256, 128, 192, 64, 64), (128, 320, 64, 64, 64), (1024, 1024, 1024, 64, 64)])
def test_fc_bf16_16_blocks_masked_backward_with_workspace(N, C, K, bn, bc):
    """bf16, bc = bk = 16 or 64, act = RELU and act_in = RELU with a workspace: dZ = dY o [Y > 0] is written to the
    workspace by a pass of its own, the tuned kernels run on it, and the producer's mask is applied to dX in place."""
    rng = np.random.default_rng(N + C + K + bn)
    d = orc.FcShape(N, C, K, bn, bc, bc)
    X = np.maximum(wl.uniform(rng, d.x_shape), 0)
    W = wl.normal(rng, d.w_shape, (1.0 / C) ** 0.5)
    Y = np.maximum(wl.uniform(rng, d.y_shape), 0)
    dY = wl.uniform(rng, d.y_shape)
    Xs, Ws, Ys, dYs = (as_seen_by_gpu(v, brg.BF16) for v in (X, W, Y, dY))
    desc = brg.FcDesc(N, C, K, bn, bc, bc)
    dX, dW, db = empty(d.x_shape, brg.BF16), empty(d.w_shape), empty((K,))
    ws = workspace(N * K * 2)
    brg.brg_fc_bwd_chain(desc, brg.BF16, dev(dY, brg.BF16), dev(Y, brg.BF16), dev(X, brg.BF16), dev(W, brg.BF16),
                         brg.ACT_RELU, brg.ACT_RELU, dX, dW, db, ws)
    torch.cuda.synchronize()
    rX, rW, rb = orc.fc_bwd(d, dYs, Ys, Xs, Ws, orc.ACT_RELU, dx_bf16=True)
    check(host(dX), rX * (Xs > 0), brg.BF16, "masked dX")
    check(host(dW), rW, brg.BF16, "dW", out=brg.F32)
    check(host(db), rb, brg.BF16, "db", out=brg.F32)
    assert (host(dX) == 0).mean() > 0.3


@pytest.mark.parametrize("knob,val", [("BRG_FC_GENERAL", "1"), ("BRG_FC_G64", "64"), ("BRG_FC_G64", "32"), ("BRG_NO_RING", "1"),
                                      ("BRG_FC_G128", "0"), ("BRG_FC_WGT_GENERAL", "1")])
@pytest.mark.parametrize("dtype,bc", [(brg.F32, 64), (brg.BF16, 16), (brg.BF16, 64)])
def test_fc_kernel_variants_forced(monkeypatch, knob, val, dtype, bc):
    """Every override that moves a fully connected layer to another kernel: same results."""
    monkeypatch.setenv(knob, val)
    brg.brg_tuning_reload()
    N, C, K = 256, 512, 256
    rng = np.random.default_rng(len(knob) + int(val))
    d = orc.FcShape(N, C, K, 64, bc, bc)
    X, W = wl.uniform(rng, d.x_shape), wl.normal(rng, d.w_shape, (1.0 / C) ** 0.5)
    b, dY = wl.normal(rng, (K,), 0.1), wl.uniform(rng, d.y_shape)
    Xs, Ws, dYs = (as_seen_by_gpu(v, dtype) for v in (X, W, dY))
    bf = dtype == brg.BF16
    Y = _fwd(d, X, W, b, brg.ACT_RELU, dtype, dtype)
    check(Y, orc.fc_fwd(d, Xs, Ws, b, orc.ACT_RELU, bf), dtype, "fwd")
    dX, dW, db = _bwd(d, dY, None, X, W, brg.ACT_NONE, dtype)
    rX, rW, rb = orc.fc_bwd(d, dYs, None, Xs, Ws, orc.ACT_NONE, dx_bf16=bf)
    check(dX, rX, dtype, "dX")
    check(dW, rW, dtype, "dW", out=brg.F32)
    check(db, rb, dtype, "db", out=brg.F32)


# Seeded random layers: block sizes 16, 32, 64 (equal or mixed), one to five blocks per dimension; forward with bias
# and ReLU, then the backward pass (with the workspace a bf16 layer needs for its masked form) on the GPU's own Y.
@pytest.mark.parametrize("dtype", [brg.F32, brg.BF16])
def test_fc_random_layers(dtype):
    rng = np.random.default_rng(777)
    for case in range(24):
        if rng.random() < 0.5:
            bn = bc = bk = int(rng.choice([16, 64]))
            if bn == 16:
                bn = int(rng.choice([16, 32, 64]))
        else:
            bn, bc, bk = (int(rng.choice([16, 32, 64])) for _ in range(3))
        N, C, K = bn * int(rng.integers(1, 6)), bc * int(rng.integers(1, 6)), bk * int(rng.integers(1, 6))
        what = "N%d C%d K%d blocks %d,%d,%d" % (N, C, K, bn, bc, bk)
        d = orc.FcShape(N, C, K, bn, bc, bk)
        X, W = wl.uniform(rng, d.x_shape), wl.normal(rng, d.w_shape, (1.0 / C) ** 0.5)
        b, dY = wl.normal(rng, (K,), 0.1), wl.uniform(rng, d.y_shape)
        Xs, Ws, dYs = (as_seen_by_gpu(v, dtype) for v in (X, W, dY))
        bf = dtype == brg.BF16
        Y = _fwd(d, X, W, b, brg.ACT_RELU, dtype, dtype)
        check(Y, orc.fc_fwd(d, Xs, Ws, b, orc.ACT_RELU, bf), dtype, what + " fwd")
        desc = brg.FcDesc(N, C, K, bn, bc, bk)
        dX, dW, db = empty(d.x_shape, dtype), empty(d.w_shape), empty((K,))
        ws = workspace(N * K * 2) if bf else None
        brg.brg_fc_bwd(desc, dtype, dev(dY, dtype), dev(Y, dtype), dev(X, dtype), dev(W, dtype), brg.ACT_RELU, dX, dW, db, ws)
        torch.cuda.synchronize()
        rX, rW, rb = orc.fc_bwd(d, dYs, Y, Xs, Ws, orc.ACT_RELU, dx_bf16=bf)
        check(host(dX), rX, dtype, what + " dX")
        check(host(dW), rW, dtype, what + " dW", out=brg.F32)
        check(host(db), rb, dtype, what + " db", out=brg.F32)
