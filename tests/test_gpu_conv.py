"""GPU parity: convolution forward / backward-data / weight-gradient against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_1906_06440_amd as brg
import workloads as wl
from gpu_util import as_seen_by_gpu, check, dev, empty, host, workspace

pytestmark = pytest.mark.gpu


def _desc(d):
    return brg.ConvDesc(d.N, d.C, d.H, d.W, d.K, d.R, d.S, d.stride, d.stride, d.pad, d.pad, d.bc, d.bk)


def gpu_fwd(d, I, W, dtype=brg.F32, out=brg.F32, bias=None, act=brg.ACT_NONE, use_ws=True):
    O = empty(d.o_shape, out)
    nws = brg.brg_conv_ws_bytes(_desc(d), dtype) if use_ws else 0
    ws = workspace(nws)
    brg.brg_conv_fwd(_desc(d), dtype, out, dev(I, dtype), dev(W, dtype), O, None if bias is None else dev(bias), act, ws)
    torch.cuda.synchronize()
    return host(O)


def gpu_bwd_data(d, dO, W, dtype=brg.F32, out=brg.F32):
    dI = empty(d.i_shape, out)
    brg.brg_conv_bwd_data(_desc(d), dtype, out, dev(dO, dtype), dev(W, dtype), dI)
    torch.cuda.synchronize()
    return host(dI)


def gpu_bwd_wgt(d, I, dO, dtype=brg.F32, use_ws=False):
    dW = empty(d.w_shape)
    nws = brg.brg_conv_bwd_wgt_ws_bytes(_desc(d), dtype) if use_ws else 0
    ws = workspace(nws)
    brg.brg_conv_bwd_wgt(_desc(d), dtype, dev(I, dtype), dev(dO, dtype), dW, ws)
    torch.cuda.synchronize()
    return host(dW)


# N C H K R stride pad: every filter/stride family of the 53-layer list at reduced size, with ragged
# pixel counts (not multiples of the tile) and more than one channel block / tile
SMALL = [
    (3, 64, 14, 64, 3, 1, 1), (2, 32, 9, 48, 3, 2, 1), (3, 64, 7, 128, 1, 1, 0), (2, 128, 10, 32, 1, 2, 0),
    (2, 16, 23, 64, 7, 2, 3), (1, 16, 5, 16, 3, 1, 0), (5, 48, 7, 80, 3, 1, 1), (2, 96, 12, 16, 3, 2, 1),
]


@pytest.mark.parametrize("N,C,H,K,R,stride,pad", SMALL)
@pytest.mark.parametrize("dtype,out", [(brg.F32, brg.F32), (brg.BF16, brg.BF16), (brg.BF16, brg.F32)])
def test_conv_all_passes_small(N, C, H, K, R, stride, pad, dtype, out):
    I, W, dO = wl.conv_tensors(N, C, H, K, R, stride, pad, cfg_index=5, seed_extra=H + R, want_dO=True)
    d = orc.ConvShape(N, C, H, H, K, R, R, stride, pad)
    Is, Ws, dOs = (as_seen_by_gpu(v, dtype) for v in (I, W, dO))
    check(gpu_fwd(d, I, W, dtype, out), orc.conv_fwd(d, Is, Ws, out_bf16=out == brg.BF16), dtype, "fwd", out)
    check(gpu_bwd_data(d, dO, W, dtype, out), orc.conv_bwd_data(d, dOs, Ws, out_bf16=out == brg.BF16), dtype, "bwd-data", out)
    if out == brg.F32 or dtype == brg.F32:
        check(gpu_bwd_wgt(d, I, dO, dtype), orc.conv_bwd_wgt(d, Is, dOs), dtype, "bwd-wgt", brg.F32)


# layers large enough for the tiled bf16 kernels (channel blocks in pairs / groups of 4 or 8, feature
# tiles of 64 and 128), with and without workspace (without: the general kernel), bias + ReLU fused
BF16_TILED = [(3, 64, 14, 64, 3, 1, 1), (2, 128, 9, 192, 3, 1, 1), (3, 64, 10, 128, 1, 1, 0), (2, 128, 7, 256, 1, 1, 0),
              (2, 256, 12, 128, 1, 2, 0), (2, 64, 16, 128, 3, 2, 1), (5, 128, 7, 64, 3, 1, 1), (2, 64, 9, 64, 3, 2, 1),
              (3, 128, 13, 64, 1, 2, 0)]


@pytest.mark.parametrize("small", ["0", "1"])   # "1": the same shapes on the few-pixel kernel (divided chain with the workspace)
@pytest.mark.parametrize("N,C,H,K,R,stride,pad", BF16_TILED)
def test_conv_bf16_tiled_fwd_bwd(monkeypatch, N, C, H, K, R, stride, pad, small):
    monkeypatch.setenv("BRG_CONV_SMALL", small)
    brg.brg_tuning_reload()
    I, W, dO = wl.conv_tensors(N, C, H, K, R, stride, pad, cfg_index=5, seed_extra=C + K, want_dO=True)
    d = orc.ConvShape(N, C, H, H, K, R, R, stride, pad)
    Is, Ws, dOs = (as_seen_by_gpu(v, brg.BF16) for v in (I, W, dO))
    bias = wl.uniform(np.random.default_rng(K), (K,))
    want = orc.conv_fwd(d, Is, Ws, bias, orc.ACT_RELU, out_bf16=True)
    for use_ws in (True, False):
        got = gpu_fwd(d, I, W, brg.BF16, brg.BF16, bias=bias, act=brg.ACT_RELU, use_ws=use_ws)
        check(got, want, brg.BF16, "bf16 fwd ws=%s" % use_ws)
    check(gpu_bwd_data(d, dO, W, brg.BF16, brg.BF16), orc.conv_bwd_data(d, dOs, Ws, out_bf16=True), brg.BF16, "bf16 bwd")

# Every kernel family selects one of three epilogue copies (none / ReLU / transcendental) by a uniform
# branch: each copy with a bias, for fp32 3x3, bf16 3x3, bf16 1x1 (streaming, split reduction and
# workgroup-tiled variants) and the bf16 stem with a channel block of 4.
ACTS = [(brg.ACT_NONE, orc.ACT_NONE), (brg.ACT_RELU, orc.ACT_RELU), (brg.ACT_SIGMOID, orc.ACT_SIGMOID),
        (brg.ACT_TANH, orc.ACT_TANH)]


@pytest.mark.parametrize("gact,oact", ACTS)
@pytest.mark.parametrize("family", ["f32_3x3", "bf16_3x3", "bf16_1x1", "bf16_1x1_split", "bf16_1x1_tiled", "bf16_stem4", "bf16_small",
                                    "bf16_small_gz1"])
def test_conv_epilogue_activations(monkeypatch, family, gact, oact):
    bc = 16
    monkeypatch.setenv("BRG_CONV_SMALL", "1" if family.startswith("bf16_small") else "0")
    if family == "bf16_small_gz1":
        monkeypatch.setenv("BRG_CONV_SMALL_GZ", "1")
    if family == "f32_3x3":
        N, C, H, K, R, stride, pad, dt = 2, 32, 9, 48, 3, 1, 1, brg.F32
    elif family in ("bf16_3x3", "bf16_small", "bf16_small_gz1"):
        N, C, H, K, R, stride, pad, dt = 2, 64, 10, 80, 3, 1, 1, brg.BF16
    elif family == "bf16_stem4":
        N, C, H, K, R, stride, pad, dt, bc = 2, 3, 26, 64, 7, 2, 3, brg.BF16, 4
    else:
        N, C, H, K, R, stride, pad, dt = 2, 256, 7, 144, 1, 1, 0, brg.BF16
        if family == "bf16_1x1_split":
            monkeypatch.setenv("BRG_CONV_1X1_SPLIT", "1")
        if family == "bf16_1x1_tiled":
            monkeypatch.setenv("BRG_CONV_1X1_LDS", "1")
    brg.brg_tuning_reload()
    I, W = wl.conv_tensors(N, C, H, K, R, stride, pad, bc=bc, cfg_index=5, seed_extra=K + int(gact))
    Cp = I.shape[1] * bc
    d = orc.ConvShape(N, Cp, H, H, K, R, R, stride, pad, bc=bc) if bc == 4 else orc.ConvShape(N, Cp, H, H, K, R, R, stride, pad)
    Is, Ws = (as_seen_by_gpu(v, dt) for v in (I, W))
    bias = wl.uniform(np.random.default_rng(K + 1), (K,))
    got = gpu_fwd(d, I, W, dt, dt, bias=bias, act=gact)
    check(got, orc.conv_fwd(d, Is, Ws, bias, oact, out_bf16=dt == brg.BF16), dt, "%s act %d" % (family, gact))


# 1x1 layers in bf16 take a streaming kernel with six (feature blocks per wave, pixel groups per wave)
# variants; the knobs pin each variant on shapes with ragged pixel counts (7x7, 5x5 images), a number
# of feature blocks that does not fill the last wave, two to sixteen channel blocks, and stride 2
# (input sub-sampling forward, output placement + zero fill backward)
ONE_BY_ONE = [(2, 32, 7, 16, 1), (3, 64, 14, 272, 1), (1, 256, 5, 80, 1), (2, 96, 9, 48, 2), (4, 64, 7, 512, 1),
              (2, 128, 11, 144, 2)]


@pytest.mark.parametrize("KW,PG", [(4, 4), (2, 4), (1, 4), (4, 2), (2, 2), (1, 2), (0, 0), (-1, -1), (-2, -2), (-3, -3)])
@pytest.mark.parametrize("N,C,H,K,stride", ONE_BY_ONE + [(2, 512, 7, 64, 1), (1, 544, 5, 32, 1), (2, 256, 14, 272, 1),
                                                         (3, 160, 9, 256, 2), (5, 320, 14, 400, 1), (3, 1024, 7, 144, 1), (4, 256, 13, 128, 2)])
def test_conv1x1_bf16_streaming(monkeypatch, N, C, H, K, stride, KW, PG):
    monkeypatch.setenv("BRG_CONV_SMALL", "0")
    if KW > 0:
        monkeypatch.setenv("BRG_CONV_1X1_KW", str(KW))
        monkeypatch.setenv("BRG_CONV_1X1_PG", str(PG))
        monkeypatch.setenv("BRG_CONV_1X1_SPLIT", "0")
    elif KW == -1:
        monkeypatch.setenv("BRG_CONV_1X1_SPLIT", "1")    # the variant that splits the reduction between waves
    elif KW <= -2:                                       # the workgroup-tiled variant (C a multiple of 128, else as (0, 0))
        monkeypatch.setenv("BRG_CONV_1X1_LDS", "1")
        monkeypatch.setenv("BRG_CONV_1X1_LDS_NGW", "4" if KW == -2 else "2")
    brg.brg_tuning_reload()
    I, W, dO = wl.conv_tensors(N, C, H, K, 1, stride, 0, cfg_index=5, seed_extra=C + K + H, want_dO=True)
    d = orc.ConvShape(N, C, H, H, K, 1, 1, stride, 0)
    Is, Ws, dOs = (as_seen_by_gpu(v, brg.BF16) for v in (I, W, dO))
    bias = wl.uniform(np.random.default_rng(K), (K,))
    check(gpu_fwd(d, I, W, brg.BF16, brg.BF16, bias=bias, act=brg.ACT_RELU),
          orc.conv_fwd(d, Is, Ws, bias, orc.ACT_RELU, out_bf16=True), brg.BF16, "1x1 fwd")
    check(gpu_bwd_data(d, dO, W, brg.BF16, brg.BF16), orc.conv_bwd_data(d, dOs, Ws, out_bf16=True), brg.BF16, "1x1 bwd")


# The few-pixel kernel (feature blocks first, chain divided between the waves of a workgroup and between
# workgroups): every (feature blocks, pixel groups) variant with 1 .. 16 ranges of the chain, on 3x3 with
# padding, stride 2, 1x1 with input sub-sampling, 2 .. 128 channel blocks, ragged pixel and feature counts,
# forward (partial results in the workspace) and backward by data (one range).
@pytest.mark.parametrize("KW,PG,GZ", [(0, 0, 0), (2, 2, 1), (1, 1, 4), (2, 1, 3), (1, 2, 16), (2, 2, 5)])
@pytest.mark.parametrize("N,C,H,K,R,stride,pad", [
    (1, 64, 14, 64, 3, 1, 1), (1, 512, 7, 512, 3, 1, 1), (1, 256, 14, 256, 3, 2, 1), (1, 2048, 7, 512, 1, 1, 0),
    (2, 96, 9, 48, 1, 2, 0), (3, 32, 5, 16, 3, 1, 1), (1, 64, 28, 80, 3, 1, 1), (1, 128, 13, 48, 3, 2, 1),
    (1, 32, 6, 272, 2, 1, 0), (2, 64, 7, 32, 4, 1, 2)])
def test_conv_small_bf16_variants(monkeypatch, N, C, H, K, R, stride, pad, KW, PG, GZ):
    monkeypatch.setenv("BRG_CONV_SMALL", "1")
    if KW:
        monkeypatch.setenv("BRG_CONV_SMALL_KW", str(KW))
        monkeypatch.setenv("BRG_CONV_SMALL_PG", str(PG))
        monkeypatch.setenv("BRG_CONV_SMALL_GZ", str(GZ))
    brg.brg_tuning_reload()
    I, W, dO = wl.conv_tensors(N, C, H, K, R, stride, pad, cfg_index=5, seed_extra=C + K + H + R, want_dO=True)
    d = orc.ConvShape(N, C, H, H, K, R, R, stride, pad)
    Is, Ws, dOs = (as_seen_by_gpu(v, brg.BF16) for v in (I, W, dO))
    bias = wl.uniform(np.random.default_rng(K), (K,))
    check(gpu_fwd(d, I, W, brg.BF16, brg.BF16, bias=bias, act=brg.ACT_RELU),
          orc.conv_fwd(d, Is, Ws, bias, orc.ACT_RELU, out_bf16=True), brg.BF16, "few-pixel fwd")
    check(gpu_fwd(d, I, W, brg.BF16, brg.BF16, use_ws=False), orc.conv_fwd(d, Is, Ws, out_bf16=True), brg.BF16, "few-pixel fwd, no workspace")
    check(gpu_bwd_data(d, dO, W, brg.BF16, brg.BF16), orc.conv_bwd_data(d, dOs, Ws, out_bf16=True), brg.BF16, "few-pixel bwd")


# fp32 backward by data of strided layers: one pass of the fp32 tiled kernel per parity class of the input pixels
# (3x3 stride 2: classes with 1x1, 1x2, 2x1 and 2x2 taps; 1x1 stride 2: one class and a zero fill), on even and
# odd image sizes (classes of different sizes), ragged tiles, and a 56-pixel-wide image (the deeper halo copy plan)
@pytest.mark.parametrize("N,C,H,K,R,stride,pad", [
    (2, 64, 16, 128, 3, 2, 1), (3, 64, 9, 64, 3, 2, 1), (2, 32, 13, 64, 3, 2, 1), (2, 256, 12, 128, 1, 2, 0),
    (3, 64, 7, 32, 1, 2, 0), (2, 32, 56, 32, 3, 2, 1), (1, 128, 28, 64, 3, 2, 1)])
def test_conv_fp32_strided_backward_tiled(N, C, H, K, R, stride, pad):
    I, W, dO = wl.conv_tensors(N, C, H, K, R, stride, pad, cfg_index=5, seed_extra=C + H, want_dO=True)
    d = orc.ConvShape(N, C, H, H, K, R, R, stride, pad)
    check(gpu_bwd_data(d, dO, W), orc.conv_bwd_data(d, dO, W), brg.F32, "fp32 strided bwd-data")
    check(gpu_fwd(d, I, W), orc.conv_fwd(d, I, W), brg.F32, "fp32 strided fwd")


def test_conv_bf16_stem_tiled():
    """7x7 stride-2 stem, C=3 zero-padded to one block: forward pairs adjacent taps inside an MFMA,
    backward by data runs as four parity classes with 3x3 .. 4x4 taps."""
    I, W, dO = wl.conv_tensors(2, 3, 40, 64, 7, 2, 3, cfg_index=5, seed_extra=77, want_dO=True)
    d = orc.ConvShape(2, 16, 40, 40, 64, 7, 7, 2, 3)
    Is, Ws, dOs = (as_seen_by_gpu(v, brg.BF16) for v in (I, W, dO))
    check(gpu_fwd(d, I, W, brg.BF16, brg.BF16), orc.conv_fwd(d, Is, Ws, out_bf16=True), brg.BF16, "stem fwd")
    check(gpu_bwd_data(d, dO, W, brg.BF16, brg.BF16), orc.conv_bwd_data(d, dOs, Ws, out_bf16=True), brg.BF16, "stem bwd")


# The stem with its 3 channels stored as ONE channel block of 4 (bc = 4): one MFMA per filter row.
# Ragged widths (Q not a multiple of 16, P not a multiple of the 4-row tile), fewer than 4 feature blocks,
# with the packed-weights workspace and without it.
@pytest.mark.parametrize("N,H,K", [(2, 40, 64), (3, 38, 32), (1, 224, 64), (2, 23, 80), (3, 50, 64)])
@pytest.mark.parametrize("use_ws", [True, False])
def test_conv_stem_channel_block_of_4(N, H, K, use_ws):
    I, W, dO = wl.conv_tensors(N, 3, H, K, 7, 2, 3, bc=4, cfg_index=5, seed_extra=H + K, want_dO=True)
    d = orc.ConvShape(N, 4, H, H, K, 7, 7, 2, 3, bc=4)
    Is, Ws = (as_seen_by_gpu(v, brg.BF16) for v in (I, W))
    bias = wl.uniform(np.random.default_rng(K), (K,))
    got = gpu_fwd(d, I, W, brg.BF16, brg.BF16, bias=bias, act=brg.ACT_RELU, use_ws=use_ws)
    check(got, orc.conv_fwd(d, Is, Ws, bias, orc.ACT_RELU, out_bf16=True), brg.BF16, "stem (bc=4) fwd")
    if use_ws:
        dOs = as_seen_by_gpu(dO, brg.BF16)
        check(gpu_bwd_data(d, dO, W, brg.BF16, brg.BF16), orc.conv_bwd_data(d, dOs, Ws, out_bf16=True), brg.BF16,
              "stem (bc=4) bwd-data")


def test_conv_bias_relu_epilogue():
    I, W = wl.conv_tensors(2, 32, 9, 32, 3, 1, 1, cfg_index=5, seed_extra=99)
    d = orc.ConvShape(2, 32, 9, 9, 32, 3, 3, 1, 1)
    bias = wl.uniform(np.random.default_rng(3), (32,))
    got = gpu_fwd(d, I, W, bias=bias, act=brg.ACT_RELU)
    check(got, orc.conv_fwd(d, I, W, bias, orc.ACT_RELU), brg.F32, "bias+relu")
    check(gpu_fwd(d, I, W, bias=bias, act=brg.ACT_RELU, use_ws=False), orc.conv_fwd(d, I, W, bias, orc.ACT_RELU), brg.F32,
          "bias+relu, weights as stored")
    assert (got == 0).mean() > 0.2


def test_conv_stem_padded_channels():
    """7x7 stride-2 stem with C=3 stored zero-padded to one 16-channel block."""
    I, W = wl.conv_tensors(2, 3, 32, 64, 7, 2, 3, cfg_index=5, seed_extra=7)
    d = orc.ConvShape(2, 16, 32, 32, 64, 7, 7, 2, 3)
    check(gpu_fwd(d, I, W), orc.conv_fwd(d, I, W), brg.F32, "stem fwd")


def test_conv_bwd_data_untouched_pixels_are_zero():
    I, W, dO = wl.conv_tensors(1, 16, 8, 16, 1, 2, 0, cfg_index=5, seed_extra=11, want_dO=True)
    d = orc.ConvShape(1, 16, 8, 8, 16, 1, 1, 2, 0)
    dI = gpu_bwd_data(d, dO, W)
    assert np.all(dI[:, :, 1::2, :, :] == 0) and np.all(dI[:, :, :, 1::2, :] == 0)


def _wgt_widen(d):
    """The weight gradient sums N*P*Q products per element in fp32: beyond 4096 terms the rounding error of
    the sum grows like the square root of the length, and the element-wise bound is widened by that factor."""
    return max(1.0, (d.N * d.P * d.Q / 4096.0) ** 0.5)


def _sample_idx(rng, dims, n):
    idx = np.stack([rng.integers(0, hi, n) for hi in dims], axis=1)
    corners = [[0] * 4, [hi - 1 for hi in dims], [dims[0] - 1, 0, dims[2] - 1, 0], [0, dims[1] - 1, 0, dims[3] - 1]]
    return np.concatenate([np.array(corners), idx]).astype(np.int64)


def test_config2_full_size_fp32():
    """N=64, 64->64 channels, 56x56, 3x3 stride 1 pad 1: first and last image element by element,
    plus sampled outputs over the whole tensor."""
    I, W = wl.cfg2_conv()
    d = orc.ConvShape(64, 64, 56, 56, 64, 3, 3, 1, 1)
    got = gpu_fwd(d, I, W)              # (with the workspace, as the benchmark runs it)
    assert np.array_equal(got, gpu_fwd(d, I, W, use_ws=False)), "the two weight paths sum in the same order"
    d1 = orc.ConvShape(1, 64, 56, 56, 64, 3, 3, 1, 1)
    for n in (0, 63):
        check(got[n:n + 1], orc.conv_fwd(d1, I[n:n + 1], W), brg.F32, "image %d" % n)
    idx = _sample_idx(np.random.default_rng(2), (64, 64, 56, 56), 20000)
    want = orc.conv_fwd_sample(d, I, W, idx)
    smp = got[idx[:, 0], idx[:, 1] // 16, idx[:, 2], idx[:, 3], idx[:, 1] % 16]
    check(smp, want, brg.F32, "sampled")


# config 5 at full size (N = 64, bf16 in and out, with the workspaces: the launch configuration the benchmark
# times): EVERY one of the 23 distinct layer shapes, the 3-channel stem stored as one channel block of 4 as the
# benchmark stores it (and once more as a block of 16).  The whole output must be finite (buffers start as NaN, so
# an unwritten region shows); outputs sampled over the whole tensor (corners included) are compared with the oracle.
CFG5_NAMES = [l.name for l in wl.resnet50_v15_layers()]


def _cfg5_layer(name, N, bc_stem=4):
    L = [l for l in wl.resnet50_v15_layers() if l.name == name.replace("_bc16", "")][0]
    bc = (16 if name.endswith("_bc16") else bc_stem) if L.C < 16 else 16
    I, W, dO = wl.conv_tensors(N, L.C, L.H, L.K, L.R, L.stride, L.pad, bc=bc, cfg_index=5, want_dO=True)
    Cp = I.shape[1] * bc
    d = orc.ConvShape(N, Cp, L.H, L.H, L.K, L.R, L.R, L.stride, L.pad, bc=bc)
    return L, d, I, W, dO


@pytest.mark.parametrize("name", CFG5_NAMES + ["stem_bc16"])
def test_config5_full_size_bf16_sampled(name):
    N = 64
    L, d, I, W, dO = _cfg5_layer(name, N)
    bc = d.bc
    Is, Ws, dOs = (as_seen_by_gpu(v, brg.BF16) for v in (I, W, dO))
    rng = np.random.default_rng(L.H + L.K)
    got = gpu_fwd(d, I, W, brg.BF16, brg.BF16)
    assert np.isfinite(got).all(), name + ": forward left part of the output unwritten or non-finite"
    idx = _sample_idx(rng, (N, L.K, d.P, d.Q), 4000)
    smp = got[idx[:, 0], idx[:, 1] // 16, idx[:, 2], idx[:, 3], idx[:, 1] % 16]
    check(smp, orc.conv_fwd_sample(d, Is, Ws, idx, out_bf16=True), brg.BF16, name + " fwd sampled")
    del got
    got = gpu_bwd_data(d, dO, W, brg.BF16, brg.BF16)
    assert np.isfinite(got).all(), name + ": backward by data left part of the output unwritten or non-finite"
    idx = _sample_idx(rng, (N, d.C, L.H, L.H), 4000)
    smp = got[idx[:, 0], idx[:, 1] // bc, idx[:, 2], idx[:, 3], idx[:, 1] % bc]
    check(smp, orc.conv_bwd_data_sample(d, dOs, Ws, idx, out_bf16=True), brg.BF16, name + " bwd-data sampled")


# Inference shapes (minibatch 1, the workload of the paper's inference experiment, section 4.3) and the
# paper's own training minibatch per socket (28, section 4.1.2): every distinct ResNet-50 layer, bf16 in and out
@pytest.mark.parametrize("N", [1, 28])
def test_resnet50_layers_small_minibatch_bf16(N):
    rng = np.random.default_rng(1000 + N)
    for L in wl.resnet50_v15_layers():
        bc = 4 if L.C == 3 else 16
        I, W, dO = wl.conv_tensors(N, L.C, L.H, L.K, L.R, L.stride, L.pad, bc=bc, cfg_index=5, want_dO=True)
        Cp = I.shape[1] * bc
        d = orc.ConvShape(N, Cp, L.H, L.H, L.K, L.R, L.R, L.stride, L.pad, bc=bc)
        P = (L.H + 2 * L.pad - L.R) // L.stride + 1
        Is, Ws, dOs = (as_seen_by_gpu(v, brg.BF16) for v in (I, W, dO))
        got = gpu_fwd(d, I, W, brg.BF16, brg.BF16)
        assert np.isfinite(got).all(), L.name
        if N == 1:
            check(got, orc.conv_fwd(d, Is, Ws, out_bf16=True), brg.BF16, "%s N=1 fwd" % L.name)
        else:
            idx = _sample_idx(rng, (N, L.K, P, P), 1500)
            smp = got[idx[:, 0], idx[:, 1] // 16, idx[:, 2], idx[:, 3], idx[:, 1] % 16]
            check(smp, orc.conv_fwd_sample(d, Is, Ws, idx, out_bf16=True), brg.BF16, "%s N=%d fwd sampled" % (L.name, N))
        del got
        got = gpu_bwd_data(d, dO, W, brg.BF16, brg.BF16)
        idx = _sample_idx(rng, (N, Cp, L.H, L.H), 1500)
        smp = got[idx[:, 0], idx[:, 1] // bc, idx[:, 2], idx[:, 3], idx[:, 1] % bc]
        check(smp, orc.conv_bwd_data_sample(d, dOs, Ws, idx, out_bf16=True), brg.BF16,
              "%s N=%d bwd-data sampled" % (L.name, N))
        del got


# Weight gradient (the UPD pass of section 3.2) of bf16 layers on the tuned kernel: pixel ranges summed through
# the workspace.  Shapes: ragged images (196 and 49 pixels), one range only, both wave-tile sizes of the 1x1
# kernel, stride-2 1x1; 3x3 with padding 1 on 6 to 56 pixel wide images (borders masked per lane, windows of 46
# to 146 pixels); 3x3 stride 2 (phase planes) with even and odd image sizes.
@pytest.mark.parametrize("N,C,H,K,R,stride", [
    (4, 64, 14, 128, 1, 1), (2, 128, 8, 128, 1, 1), (3, 256, 7, 512, 1, 1), (2, 512, 7, 512, 1, 1), (16, 64, 28, 256, 1, 1),
    (4, 128, 14, 256, 1, 2), (2, 64, 28, 128, 1, 2), (3, 64, 13, 64, 1, 2),
    (4, 64, 14, 64, 3, 1), (2, 64, 8, 128, 3, 1), (3, 128, 7, 64, 3, 1), (2, 64, 56, 64, 3, 1), (16, 64, 28, 64, 3, 1),
    (1, 64, 6, 64, 3, 1),
    (4, 64, 14, 64, 3, 2), (2, 64, 28, 128, 3, 2), (2, 128, 56, 64, 3, 2), (3, 64, 13, 64, 3, 2), (1, 64, 15, 64, 3, 2)])
@pytest.mark.parametrize("dtype", [brg.BF16, brg.F32])
def test_conv_bwd_wgt_bf16_tuned(N, C, H, K, R, stride, dtype):
    """(fp32: the same shapes on the fp32 forms of the kernels)"""
    pad = (R - 1) // 2
    I, W, dO = wl.conv_tensors(N, C, H, K, R, stride, pad, cfg_index=5, seed_extra=N + H, want_dO=True)
    d = orc.ConvShape(N, C, H, H, K, R, R, stride, pad)
    assert brg.brg_conv_bwd_wgt_ws_bytes(_desc(d), dtype) >= 0
    Is, dOs = (as_seen_by_gpu(v, dtype) for v in (I, dO))
    want = orc.conv_bwd_wgt(d, Is, dOs)
    check(gpu_bwd_wgt(d, I, dO, dtype, use_ws=True), want, dtype, "bwd-wgt (workspace)", brg.F32, widen=_wgt_widen(d))
    check(gpu_bwd_wgt(d, I, dO, dtype), want, dtype, "bwd-wgt (no workspace)", brg.F32, widen=_wgt_widen(d))


# weight gradient at full size (N = 64, with the workspace: the launch configuration of the benchmark's sweep):
# every one of the 23 layer shapes (the stem as a channel block of 4), the whole result element by element
@pytest.mark.parametrize("name", CFG5_NAMES)
def test_config5_full_size_weight_gradient_bf16(name):
    N = 64
    L, d, I, W, dO = _cfg5_layer(name, N)
    assert brg.brg_conv_bwd_wgt_ws_bytes(_desc(d), brg.BF16) > 0, "the tuned kernel should apply to this layer"
    Is, dOs = (as_seen_by_gpu(v, brg.BF16) for v in (I, dO))
    check(gpu_bwd_wgt(d, I, dO, brg.BF16, use_ws=True), orc.conv_bwd_wgt(d, Is, dOs), brg.BF16, name + " bwd-wgt",
          brg.F32, widen=_wgt_widen(d))


@pytest.mark.parametrize("N,H,K", [(2, 64, 64), (1, 70, 128), (3, 100, 64), (64, 224, 64)])
def test_conv_bwd_wgt_bf16_stem_channel_block_of_4(N, H, K):
    """Weight gradient of the 7x7 stride-2 padding-3 stem with the 3 channels stored as one block of 4."""
    I, W, dO = wl.conv_tensors(N, 3, H, K, 7, 2, 3, bc=4, cfg_index=5, seed_extra=H, want_dO=True)
    d = orc.ConvShape(N, 4, H, H, K, 7, 7, 2, 3, bc=4)
    Is, dOs = (as_seen_by_gpu(v, brg.BF16) for v in (I, dO))
    got = gpu_bwd_wgt(d, I, dO, brg.BF16, use_ws=True)
    check(got, orc.conv_bwd_wgt(d, Is, dOs), brg.BF16, "stem bwd-wgt", brg.F32, widen=_wgt_widen(d))
    assert np.all(got[:, :, :, :, 3, :] == 0), "the pad channel of the block has no gradient"


# images that are not square (the generators above only make square ones): every pass, fp32 and bf16, and the
# tuned weight gradient with its workspace
@pytest.mark.parametrize("H,W,R,stride", [(9, 14, 3, 1), (14, 9, 1, 1), (12, 20, 3, 2), (16, 10, 1, 2), (7, 30, 3, 1)])
@pytest.mark.parametrize("dtype", [brg.F32, brg.BF16])
def test_conv_rectangular_images(H, W, R, stride, dtype):
    N, C, K = 3, 64, 128
    pad = (R - 1) // 2
    rng = np.random.default_rng(H * 100 + W)
    d = orc.ConvShape(N, C, H, W, K, R, R, stride, pad)
    I = wl.uniform(rng, d.i_shape)
    Wt = wl.normal(rng, d.w_shape, (2.0 / (C * R * R)) ** 0.5)
    dO = wl.uniform(rng, d.o_shape)
    Is, Ws, dOs = (as_seen_by_gpu(v, dtype) for v in (I, Wt, dO))
    bf = dtype == brg.BF16
    check(gpu_fwd(d, I, Wt, dtype, dtype), orc.conv_fwd(d, Is, Ws, out_bf16=bf), dtype, "fwd")
    check(gpu_bwd_data(d, dO, Wt, dtype, dtype), orc.conv_bwd_data(d, dOs, Ws, out_bf16=bf), dtype, "bwd-data")
    check(gpu_bwd_wgt(d, I, dO, dtype, use_ws=True), orc.conv_bwd_wgt(d, Is, dOs), dtype, "bwd-wgt", brg.F32)


@pytest.mark.parametrize("N,C,H,K,R,stride,pad", [(2, 64, 14, 64, 3, 1, 1), (2, 128, 10, 32, 1, 2, 0), (3, 64, 9, 64, 3, 2, 1)])
@pytest.mark.parametrize("dtype", [brg.F32, brg.BF16])
def test_conv_general_kernel_forced(monkeypatch, N, C, H, K, R, stride, pad, dtype):
    """BRG_CONV_GENERAL / BRG_CONV_WGT_GENERAL: shapes that normally take the tuned kernels, on the general one."""
    monkeypatch.setenv("BRG_CONV_GENERAL", "1")
    monkeypatch.setenv("BRG_CONV_WGT_GENERAL", "1")
    brg.brg_tuning_reload()
    I, W, dO = wl.conv_tensors(N, C, H, K, R, stride, pad, cfg_index=5, seed_extra=3 * H + R, want_dO=True)
    d = orc.ConvShape(N, C, H, H, K, R, R, stride, pad)
    Is, Ws, dOs = (as_seen_by_gpu(v, dtype) for v in (I, W, dO))
    bf = dtype == brg.BF16
    check(gpu_fwd(d, I, W, dtype, dtype), orc.conv_fwd(d, Is, Ws, out_bf16=bf), dtype, "fwd (general)")
    check(gpu_bwd_data(d, dO, W, dtype, dtype), orc.conv_bwd_data(d, dOs, Ws, out_bf16=bf), dtype, "bwd-data (general)")
    check(gpu_bwd_wgt(d, I, dO, dtype, use_ws=True), orc.conv_bwd_wgt(d, Is, dOs), dtype, "bwd-wgt (general)", brg.F32)


# Seeded random shapes: the planners choose between a dozen kernels by thresholds on N, C, K, the image size, the
# filter and the stride; forty random layers per input type (rectangular images, any multiple of 16 channels up to
# 192, filters 1..4 with any padding below the filter, stride 1..2, with and without a workspace) go through
# whatever each call picks, all three passes, against the oracle.
def _random_layers(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        N = int(rng.integers(1, 5))
        C, K = 16 * int(rng.integers(1, 13)), 16 * int(rng.integers(1, 13))
        H, W = int(rng.integers(3, 34)), int(rng.integers(3, 34))
        R, S = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        if rng.random() < 0.6:
            S = R
        stride = int(rng.integers(1, 3))
        pad = int(rng.integers(0, min(R, S)))
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        out.append((N, C, H, W, K, R, S, stride, pad, bool(rng.random() < 0.7)))
    return out


@pytest.mark.parametrize("dtype", [brg.BF16, brg.F32])
@pytest.mark.parametrize("chunk", range(4))
def test_conv_random_layers(dtype, chunk):
    out = dtype
    for (N, C, H, W, K, R, S, stride, pad, use_ws) in _random_layers(4242 + chunk, 10):
        what = "N%d C%d %dx%d K%d %dx%d s%d p%d ws%d" % (N, C, H, W, K, R, S, stride, pad, use_ws)
        d = orc.ConvShape(N, C, H, W, K, R, S, stride, pad)
        rng = np.random.default_rng(N * 1000 + C + K + H)
        I, Wt, dO = wl.uniform(rng, d.i_shape), wl.normal(rng, d.w_shape, (2.0 / (C * R * S)) ** 0.5), wl.uniform(rng, d.o_shape)
        Is, Ws, dOs = (as_seen_by_gpu(v, dtype) for v in (I, Wt, dO))
        bias = wl.uniform(rng, (K,))
        bf = dtype == brg.BF16
        check(gpu_fwd(d, I, Wt, dtype, out, bias=bias, act=brg.ACT_RELU, use_ws=use_ws),
              orc.conv_fwd(d, Is, Ws, bias, orc.ACT_RELU, out_bf16=bf), dtype, what + " fwd", out)
        check(gpu_bwd_data(d, dO, Wt, dtype, out), orc.conv_bwd_data(d, dOs, Ws, out_bf16=bf), dtype, what + " bwd-data", out)
        check(gpu_bwd_wgt(d, I, dO, dtype, use_ws=use_ws), orc.conv_bwd_wgt(d, Is, dOs), dtype, what + " bwd-wgt", brg.F32,
              widen=_wgt_widen(d))
