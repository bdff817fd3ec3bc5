"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no
memset nodes), so its calls can be captured into a HIP graph.  Replays are checked against the eager
result, several times, with eager work and synchronisations in between."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_1906_06440_amd as brg
import workloads as wl
from gpu_util import as_seen_by_gpu, check, dev, empty, host, workspace

pytestmark = pytest.mark.gpu


def test_graph_replay_matches_eager_conv_and_fc():
    N, C, H, K = 2, 64, 14, 128
    I, W, dO = wl.conv_tensors(N, C, H, K, 1, 1, 0, cfg_index=5, seed_extra=5, want_dO=True)
    I3, W3 = wl.conv_tensors(N, C, H, C, 3, 1, 1, cfg_index=5, seed_extra=6)
    d1 = brg.ConvDesc(N, C, H, H, K, 1, 1, 1, 1, 0, 0, 16, 16)
    d3 = brg.ConvDesc(N, C, H, H, C, 3, 3, 1, 1, 1, 1, 16, 16)
    dI, dW, dI3, dW3 = dev(I, brg.BF16), dev(W, brg.BF16), dev(I3, brg.BF16), dev(W3, brg.BF16)
    O1 = empty((N, K // 16, H, H, 16), brg.BF16)
    O3 = empty((N, C // 16, H, H, 16), brg.BF16)
    G1 = empty((N, C // 16, H, H, 16), brg.BF16)
    ddO = dev(dO, brg.BF16)
    ws1 = workspace(max(16, brg.brg_conv_ws_bytes(d1, brg.BF16)))
    ws3 = workspace(max(16, brg.brg_conv_ws_bytes(d3, brg.BF16)))
    X0, Ws, bs, _ = wl.cfg3_mlp()
    fd = brg.FcDesc(1024, 1024, 1024, 64, 64, 64)
    X, Wf, bf, Y = dev(X0), dev(Ws[0]), dev(bs[0]), torch.empty((16, 16, 64, 64), device="cuda")
    dYf = dev(wl.cfg3_mlp()[3])
    # weight gradients with their workspaces (partial sums of the pixel ranges, then the range sum)
    I16, _, dO16 = wl.conv_tensors(16, C, 28, K, 1, 1, 0, cfg_index=5, seed_extra=7, want_dO=True)
    I16b, _, dO16b = wl.conv_tensors(16, C, 28, C, 3, 1, 1, cfg_index=5, seed_extra=8, want_dO=True)
    dw1 = brg.ConvDesc(16, C, 28, 28, K, 1, 1, 1, 1, 0, 0, 16, 16)
    dw3 = brg.ConvDesc(16, C, 28, 28, C, 3, 3, 1, 1, 1, 1, 16, 16)
    gI16, gO16, gI16b, gO16b = dev(I16, brg.BF16), dev(dO16, brg.BF16), dev(I16b, brg.BF16), dev(dO16b, brg.BF16)
    gW1 = torch.empty((K // 16, C // 16, 1, 1, 16, 16), device="cuda")
    gW3 = torch.empty((C // 16, C // 16, 3, 3, 16, 16), device="cuda")
    wsw1 = workspace(max(16, brg.brg_conv_bwd_wgt_ws_bytes(dw1, brg.BF16)))
    wsw3 = workspace(max(16, brg.brg_conv_bwd_wgt_ws_bytes(dw3, brg.BF16)))
    assert wsw1.numel() > 16 and wsw3.numel() > 16, "these shapes should split the pixel range"
    gX, gW, gb = torch.empty_like(X), torch.empty_like(Wf), torch.empty(1024, device="cuda")

    def work():
        brg.brg_conv_fwd(d1, brg.BF16, brg.BF16, dI, dW, O1, None, brg.ACT_NONE, ws1)
        brg.brg_conv_fwd(d3, brg.BF16, brg.BF16, dI3, dW3, O3, None, brg.ACT_RELU, ws3)
        brg.brg_conv_bwd_data(d1, brg.BF16, brg.BF16, ddO, dW, G1)
        brg.brg_fc_fwd(fd, brg.F32, brg.F32, X, Wf, bf, brg.ACT_RELU, Y)
        # fused backward launch (by data + weights + bias) with the ReLU mask and the producer mask
        brg.brg_fc_bwd_chain(fd, brg.F32, dYf, Y, X, Wf, brg.ACT_RELU, brg.ACT_RELU, gX, gW, gb)
        brg.brg_conv_bwd_wgt(dw1, brg.BF16, gI16, gO16, gW1, wsw1)
        brg.brg_conv_bwd_wgt(dw3, brg.BF16, gI16b, gO16b, gW3, wsw3)

    work()                                  # eager: sets per-kernel attributes, gives the expected values
    torch.cuda.synchronize()
    outs = (O1, O3, G1, Y, gX, gW, gb, gW1, gW3)
    want = [host(t).copy() for t in outs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        work()
    for rep in range(3):
        for t in outs:
            t.zero_()                       # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, w, name in zip(outs, want, ("1x1 fwd", "3x3 fwd", "1x1 bwd", "fc fwd", "fc dX", "fc dW", "fc db", "1x1 wgt", "3x3 wgt")):
            assert np.array_equal(host(got), w), "replay %d differs from the eager result: %s" % (rep, name)


def test_graph_replay_matches_eager_lstm_forward_and_backward():
    """The LSTM layer (resident forward kernel with its barrier words, backward pass with ~200 launches) replayed
    from a HIP graph: every replay equals the eager result."""
    T, N, Cc, K = 6, 64, 128, 256
    x, W4, R4, b4 = wl.cfg4_lstm(T, N, Cc, K, 64, 64, with_bias=True, seed_extra=3)
    desc = brg.LstmDesc(T, N, Cc, K, 16, 64, 64)
    gx, gW4, gR4, gb4 = dev(x), dev(W4), dev(R4), dev(b4)
    h, s, g = empty((T, N, K)), empty((T, N, K)), empty((4, T, N, K))
    dh = dev(wl.uniform(np.random.default_rng(9), (T, N, K)))
    dx, dW, dR, db = empty((T, N, Cc)), empty(W4.shape), empty(R4.shape), empty((4, K))
    ws_f = workspace(64)
    ws_b = workspace(max(16, brg.brg_lstm_bwd_ws_bytes(desc)))

    def work():
        brg.brg_lstm_fwd(desc, brg.F32, gx, gW4, gR4, gb4, None, None, h, s, g, ws_f)
        brg.brg_lstm_bwd(desc, brg.F32, gx, gW4, gR4, None, None, h, s, g, dh, None, dx, dW, dR, db, None, None, ws_b)

    work()
    torch.cuda.synchronize()
    outs = (h, s, dx, dW, dR, db)
    want = [host(t).copy() for t in outs]
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr):
        work()
    for rep in range(3):
        for t in outs:
            t.zero_()
        torch.cuda.synchronize()
        gr.replay()
        torch.cuda.synchronize()
        assert int(ws_f[:8].view(torch.int32)[1].item()) == 0, "recurrent kernel reported a barrier time-out"
        for got, w, name in zip(outs, want, ("h", "s", "dx", "dW", "dR", "db")):
            assert np.array_equal(host(got), w), "replay %d differs from the eager result: %s" % (rep, name)
