#!/usr/bin/env python3
"""Benchmark of the batch-reduce GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg3|cfg4|cfg5|cfg1|cfg3_bf16|cfg4_bwd]
                    [--batch N] [--no-cpu-baseline] [--no-others]

A step is one pass of the selected workload (default: the configuration the headline metric is quoted
on, the ResNet-50 3x3 convolution layer, forward, fp32, N=64) over synthetic inputs that are already
resident in HBM.  Prints ONE JSON line: metric/value are GFLOP/s (algorithmic flops: 2 per
multiply-add of the definition), `roofline` prices the kernel against the MI355X matrix-core
peak for its dtype, `cpu_baseline` is the CPU oracle timed on a bounded sample of the same
workload on the host cores, `others` carries the remaining configurations measured the same way.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}   # MI355X dense MFMA peaks (published)

# HBM bytes per launch of the dominant kernel, from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE,
# KiB per dispatch), each scaled by what the same counter reads for a plain 256 MiB device copy
# (FETCH_SIZE reads 131084 KiB for 262144 KiB copied => x2.0; WRITE_SIZE reads 262144 => x1.0).
# The counter summaries are kept with the kernel-trace summaries of the same workloads.
MEASURED_TRAFFIC_BYTES = {
    "cfg2": int((25801.2 * 262144.0 / 131084.0 + 50176.0) * 1024),   # 104.2 MB (algorithmic: 102.9 MB)
    # per step = 4 forward launches + 4 fused backward launches (fabric traffic into the 8 XCD L2s)
    "cfg3": int(4 * ((12332.0 + 26767.9) * 262144.0 / 131084.0 + 4096.0 + 8196.0) * 1024),   # 370.6 MB (algorithmic: 151 MB)
}


def _dev(a, bf16=False):
    import numpy as np
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def _time_graph(fn, steps, warmup, prewarm_s=0.05):
    """Like _time_steps, but the K calls are captured once into a HIP graph and replayed: the library
    only enqueues kernels on the stream it is given, so a caller whose layers are shorter than the
    host-side launch cost (about 5 us per kernel) can keep the GPU fed this way.  Returns device seconds
    for the K steps."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(steps):
            fn()
    g.replay()                      # untimed replay (first replay pays the graph upload)
    torch.cuda.synchronize()
    t0 = time.perf_counter()        # untimed replays until the clocks have left the idle state (see _prewarm)
    while time.perf_counter() - t0 < prewarm_s:
        g.replay()
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3


PREWARM_S = 0.3


def _prewarm(fn, seconds=PREWARM_S):
    """Untimed: keep the GPU busy with the workload until its clocks have left the idle state.  After the
    host-side set-up the first ~20 ms of work run up to 40 % slower than the steady state (measured on the
    fp32 3x3 layer: 179, 131, 128, 128, ... us per step over consecutive 100-step chunks), so the W warm-up
    steps of a short run would otherwise end inside the ramp."""
    import torch
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()


def _time_steps(fn, steps, warmup):
    """Clock pre-warm, W untimed calls, then exactly K calls bracketed by synchronize; returns (wall
    seconds, device seconds from HIP events on the launch stream)."""
    import torch
    _prewarm(fn)
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, e0.elapsed_time(e1) * 1e-3


def _lstm_completed(ws, h):
    import torch
    torch.cuda.synchronize()
    gave_up = int(ws[:8].view(torch.int32)[1].item())
    if gave_up or not bool(torch.isfinite(h).all().item()):
        raise RuntimeError("bench.py: the resident LSTM kernel gave up at its step barrier; the timing is void")


# ------------------------------------------------------------------ workloads ----
def make_cfg1():
    import torch
    import paper_1906_06440_amd as brg
    import workloads as wl
    A, B = wl.cfg1_brgemm()
    dA, dB, dC = _dev(A), _dev(B), torch.empty((64, 64), device="cuda")
    fn = lambda: brg.brg_gemm_strided(brg.F32, brg.F32, 64, 64, 64, 64, 64, 64, dA, 4096, dB, 4096, dC, 16)
    return fn, 2.0 * 64 * 64 * 64 * 16, "f32", "cfg1: one BRGEMM, 16 x (64x64x64), fp32"


def make_cfg1_ptrs():
    """cfg1 in the address-list form of section 2 (two device arrays of 16 block pointers, scrambled order)."""
    import numpy as np
    import torch
    import paper_1906_06440_amd as brg
    import workloads as wl
    A, B = wl.cfg1_brgemm()
    dA, dB, dC = _dev(A), _dev(B), torch.empty((64, 64), device="cuda")
    perm = np.random.default_rng(1).permutation(16)
    ap = torch.tensor([dA.data_ptr() + int(i) * 4096 * 4 for i in perm], dtype=torch.int64, device="cuda")
    bp = torch.tensor([dB.data_ptr() + int(i) * 4096 * 4 for i in perm], dtype=torch.int64, device="cuda")
    fn = lambda: brg.brg_gemm(brg.F32, brg.F32, 64, 64, 64, 64, 64, 64, ap, bp, dC, 16)
    fn.keep = (dA, dB)
    return fn, 2.0 * 64 * 64 * 64 * 16, "f32", "cfg1 as an address list: one BRGEMM, 16 x (64x64x64) block pointers, fp32"


def make_cfg1_bf16():
    """cfg1's chain with bf16 blocks and fp32 result (strided form)."""
    import torch
    import paper_1906_06440_amd as brg
    import workloads as wl
    A, B = wl.cfg1_brgemm()
    dA, dB, dC = _dev(A, True), _dev(B, True), torch.empty((64, 64), device="cuda")
    fn = lambda: brg.brg_gemm_strided(brg.BF16, brg.F32, 64, 64, 64, 64, 64, 64, dA, 4096, dB, 4096, dC, 16)
    return fn, 2.0 * 64 * 64 * 64 * 16, "bf16", "cfg1 in bf16: one BRGEMM, 16 x (64x64x64), bf16 in, fp32 out"


def make_cfg2(N=64):
    import torch
    import paper_1906_06440_amd as brg
    import workloads as wl
    I, W = wl.cfg2_conv(N)
    dI, dW = _dev(I), _dev(W)
    dO = torch.empty((N, 4, 56, 56, 16), device="cuda")
    desc = brg.ConvDesc(N, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 16, 16)
    # workspace for the transposed weight blocks (written by a pre-pass inside every timed call)
    ws = torch.empty(brg.brg_conv_ws_bytes(desc, brg.F32), dtype=torch.uint8, device="cuda")
    fn = lambda: brg.brg_conv_fwd(desc, brg.F32, brg.F32, dI, dW, dO, None, brg.ACT_NONE, ws)
    flops = 2.0 * N * 64 * 64 * 9 * 56 * 56
    return fn, flops, "f32", "cfg2: ResNet-50 3x3 conv fwd, N=%d C=K=64 56x56 s1 p1, fp32, NCHW16c/KCRS16c16k" % N


def make_cfg3(N=1024):
    import torch
    import paper_1906_06440_amd as brg
    import workloads as wl
    X0, Ws, bs, dYl = wl.cfg3_mlp(N=N)
    desc = brg.FcDesc(N, 1024, 1024, 64, 64, 64)
    dWs, dbs = [_dev(w) for w in Ws], [_dev(b) for b in bs]
    acts = [_dev(X0)] + [torch.empty_like(_dev(X0)) for _ in range(4)]
    grads = [torch.empty_like(acts[0]) for _ in range(4)] + [_dev(dYl)]
    dWg = [torch.empty_like(w) for w in dWs]

    dbg = [torch.empty(1024, device="cuda") for _ in range(4)]

    def fn():
        for l in range(4):
            brg.brg_fc_fwd(desc, brg.F32, brg.F32, acts[l], dWs[l], dbs[l], brg.ACT_RELU, acts[l + 1])
        # backward chain: the ReLU backward of the producing layer is fused into each dX epilogue, so
        # only the last layer has to mask its incoming gradient; dW and db come from the same launch
        for l in reversed(range(4)):
            last = l == 3
            brg.brg_fc_bwd_chain(desc, brg.F32, grads[l + 1], acts[l + 1] if last else None, acts[l], dWs[l],
                                 brg.ACT_RELU if last else brg.ACT_NONE,
                                 brg.ACT_RELU if l > 0 else brg.ACT_NONE, grads[l], dWg[l], dbg[l])
    return fn, 12 * 2.0 * N * 1024 ** 2, "f32", "cfg3: MLP 4 x FC 1024->1024 bias+ReLU, N=%d, fwd+bwd-data+wgt, fp32, 64^3 blocks" % N


def make_cfg3_bf16(N=1024):
    """Context row: the cfg3 MLP in bf16 on 16-wide blocks (bn = 64), forward with bias + ReLU and the chained
    backward pass with the workspace that lets the masked last layer use the tuned kernels."""
    import numpy as np
    import torch
    import paper_1906_06440_amd as brg
    import workloads as wl
    X0, Ws, bs, dYl = wl.cfg3_mlp(N=N, bc=16, bk=16)
    desc = brg.FcDesc(N, 1024, 1024, 64, 16, 16)
    dWs, dbs = [_dev(w, True) for w in Ws], [_dev(b) for b in bs]
    acts = [_dev(X0, True)] + [torch.empty_like(_dev(X0, True)) for _ in range(4)]
    grads = [torch.empty_like(acts[0]) for _ in range(4)] + [_dev(dYl, True)]
    dWg = [torch.empty(w.shape, device="cuda") for w in Ws]
    dbg = [torch.empty(1024, device="cuda") for _ in range(4)]
    ws = torch.empty(N * 1024 * 2, dtype=torch.uint8, device="cuda")

    def fn():
        for l in range(4):
            brg.brg_fc_fwd(desc, brg.BF16, brg.BF16, acts[l], dWs[l], dbs[l], brg.ACT_RELU, acts[l + 1])
        for l in reversed(range(4)):
            last = l == 3
            brg.brg_fc_bwd_chain(desc, brg.BF16, grads[l + 1], acts[l + 1] if last else None, acts[l], dWs[l],
                                 brg.ACT_RELU if last else brg.ACT_NONE,
                                 brg.ACT_RELU if l > 0 else brg.ACT_NONE, grads[l], dWg[l], dbg[l], ws)
    return fn, 12 * 2.0 * N * 1024 ** 2, "bf16", "cfg3 in bf16: MLP 4 x FC 1024->1024 bias+ReLU, N=%d, fwd+bwd-data+wgt, bn=64 bc=bk=16" % N


def make_cfg4():
    import torch
    import paper_1906_06440_amd as brg
    import workloads as wl
    x, W4, R4, _ = wl.cfg4_lstm()
    dx, dW, dR = _dev(x), _dev(W4), _dev(R4)
    h, s = torch.empty((50, 64, 1024), device="cuda"), torch.empty((50, 64, 1024), device="cuda")
    g = torch.empty((4, 50, 64, 1024), device="cuda")
    desc = brg.LstmDesc(50, 64, 1024, 1024, 16, 64, 64)
    ws = torch.zeros(64, dtype=torch.uint8, device="cuda")   # grid-barrier words of the resident kernel
    fn = lambda: brg.brg_lstm_fwd(desc, brg.F32, dx, dW, dR, None, None, None, h, s, g, ws)
    # after the timed region: the resident kernel reports a barrier time-out through word 1 (and NaN-fills its outputs)
    fn.verify = lambda: _lstm_completed(ws, h)
    return fn, 50 * 2.0 * 64 * 4 * 1024 * 2048, "f32", "cfg4: LSTM fwd T=50 N=64 C=K=1024, fp32"


def make_cfg4_variant(N=64, bf16=False):
    """Context rows of the LSTM layer: the paper's own minibatch (N = 168, section 4.1.1) and bf16 operands."""
    import torch
    import paper_1906_06440_amd as brg
    import workloads as wl
    x, W4, R4, _ = wl.cfg4_lstm(50, N)
    dt = brg.BF16 if bf16 else brg.F32
    dx, dW, dR = _dev(x, bf16), _dev(W4, bf16), _dev(R4, bf16)
    h = torch.empty((50, N, 1024), device="cuda", dtype=torch.bfloat16 if bf16 else torch.float32)
    s = torch.empty((50, N, 1024), device="cuda")
    g = torch.empty((4, 50, N, 1024), device="cuda")
    desc = brg.LstmDesc(50, N, 1024, 1024, 16, 64, 64)
    ws = torch.zeros(64, dtype=torch.uint8, device="cuda")
    fn = lambda: brg.brg_lstm_fwd(desc, dt, dx, dW, dR, None, None, None, h, s, g, ws)
    fn.verify = lambda: _lstm_completed(ws, h)
    return fn, 50 * 2.0 * N * 4 * 1024 * 2048, "bf16" if bf16 else "f32", "LSTM fwd T=50 N=%d C=K=1024, %s" % (N, "bf16 operands, fp32 state" if bf16 else "fp32")


def make_cfg4_bwd():
    """Context row: backward pass of the cfg4 LSTM layer (dx, dW, dR, db from a random dh), fp32; the forward
    results it differentiates are computed once outside the timed region.  Flops: twice the forward's."""
    import torch
    import paper_1906_06440_amd as brg
    import workloads as wl
    x, W4, R4, _ = wl.cfg4_lstm()
    dx, dW, dR = _dev(x), _dev(W4), _dev(R4)
    h, s = torch.empty((50, 64, 1024), device="cuda"), torch.empty((50, 64, 1024), device="cuda")
    g = torch.empty((4, 50, 64, 1024), device="cuda")
    desc = brg.LstmDesc(50, 64, 1024, 1024, 16, 64, 64)
    ws = torch.zeros(64, dtype=torch.uint8, device="cuda")
    brg.brg_lstm_fwd(desc, brg.F32, dx, dW, dR, None, None, None, h, s, g, ws)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4)
    dh = torch.rand((50, 64, 1024), device="cuda", generator=gen) * 0.2 - 0.1
    gx, gW, gR, gb = torch.empty_like(dx), torch.empty_like(dW), torch.empty_like(dR), torch.empty((4, 1024), device="cuda")
    wsb = torch.empty(brg.brg_lstm_bwd_ws_bytes(desc), dtype=torch.uint8, device="cuda")
    fn = lambda: brg.brg_lstm_bwd(desc, brg.F32, dx, dW, dR, None, None, h, s, g, dh, None, gx, gW, gR, gb, None, None, wsb)
    return fn, 2 * 50 * 2.0 * 64 * 4 * 1024 * 2048, "f32", "cfg4 backward: LSTM bwd (dx, dW, dR, db) T=50 N=64 C=K=1024, fp32"


def make_cfg5_layers(N=64, only=None):
    """Returns [(layer, fwd_fn, bwd_fn)] for the 23 distinct ResNet-50 v1.5 shapes, bf16 in/out."""
    import torch
    import paper_1906_06440_amd as brg
    import workloads as wl
    out = []
    for L in wl.resnet50_v15_layers():
        if only and L.name not in only:
            continue
        # the 3-channel stem is stored as one channel block of 4 (8 bytes per pixel), every other layer in blocks of 16
        bc = 4 if L.C < 16 else 16
        I, W, dO = wl.conv_tensors(N, L.C, L.H, L.K, L.R, L.stride, L.pad, bc=bc, cfg_index=5, want_dO=True)
        Cp = I.shape[1] * bc
        dI, dW, ddO = _dev(I, True), _dev(W, True), _dev(dO, True)
        O = torch.empty(ddO.shape, dtype=torch.bfloat16, device="cuda")
        gI = torch.empty(dI.shape, dtype=torch.bfloat16, device="cuda")
        desc = brg.ConvDesc(N, Cp, L.H, L.H, L.K, L.R, L.R, L.stride, L.stride, L.pad, L.pad, bc, 16)
        ws = torch.empty(max(16, brg.brg_conv_ws_bytes(desc, brg.BF16)), dtype=torch.uint8, device="cuda")
        fwd = (lambda desc=desc, dI=dI, dW=dW, O=O, ws=ws: brg.brg_conv_fwd(desc, brg.BF16, brg.BF16, dI, dW, O,
                                                                            None, brg.ACT_NONE, ws))
        bwd = (lambda desc=desc, ddO=ddO, dW=dW, gI=gI: brg.brg_conv_bwd_data(desc, brg.BF16, brg.BF16, ddO, dW, gI))
        # weight gradient (fp32 result), with the workspace for the partial sums of the pixel ranges
        gW = torch.empty(dW.shape, dtype=torch.float32, device="cuda")
        wws = torch.empty(max(16, brg.brg_conv_bwd_wgt_ws_bytes(desc, brg.BF16)), dtype=torch.uint8, device="cuda")
        upd = (lambda desc=desc, dI=dI, ddO=ddO, gW=gW, wws=wws: brg.brg_conv_bwd_wgt(desc, brg.BF16, dI, ddO, gW, wws))
        out.append((L, fwd, bwd, upd))
    return out


def run_cfg5(steps, warmup, N=64, use_graph=True, with_upd=False, only=None):
    """Weighted efficiency (sum n_i F_i) / (sum n_i t_i) over the 53 layers, fwd and bwd-data (and, on request,
    the weight gradient).  Each layer's K timed calls are replayed from one
    HIP graph (see _time_graph) unless use_graph is False."""
    res = {}
    layers = make_cfg5_layers(N, only)
    for name, sel in (("fwd", 1), ("bwd_data", 2)) + ((("bwd_wgt", 3),) if with_upd else ()):
        F = T = 0.0
        per = []
        for tup in layers:
            L = tup[0]
            if tup[sel] is None:
                continue
            st = steps
            if sel == 3:   # layers without a tuned weight-gradient kernel run for milliseconds: fewer calls
                tup[sel]()
                import torch
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                tup[sel]()
                torch.cuda.synchronize()
                if time.perf_counter() - t0 > 1e-3:
                    st = 2
            dev_s = _time_graph(tup[sel], st, min(warmup, st)) if use_graph else _time_steps(tup[sel], st, min(warmup, st))[1]
            t = dev_s / st
            F += L.count * L.flops(N)
            T += L.count * t
            per.append({"layer": L.name, "us": round(t * 1e6, 1), "tflops": round(L.flops(N) / t / 1e12, 2)})
        res[name] = {"weighted_tflops": round(F / T / 1e12, 2), "total_ms_53_layers": round(T * 1e3, 3),
                     "frac_of_bf16_peak": round(F / T / 1e12 / PEAK_TFLOPS["bf16"], 4), "layers": per}
    return res


MAKERS = {"cfg4_bf16": lambda: make_cfg4_variant(64, True), "cfg4_n168": lambda: make_cfg4_variant(168, False),
          "cfg4_n168_bf16": lambda: make_cfg4_variant(168, True), "cfg1": make_cfg1, "cfg1_ptrs": make_cfg1_ptrs, "cfg1_bf16": make_cfg1_bf16, "cfg2": make_cfg2, "cfg3": make_cfg3, "cfg4": make_cfg4, "cfg3_bf16": make_cfg3_bf16, "cfg4_bwd": make_cfg4_bwd}


def cpu_baseline_cfg2():
    """The oracle (as it stands) on a bounded sample of the cfg2 workload: the first images."""
    import oracle as orc
    import workloads as wl
    n = 8
    I, W = wl.cfg2_conv(n)
    d = orc.ConvShape(n, 64, 56, 56, 64, 3, 3, 1, 1)
    orc.conv_fwd(orc.ConvShape(1, 64, 56, 56, 64, 3, 3, 1, 1), I[:1], W)   # warm the library
    t0 = time.perf_counter()
    orc.conv_fwd(d, I, W)
    dt = time.perf_counter() - t0
    if dt < 5.0:   # scale the sample towards ~10 s of CPU work
        n2 = int(min(64, max(n, n * 10.0 / dt)))
        I, W = wl.cfg2_conv(n2)
        d = orc.ConvShape(n2, 64, 56, 56, 64, 3, 3, 1, 1)
        t0 = time.perf_counter()
        orc.conv_fwd(d, I, W)
        dt = time.perf_counter() - t0
        n = n2
    reps = 1
    if dt < 8.0:   # still short (many host cores): repeat the same sample until about 10 s of CPU work are timed
        reps = int(min(20, max(2, 10.0 / dt)))
        t0 = time.perf_counter()
        for _ in range(reps):
            orc.conv_fwd(d, I, W)
        dt = (time.perf_counter() - t0) / reps
    flops = 2.0 * n * 64 * 64 * 9 * 56 * 56
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": round(flops / dt / 1e9, 2), "unit": "GFLOP/s", "cores": cores, "kind": "oracle",
            "sample": "conv fwd of the first %d of 64 images of cfg2, %d run(s) of %.1f s" % (n, reps, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg1_ptrs", "cfg1_bf16", "cfg2", "cfg3", "cfg4", "cfg5", "cfg3_bf16", "cfg4_bwd", "cfg4_bf16", "cfg4_n168",
                             "cfg4_n168_bf16", "copy"])
    ap.add_argument("--batch", type=int, default=None,
                    help="minibatch of cfg2 / cfg3 / cfg5 instead of the configured one (context rows: the paper's own "
                         "28 / 1344, inference at 1); such a line carries no others and no cpu_baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="cfg5: time eager launches instead of a HIP graph replay")
    ap.add_argument("--upd", action="store_true", help="cfg5: also time the weight gradient")
    ap.add_argument("--layers", default=None, help="cfg5: comma-separated layer names to run instead of all 23 shapes")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.batch is not None:
        if args.workload not in ("cfg2", "cfg3", "cfg5") or args.batch < 1 or (args.workload == "cfg3" and args.batch % 64):
            print("bench.py: --batch applies to cfg2, cfg3 (a multiple of 64) and cfg5", file=sys.stderr)
            sys.exit(2)
        args.no_others = args.no_cpu_baseline = True

    import torch
    import paper_1906_06440_amd as brg
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    brg.load()

    if args.workload == "copy":
        # calibration run for the HBM-traffic counters: a plain device-to-device copy of known size
        n = 64 << 20
        src, dst = torch.ones(n, device="cuda"), torch.empty(n, device="cuda")
        _, dev_s = _time_steps(lambda: dst.copy_(src), args.steps, args.warmup)
        print(json.dumps({"workload": "copy: %d MiB fp32 device-to-device (reads and writes %d bytes each)"
                          % (4 * n >> 20, 4 * n), "us_per_launch": round(dev_s / args.steps * 1e6, 2),
                          "GBps_read_plus_write": round(8.0 * n / (dev_s / args.steps) / 1e9, 1)}))
        return

    if args.workload == "cfg5":
        nb = args.batch or 64
        r5 = run_cfg5(max(3, args.steps // 10), max(1, args.warmup // 5), N=nb, use_graph=not args.no_graph, with_upd=args.upd,
                      only=args.layers.split(",") if args.layers else None)
        tf = r5["fwd"]["weighted_tflops"]
        line = {"metric": "GFLOP/s and % of MI355X MFMA peak for BRGEMM conv/FC/LSTM on 1 GPU",
                "value": tf * 1e3, "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                "ms_per_step": r5["fwd"]["total_ms_53_layers"], "higher_is_better": True, "scaling": "weak",
                "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                "config": {"workload": "cfg5: 53 conv layers of ResNet-50 v1.5, N=%d, bf16, fwd (weighted)" % nb,
                           "launch": "eager" if args.no_graph else "hip graph replay of the timed calls"},
                "roofline": {"bound": "mfma", "achieved": tf, "peak": PEAK_TFLOPS["bf16"], "unit": "TFLOP/s",
                             "frac": round(tf / PEAK_TFLOPS["bf16"], 4), "traffic": None},
                "cfg5": r5}
        print(json.dumps(line))
        return

    fn, flops, dt, name = MAKERS[args.workload](args.batch) if args.batch else MAKERS[args.workload]()
    wall, dev_s = _time_steps(fn, args.steps, args.warmup)
    if hasattr(fn, "verify"):
        fn.verify()
    per_step = wall / args.steps
    gflops = flops / per_step / 1e9
    kern_tflops = flops / (dev_s / args.steps) / 1e12
    line = {
        "metric": "GFLOP/s and % of MI355X MFMA peak for BRGEMM conv/FC/LSTM on 1 GPU",
        "value": round(gflops, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(per_step * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dt, "data": "synthetic",
        "config": {"workload": name, "untimed_clock_prewarm_s": PREWARM_S},
        "pct_of_mfma_peak": round(100 * gflops / 1e3 / PEAK_TFLOPS[dt], 2),
        "roofline": {"bound": "mfma", "achieved": round(kern_tflops, 3), "peak": PEAK_TFLOPS[dt],
                     "unit": "TFLOP/s", "frac": round(kern_tflops / PEAK_TFLOPS[dt], 4),
                     "traffic": None if args.batch else MEASURED_TRAFFIC_BYTES.get(args.workload),
                     "us_per_launch": round(dev_s / args.steps * 1e6, 2)},
    }
    if not args.no_others:
        others = {}
        for key in ("cfg1", "cfg1_ptrs", "cfg1_bf16", "cfg2", "cfg3", "cfg4", "cfg3_bf16", "cfg4_bwd", "cfg4_bf16", "cfg4_n168", "cfg4_n168_bf16"):
            if key == args.workload:
                continue
            f2, fl2, dt2, nm2 = MAKERS[key]()
            st, wu = (30, 5) if key.startswith("cfg4") else (100, 10)
            _, d2 = _time_steps(f2, st, wu)
            if hasattr(f2, "verify"):
                f2.verify()
            t = d2 / st
            others[key] = {"workload": nm2, "us_per_step": round(t * 1e6, 2), "gflops": round(fl2 / t / 1e9, 1),
                           "pct_of_mfma_peak": round(100 * fl2 / t / 1e12 / PEAK_TFLOPS[dt2], 2)}
            del f2
            torch.cuda.empty_cache()
        r5 = run_cfg5(20, 5, with_upd=True)
        others["cfg5"] = {"workload": "53 conv layers of ResNet-50 v1.5, N=64, bf16 in/out, weighted (bwd_wgt: fp32 result)",
                          "fwd": {k: v for k, v in r5["fwd"].items() if k != "layers"},
                          "bwd_data": {k: v for k, v in r5["bwd_data"].items() if k != "layers"},
                          "bwd_wgt": {k: v for k, v in r5["bwd_wgt"].items() if k != "layers"}}
        line["others"] = others
    if not args.no_cpu_baseline and args.workload == "cfg2":
        line["cpu_baseline"] = cpu_baseline_cfg2()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
