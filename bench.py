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

# HBM bytes per launch of the dominant kernel come from a committed rocprofv3 counter summary, never from a
# constant in this file: profiles/<name>.txt carries one line `TRAFFIC {json}` written by
# `python -m paper_1906_06440_amd.profile_summary` from two --pmc runs (FETCH_SIZE, WRITE_SIZE, KiB per dispatch,
# each scaled by what the same counter reads for a plain device copy of known size) together with a hash of the
# kernel sources it was measured on.  The figure is reported only while those sources are unchanged.
TRAFFIC_PROFILE = {"cfg2": "conv_tile_f32__cfg2_conv3x3_fwd.txt", "cfg3": "block_ring_f32_g128__cfg3_mlp.txt"}


def kernel_sources_sha(files):
    import hashlib
    h = hashlib.sha1()
    for f in sorted(files):
        with open(os.path.join(ROOT, "paper_1906_06440_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, profiles_dir=None):
    """(bytes per step, source) from the committed profile of this workload, or (None, reason)."""
    name = TRAFFIC_PROFILE.get(workload)
    if not name:
        return None, "no counter profile for this workload"
    path = os.path.join(profiles_dir or os.path.join(ROOT, "profiles"), name)
    try:
        for line in open(path):
            if line.startswith("TRAFFIC "):
                t = json.loads(line[len("TRAFFIC "):])
                if kernel_sources_sha(t["sources"]) != t["sources_sha"]:
                    return None, "profiles/%s was measured on other kernel sources" % name
                return int(t["bytes_per_step"]), "profiles/" + name
    except OSError:
        pass
    return None, "profiles/%s has no TRAFFIC line" % name


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


def make_cfg3_bf16(N=1024, blk=16):
    """Context rows: the cfg3 MLP in bf16 on 16-wide blocks (bn = 64) or on cfg3's own 64-wide blocks, forward with
    bias + ReLU and the chained backward pass with the workspace that lets the masked last layer use the tuned kernels."""
    import numpy as np
    import torch
    import paper_1906_06440_amd as brg
    import workloads as wl
    X0, Ws, bs, dYl = wl.cfg3_mlp(N=N, bc=blk, bk=blk)
    desc = brg.FcDesc(N, 1024, 1024, 64, blk, blk)
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
    return fn, 12 * 2.0 * N * 1024 ** 2, "bf16", "cfg3 in bf16: MLP 4 x FC 1024->1024 bias+ReLU, N=%d, fwd+bwd-data+wgt, bn=64 bc=bk=%d" % (N, blk)


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


def make_cfg4_bwd(bf16=False):
    """Context row: backward pass of the cfg4 LSTM layer (dx, dW, dR, db from a random dh); the forward
    results it differentiates are computed once outside the timed region.  Flops: twice the forward's.
    bf16: x, W4, R4 and h are bf16, the pass widens them and runs in fp32."""
    import torch
    import paper_1906_06440_amd as brg
    import workloads as wl
    x, W4, R4, _ = wl.cfg4_lstm()
    dt = brg.BF16 if bf16 else brg.F32
    dx, dW, dR = _dev(x, bf16), _dev(W4, bf16), _dev(R4, bf16)
    h = torch.empty((50, 64, 1024), device="cuda", dtype=torch.bfloat16 if bf16 else torch.float32)
    s = torch.empty((50, 64, 1024), device="cuda")
    g = torch.empty((4, 50, 64, 1024), device="cuda")
    desc = brg.LstmDesc(50, 64, 1024, 1024, 16, 64, 64)
    ws = torch.zeros(64, dtype=torch.uint8, device="cuda")
    brg.brg_lstm_fwd(desc, dt, dx, dW, dR, None, None, None, h, s, g, ws)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4)
    dh = torch.rand((50, 64, 1024), device="cuda", generator=gen) * 0.2 - 0.1
    f32 = dict(device="cuda", dtype=torch.float32)
    gx, gW, gR, gb = torch.empty(dx.shape, **f32), torch.empty(dW.shape, **f32), torch.empty(dR.shape, **f32), torch.empty((4, 1024), **f32)
    wsb = torch.empty(brg.brg_lstm_bwd_ws_bytes_dtype(desc, dt), dtype=torch.uint8, device="cuda")
    fn = lambda: brg.brg_lstm_bwd(desc, dt, dx, dW, dR, None, None, h, s, g, dh, None, gx, gW, gR, gb, None, None, wsb)
    return fn, 2 * 50 * 2.0 * 64 * 4 * 1024 * 2048, "f32", "cfg4 backward: LSTM bwd (dx, dW, dR, db) T=50 N=64 C=K=1024, %s" % (
        "bf16 operands widened, fp32 arithmetic" if bf16 else "fp32")


HBM_BYTES_PER_S = 8.0e12        # MI355X HBM3E peak


def make_cfg5_layers(N=64, only=None, cold_bytes=0):
    """For each of the 23 distinct ResNet-50 v1.5 shapes (bf16 in/out): the layer, its algorithmic HBM bytes per
    direction, and per direction a LIST of closures, one per buffer set.  Set 0 is the warm set; with cold_bytes > 0
    every layer gets enough further sets (at least 4 in all) that cycling through them touches more than that many
    bytes between two uses of the same set, i.e. nothing is left in the 256 MB memory-side cache."""
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
        desc = brg.ConvDesc(N, Cp, L.H, L.H, L.K, L.R, L.R, L.stride, L.stride, L.pad, L.pad, bc, 16)
        b_in, b_w, b_out = I.size * 2, W.size * 2, dO.size * 2
        nbytes = {"fwd": b_in + b_w + b_out, "bwd_data": b_in + b_w + b_out, "bwd_wgt": b_in + b_out + W.size * 4}
        nsets = 1 if not cold_bytes else int(min(48, max(4, -(-cold_bytes // (b_in + b_out)) + 1)))
        base = (_dev(I, True), _dev(W, True), _dev(dO, True))
        fns = {"fwd": [], "bwd_data": [], "bwd_wgt": []}
        for k in range(nsets):
            dI, dW, ddO = base if k == 0 else tuple(t.clone() for t in base)
            O = torch.empty(ddO.shape, dtype=torch.bfloat16, device="cuda")
            gI = torch.empty(dI.shape, dtype=torch.bfloat16, device="cuda")
            ws = torch.empty(max(16, brg.brg_conv_ws_bytes(desc, brg.BF16)), dtype=torch.uint8, device="cuda")
            fns["fwd"].append(lambda desc=desc, dI=dI, dW=dW, O=O, ws=ws: brg.brg_conv_fwd(desc, brg.BF16, brg.BF16, dI, dW, O,
                                                                                         None, brg.ACT_NONE, ws))
            fns["bwd_data"].append(lambda desc=desc, ddO=ddO, dW=dW, gI=gI: brg.brg_conv_bwd_data(desc, brg.BF16, brg.BF16, ddO, dW, gI))
            # weight gradient (fp32 result), with the workspace for the partial sums of the pixel ranges
            gW = torch.empty(dW.shape, dtype=torch.float32, device="cuda")
            wws = torch.empty(max(16, brg.brg_conv_bwd_wgt_ws_bytes(desc, brg.BF16)), dtype=torch.uint8, device="cuda")
            fns["bwd_wgt"].append(lambda desc=desc, dI=dI, ddO=ddO, gW=gW, wws=wws: brg.brg_conv_bwd_wgt(desc, brg.BF16, dI, ddO, gW, wws))
        out.append((L, nbytes, fns))
    return out


def _cycle(fns):
    """A callable that runs the closures of the buffer sets in turn, one per call."""
    state = {"i": 0}

    def fn():
        fns[state["i"] % len(fns)]()
        state["i"] += 1
    return fn


def run_cfg5(steps, warmup, N=64, use_graph=True, with_upd=False, only=None, cold=True):
    """Weighted efficiency (sum n_i F_i) / (sum n_i t_i) over the 53 layers, fwd and bwd-data (and, on request, the
    weight gradient).  Each layer's K timed calls are replayed from one HIP graph (see _time_graph) unless use_graph
    is False.  Every layer is priced against its own roofline max(F / 2.5 PFLOP/s, B / 8 TB/s) with B the
    algorithmic bytes (input + weights + output of the direction), and timed twice: `warm` on one buffer set (fits the
    256 MB memory-side cache) and `cold` cycling through buffer sets of more than 512 MB in all."""
    import torch
    res = {}
    timer = (lambda f, st, wu: _time_graph(f, st, wu)) if use_graph else (lambda f, st, wu: _time_steps(f, st, wu)[1])
    for name in ("fwd", "bwd_data") + (("bwd_wgt",) if with_upd else ()):
        res[name] = {"layers": []}
    # layers are built one at a time so that only one layer's buffer sets are alive
    import workloads as wl
    names = [l.name for l in wl.resnet50_v15_layers() if not only or l.name in only]
    tot = {k: {"F": 0.0, "T": 0.0, "Tc": 0.0, "R": 0.0} for k in res}
    for lname in names:
        (L, nbytes, fns), = make_cfg5_layers(N, [lname], cold_bytes=(512 << 20) if cold else 0)
        for name in res:
            st = steps
            if name == "bwd_wgt":   # layers without a tuned weight-gradient kernel run for milliseconds: fewer calls
                fns[name][0]()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                fns[name][0]()
                torch.cuda.synchronize()
                if time.perf_counter() - t0 > 1e-3:
                    st = 2
            t = timer(fns[name][0], st, min(warmup, st)) / st
            nset = len(fns[name])
            stc = max(st, nset) if st > 2 else st
            tc = timer(_cycle(fns[name]), stc, nset) / stc if cold and nset > 1 else None
            F, B = L.flops(N), nbytes[name]
            roof = max(F / (PEAK_TFLOPS["bf16"] * 1e12), B / HBM_BYTES_PER_S)
            row = {"layer": L.name, "n": L.count, "us": round(t * 1e6, 1), "tflops": round(F / t / 1e12, 1),
                   "GBps": round(B / t / 1e9), "bound": "hbm" if B / HBM_BYTES_PER_S >= F / (PEAK_TFLOPS["bf16"] * 1e12) else "mfma",
                   "roof_us": round(roof * 1e6, 1), "frac": round(roof / t, 3)}
            if tc is not None:
                row.update({"us_cold": round(tc * 1e6, 1), "GBps_cold": round(B / tc / 1e9), "frac_cold": round(roof / tc, 3)})
            res[name]["layers"].append(row)
            a = tot[name]
            a["F"] += L.count * F; a["T"] += L.count * t; a["R"] += L.count * roof
            a["Tc"] += L.count * (tc if tc is not None else t)
        del fns
        torch.cuda.empty_cache()
    for name, a in tot.items():
        tf = a["F"] / a["T"] / 1e12
        res[name].update({
            "weighted_tflops": round(tf, 2), "total_ms_53_layers": round(a["T"] * 1e3, 3),
            "frac_of_bf16_peak": round(tf / PEAK_TFLOPS["bf16"], 4),
            # the sum of the per-layer rooflines against the sum of the measured times
            "roofline": {"bound": "per layer: max(flops / 2.5 PFLOP/s, bytes / 8 TB/s)", "achieved": round(a["T"] * 1e3, 3),
                         "peak": round(a["R"] * 1e3, 3), "unit": "ms for the 53 layers (lower is better)",
                         "frac": round(a["R"] / a["T"], 4), "frac_cold": round(a["R"] / a["Tc"], 4) if cold else None,
                         "total_ms_cold": round(a["Tc"] * 1e3, 3) if cold else None}})
    return res


MAKERS = {"cfg4_bf16": lambda: make_cfg4_variant(64, True), "cfg4_n168": lambda: make_cfg4_variant(168, False),
          "cfg4_n168_bf16": lambda: make_cfg4_variant(168, True), "cfg1": make_cfg1, "cfg1_ptrs": make_cfg1_ptrs, "cfg1_bf16": make_cfg1_bf16, "cfg2": make_cfg2, "cfg3": make_cfg3, "cfg4": make_cfg4, "cfg3_bf16": make_cfg3_bf16, "cfg4_bwd": make_cfg4_bwd,
          "cfg4_bwd_bf16": lambda: make_cfg4_bwd(True), "cfg3_bf16_b64": lambda: make_cfg3_bf16(1024, 64)}


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
    out = {"value": round(flops / dt / 1e9, 2), "unit": "GFLOP/s", "cores": cores, "kind": "oracle",
           "sample": "conv fwd of the first %d of 64 images of cfg2, %d run(s) of %.1f s" % (n, reps, dt)}
    # the same routine on ONE thread (the OpenMP runtime the oracle library is linked with is told so), two images
    try:
        import ctypes
        omp = ctypes.CDLL("libgomp.so.1")
        omp.omp_set_num_threads(1)
        I1, W1 = wl.cfg2_conv(2)
        d1 = orc.ConvShape(2, 64, 56, 56, 64, 3, 3, 1, 1)
        t0 = time.perf_counter()
        orc.conv_fwd(d1, I1, W1)
        dt1 = time.perf_counter() - t0
        omp.omp_set_num_threads(cores)
        out["single_thread"] = {"value": round(2 * 2.0 * 64 * 64 * 9 * 56 * 56 / dt1 / 1e9, 3), "unit": "GFLOP/s", "cores": 1,
                                "sample": "conv fwd of the first 2 images of cfg2, one run of %.1f s" % dt1}
    except OSError:
        pass
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg1_ptrs", "cfg1_bf16", "cfg2", "cfg3", "cfg4", "cfg5", "cfg3_bf16", "cfg3_bf16_b64", "cfg4_bwd", "cfg4_bf16", "cfg4_n168",
                             "cfg4_n168_bf16", "cfg4_bwd_bf16", "cfg3_bf16_b64", "copy"])
    ap.add_argument("--batch", type=int, default=None,
                    help="minibatch of cfg2 / cfg3 / cfg5 instead of the configured one (context rows: the paper's own "
                         "28 / 1344, inference at 1); such a line carries no others and no cpu_baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="cfg5: time eager launches instead of a HIP graph replay")
    ap.add_argument("--upd", action="store_true", help="cfg5: also time the weight gradient")
    ap.add_argument("--no-cold", action="store_true", help="cfg5: skip the rotating-buffer (cache-cold) timings")
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
                      only=args.layers.split(",") if args.layers else None, cold=not args.no_cold)
        tf = r5["fwd"]["weighted_tflops"]
        line = {"metric": "GFLOP/s and % of MI355X MFMA peak for BRGEMM conv/FC/LSTM on 1 GPU",
                "value": tf * 1e3, "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                "ms_per_step": r5["fwd"]["total_ms_53_layers"], "higher_is_better": True, "scaling": "weak",
                "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                "config": {"workload": "cfg5: 53 conv layers of ResNet-50 v1.5, N=%d, bf16, fwd (weighted)" % nb,
                           "launch": "eager" if args.no_graph else "hip graph replay of the timed calls"},
                "roofline": dict(r5["fwd"]["roofline"], traffic=None),
                "pct_of_mfma_peak": round(100 * tf / PEAK_TFLOPS["bf16"], 2),
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
                     "traffic": None, "us_per_launch": round(dev_s / args.steps * 1e6, 2)},
    }
    if not args.batch:
        line["roofline"]["traffic"], line["roofline"]["traffic_source"] = measured_traffic(args.workload)
    if not args.no_others:
        others = {}
        for key in ("cfg1", "cfg1_ptrs", "cfg1_bf16", "cfg2", "cfg3", "cfg4", "cfg3_bf16", "cfg3_bf16_b64", "cfg4_bwd", "cfg4_bwd_bf16", "cfg4_bf16", "cfg4_n168", "cfg4_n168_bf16"):
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
        r5 = run_cfg5(10, 3, with_upd=True)
        others["cfg5"] = dict({"workload": "53 conv layers of ResNet-50 v1.5, N=64, bf16 in/out, weighted (bwd_wgt: fp32 result); "
                                           "per layer: warm = one buffer set, cold = rotating buffer sets > 512 MB"}, **r5)
        r1 = run_cfg5(10, 3, N=1, cold=False)   # the inference shapes of section 4.3: one image
        others["cfg5_n1"] = {"workload": "53 conv layers of ResNet-50 v1.5, N=1, bf16 in/out, weighted, forward (inference)",
                             "weighted_tflops": r1["fwd"]["weighted_tflops"], "total_ms_53_layers": r1["fwd"]["total_ms_53_layers"],
                             "us_per_layer": {row["layer"]: row["us"] for row in r1["fwd"]["layers"]}}
        line["others"] = others
    if not args.no_cpu_baseline and args.workload == "cfg2":
        line["cpu_baseline"] = cpu_baseline_cfg2()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
