"""brg_conv_bwd_wgt_noalloc (the entry point that allocates nothing: partial sums in a device array built
into the library) against brg_conv_bwd_wgt with a caller workspace -- the same kernels, so bit for bit --
and against the oracle, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_1906_06440_amd as brg
import workloads as wl
from gpu_util import as_seen_by_gpu, check, dev, empty, host, workspace


def _desc(d):
    return brg.ConvDesc(d.N, d.C, d.H, d.W, d.K, d.R, d.S, d.stride, d.stride, d.pad, d.pad, d.bc, d.bk)


def test_noalloc_rejects_layers_beyond_its_scratch_before_any_gpu_call():
    # 3x3, 1152 -> 1152 channels: two pixel ranges of 72 x 72 blocks x 9 taps x 1 KiB = 91 MiB of partial sums
    d = brg.ConvDesc(64, 1152, 14, 14, 1152, 3, 3, 1, 1, 1, 1, 16, 16)
    need = brg.brg_conv_bwd_wgt_ws_bytes(d, brg.BF16)
    assert need > brg.CONV_BWD_WGT_NOALLOC_MAX_BYTES
    rc = brg.load().brg_conv_bwd_wgt_noalloc(d, brg.BF16, 0x1000, 0x1000, 0x1000, None)
    assert rc == brg.EUNSUPPORTED and str(need) in brg.last_error()
    assert brg.load().brg_conv_bwd_wgt_noalloc(d, brg.BF16, 0x1000, 0x1004, 0x1000, None) == brg.EALIGN
    assert brg.load().brg_conv_bwd_wgt_noalloc(d, brg.BF16, None, 0x1000, 0x1000, None) == brg.EINVAL


@pytest.mark.gpu
def test_noalloc_matches_workspace_form_twice_in_a_row_second_call_smaller():
    # first call: a large layer (pixel ranges: 36 MiB of partial sums); second: a small one whose partial sums
    # cover only the start of the scratch the first call left behind; third: a layer that needs no scratch
    cases = [(64, 256, 14, 256, 3, 2, 1), (4, 64, 14, 128, 1, 1, 0), (1, 64, 6, 64, 3, 1, 1)]
    sizes = []
    for (N, C, H, K, R, stride, pad) in cases:
        I, W, dO = wl.conv_tensors(N, C, H, K, R, stride, pad, cfg_index=5, seed_extra=N + K, want_dO=True)
        d = orc.ConvShape(N, C, H, H, K, R, R, stride, pad)
        need = brg.brg_conv_bwd_wgt_ws_bytes(_desc(d), brg.BF16)
        sizes.append(need)
        gI, gO = dev(I, brg.BF16), dev(dO, brg.BF16)
        ref, got = empty(d.w_shape), empty(d.w_shape)
        brg.brg_conv_bwd_wgt(_desc(d), brg.BF16, gI, gO, ref, workspace(need))
        brg.brg_conv_bwd_wgt_noalloc(_desc(d), brg.BF16, gI, gO, got)
        torch.cuda.synchronize()
        g, r = host(got), host(ref)
        assert np.array_equal(g, r), "the two entry points run the same kernels: results must be identical"
        Is, dOs = (as_seen_by_gpu(v, brg.BF16) for v in (I, dO))
        check(g, orc.conv_bwd_wgt(d, Is, dOs), brg.BF16, "no-alloc weight gradient %s" % (cases,), brg.F32,
              widen=max(1.0, (d.N * d.P * d.Q / 4096.0) ** 0.5))
    assert sizes[0] > sizes[1] > 0 and sizes[2] == 0, sizes
