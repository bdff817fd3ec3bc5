"""Helpers shared by the GPU parity tests: move seeded host arrays to the device, run the
HIP path through the C ABI, bring results back as float32 numpy for comparison with the oracle.

Every output and workspace buffer the tests hand to the library sits between two 4 KiB guard bands
filled with a canary byte; `host()` and `check()` verify all live bands, so a store before the start
or past the end of any buffer fails the test that made it."""
import os
import weakref

import numpy as np
import torch

import oracle as orc
import paper_1906_06440_amd as brg

TOL = {brg.F32: 1e-5, brg.BF16: 1e-2}   # relative Frobenius error (spec tolerances)

GUARD = 4096
CANARY = 0xA5
_guarded = []      # weak references to the tensors handed out by empty() / workspace()


def dev(a, dtype=brg.F32):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if dtype == brg.BF16 else t


def as_seen_by_gpu(a, dtype):
    """The float32 values the kernels actually read: unchanged for fp32, RNE-rounded to bf16
    (by torch's cast on the host) for bf16.  The oracle is fed exactly these."""
    if dtype == brg.BF16:
        return torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).float().numpy()
    return np.ascontiguousarray(a, dtype=np.float32)


def tdtype(dtype):
    return torch.bfloat16 if dtype == brg.BF16 else torch.float32


def _banded(nbytes):
    """A uint8 view of `nbytes` bytes with GUARD canary bytes directly before and after it."""
    base = torch.full((GUARD + nbytes + GUARD,), CANARY, dtype=torch.uint8, device="cuda")
    body = base[GUARD:GUARD + nbytes]
    return body


def _register(t, nbytes):
    _guarded.append((weakref.ref(t), nbytes))
    return t


def empty(shape, dtype=brg.F32, fill=float("nan")):
    """Output buffer pre-filled with `fill` (NaN: an element the library leaves unwritten shows up as
    non-finite), between guard bands."""
    td = tdtype(dtype)
    n = int(np.prod(shape)) if len(shape) else 1
    nbytes = n * (2 if dtype == brg.BF16 else 4)
    t = _banded(nbytes).view(td).view(tuple(shape))
    t.fill_(fill)
    return _register(t, nbytes)


def workspace(nbytes):
    """Workspace of exactly `nbytes` bytes between guard bands (None for 0)."""
    if not nbytes:
        return None
    return _register(_banded(int(nbytes)), int(nbytes))


def check_guards():
    """Every live guarded buffer still has both canary bands intact."""
    torch.cuda.synchronize()
    alive = []
    for ref, nbytes in _guarded:
        t = ref()
        if t is None:
            continue
        alive.append((ref, nbytes))
        base = torch.empty(0, dtype=torch.uint8, device="cuda").set_(t.untyped_storage())
        assert base.numel() == nbytes + 2 * GUARD and t.storage_offset() * t.element_size() == GUARD
        lo_ok = bool((base[:GUARD] == CANARY).all().item())
        hi_ok = bool((base[GUARD + nbytes:] == CANARY).all().item())
        assert lo_ok, "write BEFORE the start of a %s buffer" % (tuple(t.shape),)
        assert hi_ok, "write PAST the end of a %s buffer" % (tuple(t.shape),)
    _guarded[:] = alive


def host(t):
    check_guards()
    return t.float().cpu().numpy()


_MARGINS = os.environ.get("BRG_TEST_MARGINS")     # path of a log of (what, norm error, element-wise excess)


def check(got, want, dtype, what="", out=None, widen=1.0):
    """Parity of one result tensor (or of sampled elements of it) with the oracle:
      * finite everywhere;
      * relative Frobenius error <= 1e-5 (fp32 inputs) / 1e-2 (bf16 inputs): the stated tolerances;
      * element by element within oracle.elem_bound: 1e-5 * widen * (|want| + rms(want)) for results stored
        in fp32 -- also when the inputs are bf16, whose products are exact in fp32 --, plus one bf16 spacing
        for results stored in bf16.
    `dtype` is the input type, `out` the stored type of the result (default: the input type)."""
    out = dtype if out is None else out
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), "non-finite output " + what
    err = orc.rel_fro(got, want)
    ex, j = orc.elem_excess(got, want, out_bf16=(out == brg.BF16), widen=widen)
    if _MARGINS:
        with open(_MARGINS, "a") as f:
            f.write("%-60s in=%d out=%d n=%d fro=%.3e excess=%.3f widen=%g\n"
                    % (what[:60], dtype, out, np.asarray(got).size, err, ex, widen))
    assert err <= TOL[dtype], "%s rel-Frobenius %.3e > %.1e" % (what, err, TOL[dtype])
    if ex > 1.0:
        g, w = np.asarray(got).ravel()[j], np.asarray(want).ravel()[j]
        raise AssertionError("%s element %d (of shape %s): got %.9g want %.9g, %.2f x the element-wise bound"
                             % (what, j, np.asarray(got).shape, g, w, ex))
    return err
