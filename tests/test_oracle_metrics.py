"""Pins of the error measures every parity assertion goes through (hand values), and of the sampled
convolution oracles (every element of small cases, with bias, activation and bf16 rounding)."""
import math

import numpy as np
import pytest

import oracle as orc
import workloads as wl


def test_rel_fro_hand_values():
    # ||(3,4) - (0,0)|| / ||(3,4)|| with got = 0  ->  5 / 5
    assert orc.rel_fro([0.0, 0.0], [3.0, 4.0]) == 1.0
    # got - want = (0.3, -0.4, 0, 0): norm 0.5; ||want|| = ||(1, 2, 2, 4)|| = 5
    assert math.isclose(orc.rel_fro([1.3, 1.6, 2.0, 4.0], [1.0, 2.0, 2.0, 4.0]), 0.1, rel_tol=1e-12)
    # not symmetric: the denominator is the SECOND argument
    assert math.isclose(orc.rel_fro([3.0, 4.0], [6.0, 8.0]), 0.5, rel_tol=1e-12)
    assert math.isclose(orc.rel_fro([6.0, 8.0], [3.0, 4.0]), 1.0, rel_tol=1e-12)
    # shape is ignored, values are taken in order; zero reference
    assert orc.rel_fro(np.zeros((2, 2)), np.zeros(4)) == 0.0
    assert orc.rel_fro([1e-30], [0.0]) == float("inf")
    # a NaN in the result is never a pass
    assert not (orc.rel_fro([float("nan"), 1.0], [1.0, 1.0]) <= 1.0)
    # computed in float64 even for float32 inputs: 1e-9 relative differences survive
    a = np.array([1.0, 1.0], np.float32)
    assert orc.rel_fro(a.astype(np.float64) + 1e-9, a) > 0


def test_bf16_ulp_hand_values():
    # bf16 has 8 significant bits: numbers in [1, 2) are spaced 2^-7, in [2, 4) 2^-6, in [0.5, 1) 2^-8
    assert orc.bf16_ulp(1.0) == 2.0 ** -7 and orc.bf16_ulp(1.999) == 2.0 ** -7
    assert orc.bf16_ulp(2.0) == 2.0 ** -6 and orc.bf16_ulp(-3.5) == 2.0 ** -6
    assert orc.bf16_ulp(0.75) == 2.0 ** -8 and orc.bf16_ulp(0.0) == 0.0
    # the spacing is what the quantiser produces: next bf16 above x minus x
    for x in (1.0, 0.3359375, 100.0, 0.00150299072265625):
        b = orc.f32_to_bf16_bits(x)
        assert orc.bf16_bits_to_f32(b) == x, "test values are bf16 numbers"
        assert orc.bf16_bits_to_f32(b + 1) - x == orc.bf16_ulp(x)


def test_elem_bound_and_excess_hand_values():
    want = np.array([3.0, -4.0, 0.0, 5.0])         # rms = sqrt(50/4)
    rms = math.sqrt(12.5)
    b = orc.elem_bound(want, want)
    assert np.allclose(b, 1e-5 * (np.abs(want) + rms), rtol=1e-14)
    assert np.allclose(orc.elem_bound(want, want, widen=3.0), 3.0 * b, rtol=1e-14)
    got = want.copy()
    got[2] += 2.0 * b[2]                            # twice the bound on the zero element
    ex, j = orc.elem_excess(got, want)
    assert j == 2 and math.isclose(ex, 2.0, rel_tol=1e-9)
    got = want.copy()
    got[3] += 0.5 * b[3]
    ex, j = orc.elem_excess(got, want)
    assert j == 3 and math.isclose(ex, 0.5, rel_tol=1e-9)
    assert orc.elem_excess(want, want) == (0.0, 0)
    got = want.copy()
    got[1] = np.nan
    assert orc.elem_excess(got, want)[0] == float("inf")
    # bf16 results: neighbouring bf16 numbers pass, two spacings apart fail
    w = np.array([1.0, 1.0, 1.0, 1.0])
    assert orc.elem_excess(w + 2.0 ** -7, w, out_bf16=True)[0] < 1.0
    assert orc.elem_excess(w + 2.0 ** -6, w, out_bf16=True)[0] > 1.0
    # a single wrong element that a whole-tensor norm of 1e-2 would let through is caught
    w = np.ones(10000)
    g = w.copy()
    g[1234] = 1.5
    assert orc.rel_fro(g, w) < 1e-2 and orc.elem_excess(g, w, out_bf16=True) == (pytest.approx(0.5 / (2e-5 + 2.0 ** -7)), 1234)


CASES = [  # N C H W K R stride pad bc
    (2, 32, 7, 9, 48, 3, 1, 1, 16), (3, 16, 8, 8, 32, 3, 2, 1, 16), (2, 48, 6, 5, 16, 1, 2, 0, 16),
    (1, 4, 13, 12, 32, 7, 2, 3, 4), (2, 32, 5, 5, 32, 1, 1, 0, 16), (1, 16, 9, 7, 16, 3, 2, 0, 16),
]


@pytest.mark.parametrize("N,C,H,W,K,R,stride,pad,bc", CASES)
@pytest.mark.parametrize("out_bf16", [False, True])
def test_sampled_conv_oracles_equal_the_full_ones_on_every_element(N, C, H, W, K, R, stride, pad, bc, out_bf16):
    """orc_conv_fwd_sample / orc_conv_bwd_data_sample are the only checkers of the full-size ResNet-50 layers:
    each must return, for EVERY index of a small case, bit for bit what the full routine stores -- with bias,
    each activation and the bf16 rounding of the result (forward), and for pixels no tap reaches (backward)."""
    rng = np.random.default_rng(N * 1000 + H * 10 + R)
    d = orc.ConvShape(N, C, H, W, K, R, R, stride, pad, bc=bc)
    I = orc.round_bf16(wl.uniform(rng, d.i_shape))
    Wt = orc.round_bf16(wl.normal(rng, d.w_shape, 0.2))
    dO = orc.round_bf16(wl.uniform(rng, d.o_shape))
    bias = wl.uniform(rng, (K,))
    n, k, p, q = np.meshgrid(np.arange(N), np.arange(K), np.arange(d.P), np.arange(d.Q), indexing="ij")
    idx = np.stack([a.ravel() for a in (n, k, p, q)], axis=1)
    for act in (orc.ACT_NONE, orc.ACT_RELU, orc.ACT_SIGMOID, orc.ACT_TANH):
        for b in (None, bias):
            full = orc.conv_fwd(d, I, Wt, b, act, out_bf16=out_bf16)
            smp = orc.conv_fwd_sample(d, I, Wt, idx, b, act, out_bf16=out_bf16)
            assert np.array_equal(smp, full[idx[:, 0], idx[:, 1] // 16, idx[:, 2], idx[:, 3], idx[:, 1] % 16])
    n, c, h, w = np.meshgrid(np.arange(N), np.arange(C), np.arange(H), np.arange(W), indexing="ij")
    idx = np.stack([a.ravel() for a in (n, c, h, w)], axis=1)
    full = orc.conv_bwd_data(d, dO, Wt, out_bf16=out_bf16)
    smp = orc.conv_bwd_data_sample(d, dO, Wt, idx, out_bf16=out_bf16)
    assert np.array_equal(smp, full[idx[:, 0], idx[:, 1] // bc, idx[:, 2], idx[:, 3], idx[:, 1] % bc])
    if out_bf16:
        assert np.array_equal(full, orc.round_bf16(full)), "stored values are bf16 numbers"
