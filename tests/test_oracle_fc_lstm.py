"""Pins for the CPU oracle's fully connected and LSTM routines (no GPU)."""
import math

import numpy as np
import pytest
import torch

import oracle as orc


def _rand(rng, shape, a=1.0):
    return ((2 * rng.random(shape, dtype=np.float32) - 1) * a).astype(np.float32)


# ------------------------------------------------------------------- FC ----
def test_fc_fwd_is_gemm_numpy():
    rng = np.random.default_rng(1)
    d = orc.FcShape(12, 20, 9, 4, 5, 3)
    X, W = _rand(rng, (d.N, d.C)), _rand(rng, (d.K, d.C))
    Y = orc.fc_fwd(d, orc.a2_to_blocked(X, d.bn, d.bc), orc.w2_to_blocked(W, d.bc, d.bk))
    assert orc.rel_fro(orc.blocked_to_a2(Y), X.astype(np.float64) @ W.astype(np.float64).T) < 1e-7


def test_fc_fwd_bias_relu_numpy():
    rng = np.random.default_rng(2)
    d = orc.FcShape(8, 16, 8, 4, 8, 4)
    X, W, b = _rand(rng, (d.N, d.C)), _rand(rng, (d.K, d.C)), _rand(rng, (d.K,))
    Y = orc.fc_fwd(d, orc.a2_to_blocked(X, d.bn, d.bc), orc.w2_to_blocked(W, d.bc, d.bk), b, orc.ACT_RELU)
    want = np.maximum(X.astype(np.float64) @ W.astype(np.float64).T + b, 0)
    assert orc.rel_fro(orc.blocked_to_a2(Y), want) < 1e-7


def test_fc_bwd_vs_numpy_and_adjoint():
    rng = np.random.default_rng(3)
    d = orc.FcShape(12, 20, 9, 4, 5, 3)
    X, W, b = _rand(rng, (d.N, d.C)), _rand(rng, (d.K, d.C)), _rand(rng, (d.K,))
    dY = _rand(rng, (d.N, d.K))
    Xb, Wb = orc.a2_to_blocked(X, d.bn, d.bc), orc.w2_to_blocked(W, d.bc, d.bk)
    Yb = orc.fc_fwd(d, Xb, Wb, b, orc.ACT_RELU)
    dX, dW, db = orc.fc_bwd(d, orc.a2_to_blocked(dY, d.bn, d.bk), Yb, Xb, Wb, orc.ACT_RELU)
    Y = orc.blocked_to_a2(Yb)
    dZ = dY.astype(np.float64) * (Y > 0)
    assert orc.rel_fro(orc.blocked_to_a2(dX), dZ @ W.astype(np.float64)) < 1e-7
    assert orc.rel_fro(orc.blocked_to_w2(dW), dZ.T @ X.astype(np.float64)) < 1e-7
    assert orc.rel_fro(db, dZ.sum(0)) < 1e-7
    # linear case: adjoint identities <W X, dY> = <X, dX> = <W, dW>
    Yl = orc.blocked_to_a2(orc.fc_fwd(d, Xb, Wb)).astype(np.float64)
    dX, dW, db = orc.fc_bwd(d, orc.a2_to_blocked(dY, d.bn, d.bk), None, Xb, Wb, orc.ACT_NONE)
    lhs = (Yl * dY).sum()
    assert abs(lhs - (X.astype(np.float64) * orc.blocked_to_a2(dX)).sum()) < 1e-6 * abs(lhs) + 1e-6
    assert abs(lhs - (W.astype(np.float64) * orc.blocked_to_w2(dW)).sum()) < 1e-6 * abs(lhs) + 1e-6


def test_fc_relu_all_negative_kills_gradients():
    d = orc.FcShape(4, 4, 4, 2, 2, 2)
    X = np.ones(d.x_shape, np.float32)
    W = -np.ones(d.w_shape, np.float32)
    Y = orc.fc_fwd(d, X, W, None, orc.ACT_RELU)
    assert np.all(Y == 0)
    dX, dW, db = orc.fc_bwd(d, np.ones(d.y_shape, np.float32), Y, X, W, orc.ACT_RELU)
    assert np.all(dX == 0) and np.all(dW == 0) and np.all(db == 0)


def test_fc_bwd_vs_torch_autograd():
    rng = np.random.default_rng(4)
    d = orc.FcShape(16, 32, 24, 8, 16, 8)
    X, W, b = _rand(rng, (d.N, d.C)), _rand(rng, (d.K, d.C)), _rand(rng, (d.K,))
    dY = _rand(rng, (d.N, d.K))
    xt = torch.from_numpy(X).double().requires_grad_(True)
    wt = torch.from_numpy(W).double().requires_grad_(True)
    bt = torch.from_numpy(b).double().requires_grad_(True)
    y = torch.relu(xt @ wt.T + bt)
    y.backward(torch.from_numpy(dY).double())
    Xb, Wb = orc.a2_to_blocked(X, d.bn, d.bc), orc.w2_to_blocked(W, d.bc, d.bk)
    Yb = orc.fc_fwd(d, Xb, Wb, b, orc.ACT_RELU)
    assert orc.rel_fro(orc.blocked_to_a2(Yb), y.detach().numpy()) < 1e-7
    dX, dW, db = orc.fc_bwd(d, orc.a2_to_blocked(dY, d.bn, d.bk), Yb, Xb, Wb, orc.ACT_RELU)
    assert orc.rel_fro(orc.blocked_to_a2(dX), xt.grad.numpy()) < 1e-6
    assert orc.rel_fro(orc.blocked_to_w2(dW), wt.grad.numpy()) < 1e-6
    assert orc.rel_fro(db, bt.grad.numpy()) < 1e-6


# ----------------------------------------------------------------- LSTM ----
def _sig(z):
    return 1.0 / (1.0 + math.exp(-z))


def test_lstm_scalar_by_hand():
    """N=C=K=1, T=2: equations (1)-(6) evaluated with python floats."""
    d = orc.LstmShape(2, 1, 1, 1, 1, 1, 1)
    W = np.array([0.5, -0.25, 0.75, 1.0], np.float32).reshape(d.w_shape)   # i, c, f, o
    R = np.array([0.125, 0.5, -0.5, 0.25], np.float32).reshape(d.r_shape)
    b = np.array([0.1, -0.2, 0.3, -0.4], np.float32).reshape(4, 1)
    x = np.array([0.5, -1.0], np.float32).reshape(2, 1, 1)
    h0 = np.array([[0.25]], np.float32)
    s0 = np.array([[-0.5]], np.float32)
    h, s, g = orc.lstm_fwd(d, x, W, R, b, h0, s0)
    hp, sp = 0.25, -0.5
    for t in range(2):
        xt = float(x[t, 0, 0])
        z = [float(W.ravel()[j]) * xt + float(R.ravel()[j]) * hp + float(b[j, 0]) for j in range(4)]
        i, c, f, o = _sig(z[0]), math.tanh(z[1]), _sig(z[2]), _sig(z[3])
        st = f * sp + i * c
        ht = o * math.tanh(st)
        assert s[t, 0, 0] == pytest.approx(st, rel=1e-6)
        assert h[t, 0, 0] == pytest.approx(ht, rel=1e-6)
        assert [g[j, t, 0, 0] for j in range(4)] == pytest.approx([i, c, f, o], rel=1e-6)
        hp, sp = float(np.float32(ht)), float(np.float32(st))


def test_lstm_zero_weights_closed_form():
    """W = R = 0: s_t = sig(b_f) s_{t-1} + sig(b_i) tanh(b_c) (geometric series), h_t = sig(b_o) tanh(s_t)."""
    d = orc.LstmShape(6, 2, 4, 4, 2, 2, 2)
    b = np.array([[0.3] * 4, [-0.7] * 4, [0.9] * 4, [0.2] * 4], np.float32)
    x = np.ones((d.T, d.N, d.C), np.float32)
    h, s, _ = orc.lstm_fwd(d, x, np.zeros(d.w_shape, np.float32), np.zeros(d.r_shape, np.float32), b)
    f, a, o = _sig(float(b[2, 0])), _sig(float(b[0, 0])) * math.tanh(float(b[1, 0])), _sig(float(b[3, 0]))
    for t in range(d.T):
        st = a * (1 - f ** (t + 1)) / (1 - f)
        assert np.allclose(s[t], st, rtol=1e-6)
        assert np.allclose(h[t], o * math.tanh(st), rtol=1e-6)


def _plain_weights(rng, d, a):
    W = _rand(rng, (4, d.K, d.C), a)
    R = _rand(rng, (4, d.K, d.K), a)
    Wb = np.stack([orc.w2_to_blocked(W[g], d.bc, d.bk) for g in range(4)])
    Rb = np.stack([orc.w2_to_blocked(R[g], d.bk, d.bk) for g in range(4)])
    return W, R, Wb, Rb


def test_lstm_single_step_is_four_gemms():
    rng = np.random.default_rng(5)
    d = orc.LstmShape(1, 6, 8, 12, 2, 4, 3)
    W, R, Wb, Rb = _plain_weights(rng, d, 0.5)
    b = _rand(rng, (4, d.K), 0.5)
    x = _rand(rng, (1, d.N, d.C))
    h, s, g = orc.lstm_fwd(d, x, Wb, Rb, b)        # h0 = s0 = 0
    z = np.einsum("gkc,nc->gnk", W.astype(np.float64), x[0].astype(np.float64)) + b[:, None, :]
    sg = lambda v: 1 / (1 + np.exp(-v))
    i, c, f, o = sg(z[0]), np.tanh(z[1]), sg(z[2]), sg(z[3])
    assert orc.rel_fro(s[0], i * c) < 1e-6
    assert orc.rel_fro(h[0], o * np.tanh(i * c)) < 1e-6
    assert orc.rel_fro(g[2, 0], f) < 1e-6


def test_lstm_stacked_large_gemm_formulation_and_torch():
    """The [W R]·[x;h] stacked formulation of section 3.1.1 and torch.nn.LSTM (float64, gates
    permuted i,c,f,o -> i,f,g,o) both reproduce the oracle."""
    rng = np.random.default_rng(6)
    d = orc.LstmShape(5, 4, 8, 12, 2, 4, 3)
    W, R, Wb, Rb = _plain_weights(rng, d, 0.4)
    b = _rand(rng, (4, d.K), 0.4)
    x = _rand(rng, (d.T, d.N, d.C))
    h0, s0 = _rand(rng, (d.N, d.K), 0.5), _rand(rng, (d.N, d.K), 0.5)
    h, s, g = orc.lstm_fwd(d, x, Wb, Rb, b, h0, s0)
    # stacked formulation
    WR = np.concatenate([W.reshape(4 * d.K, d.C), R.reshape(4 * d.K, d.K)], axis=1).astype(np.float64)
    hp, sp = h0.astype(np.float64), s0.astype(np.float64)
    sg = lambda v: 1 / (1 + np.exp(-v))
    for t in range(d.T):
        z = (np.concatenate([x[t], hp], axis=1) @ WR.T + b.reshape(-1)).reshape(d.N, 4, d.K)
        i, c, f, o = sg(z[:, 0]), np.tanh(z[:, 1]), sg(z[:, 2]), sg(z[:, 3])
        sp = f * sp + i * c
        hp = o * np.tanh(sp)
        assert orc.rel_fro(h[t], hp) < 1e-5
        assert orc.rel_fro(s[t], sp) < 1e-5
    # torch third opinion
    lstm = torch.nn.LSTM(d.C, d.K).double()
    order = [0, 2, 1, 3]  # torch rows: i, f, g(candidate), o  <- paper order i, c, f, o
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(torch.from_numpy(np.concatenate([W[j] for j in order])).double())
        lstm.weight_hh_l0.copy_(torch.from_numpy(np.concatenate([R[j] for j in order])).double())
        lstm.bias_ih_l0.copy_(torch.from_numpy(np.concatenate([b[j] for j in order])).double())
        lstm.bias_hh_l0.zero_()
        out, (hn, cn) = lstm(torch.from_numpy(x).double(),
                             (torch.from_numpy(h0).double()[None], torch.from_numpy(s0).double()[None]))
    assert orc.rel_fro(h, out.numpy()) < 1e-5
    assert orc.rel_fro(s[-1], cn[0].numpy()) < 1e-5


def test_lstm_invariants():
    rng = np.random.default_rng(8)
    d = orc.LstmShape(4, 4, 8, 8, 2, 4, 4)
    _, _, Wb, Rb = _plain_weights(rng, d, 1.0)
    h, s, g = orc.lstm_fwd(d, _rand(rng, (d.T, d.N, d.C)), Wb, Rb)
    assert np.all(np.abs(h) < 1)
    for j in (0, 2, 3):
        assert np.all((g[j] > 0) & (g[j] < 1))
    assert np.all(np.abs(g[1]) < 1)


# ------------------------------------------------------- LSTM backward ----
def _np_lstm_fwd64(x, W, R, b, h0, s0):
    """Equations 1-6 of section 3.1 in float64 on plain [4][K][C] / [4][K][K] weights (own restatement for the
    finite-difference pin; gate order i, c, f, o)."""
    sg = lambda v: 1.0 / (1.0 + np.exp(-v))
    hp, sp, hs = h0, s0, []
    for t in range(x.shape[0]):
        z = [x[t] @ W[g].T + hp @ R[g].T + b[g] for g in range(4)]
        i, c, f, o = sg(z[0]), np.tanh(z[1]), sg(z[2]), sg(z[3])
        sp = f * sp + i * c
        hp = o * np.tanh(sp)
        hs.append(hp)
    return np.stack(hs), sp


def test_lstm_bwd_matches_torch_autograd_float64():
    rng = np.random.default_rng(11)
    d = orc.LstmShape(6, 4, 8, 12, 2, 4, 3)
    W, R, Wb, Rb = _plain_weights(rng, d, 0.4)
    b = _rand(rng, (4, d.K), 0.4)
    x = _rand(rng, (d.T, d.N, d.C))
    h0, s0 = _rand(rng, (d.N, d.K), 0.5), _rand(rng, (d.N, d.K), 0.5)
    dh, ds_last = _rand(rng, (d.T, d.N, d.K)), _rand(rng, (d.N, d.K))
    h, s, g = orc.lstm_fwd(d, x, Wb, Rb, b, h0, s0)
    dx, dW4, dR4, db, dh0, ds0 = orc.lstm_bwd(d, x, Wb, Rb, h0, s0, h, s, g, dh, ds_last)
    lstm = torch.nn.LSTM(d.C, d.K).double()
    order = [0, 2, 1, 3]  # torch rows: i, f, g(candidate), o  <- paper order i, c, f, o
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(torch.from_numpy(np.concatenate([W[j] for j in order])).double())
        lstm.weight_hh_l0.copy_(torch.from_numpy(np.concatenate([R[j] for j in order])).double())
        lstm.bias_ih_l0.copy_(torch.from_numpy(np.concatenate([b[j] for j in order])).double())
        lstm.bias_hh_l0.zero_()
    xt = torch.from_numpy(x).double().requires_grad_(True)
    h0t = torch.from_numpy(h0).double()[None].requires_grad_(True)
    s0t = torch.from_numpy(s0).double()[None].requires_grad_(True)
    out, (hn, cn) = lstm(xt, (h0t, s0t))
    loss = (out * torch.from_numpy(dh).double()).sum() + (cn[0] * torch.from_numpy(ds_last).double()).sum()
    loss.backward()
    unperm = lambda a, n: np.stack([a[order.index(j) * n:(order.index(j) + 1) * n] for j in range(4)])
    tW = unperm(lstm.weight_ih_l0.grad.numpy(), d.K)
    tR = unperm(lstm.weight_hh_l0.grad.numpy(), d.K)
    tb = unperm(lstm.bias_ih_l0.grad.numpy(), d.K)
    assert orc.rel_fro(dx, xt.grad.numpy()) < 1e-5
    assert orc.rel_fro(dh0, h0t.grad.numpy()[0]) < 1e-5
    assert orc.rel_fro(ds0, s0t.grad.numpy()[0]) < 1e-5
    assert orc.rel_fro(db, tb) < 1e-5
    assert orc.rel_fro(np.stack([orc.blocked_to_w2(dW4[j]) for j in range(4)]), tW) < 1e-5
    assert orc.rel_fro(np.stack([orc.blocked_to_w2(dR4[j]) for j in range(4)]), tR) < 1e-5


def test_lstm_bwd_matches_central_differences():
    """Directional derivatives of L = sum(dh * h) + sum(ds_last * s_T) by central differences in float64."""
    rng = np.random.default_rng(12)
    d = orc.LstmShape(3, 2, 4, 6, 2, 2, 3)
    W, R, Wb, Rb = _plain_weights(rng, d, 0.5)
    b = _rand(rng, (4, d.K), 0.3)
    x = _rand(rng, (d.T, d.N, d.C))
    h0, s0 = _rand(rng, (d.N, d.K), 0.5), _rand(rng, (d.N, d.K), 0.5)
    dh, ds_last = _rand(rng, (d.T, d.N, d.K)), _rand(rng, (d.N, d.K))
    h, s, g = orc.lstm_fwd(d, x, Wb, Rb, b, h0, s0)
    dx, dW4, dR4, db, dh0, ds0 = orc.lstm_bwd(d, x, Wb, Rb, h0, s0, h, s, g, dh, ds_last)
    dWp = np.stack([orc.blocked_to_w2(dW4[j]) for j in range(4)])
    dRp = np.stack([orc.blocked_to_w2(dR4[j]) for j in range(4)])
    f64 = lambda a: np.asarray(a, np.float64)
    args = [f64(x), f64(W), f64(R), f64(b), f64(h0), f64(s0)]
    grads = [dx, dWp, dRp, db, dh0, ds0]

    def loss(a):
        hs, sT = _np_lstm_fwd64(*a)
        return float((hs * dh).sum() + (sT * ds_last).sum())

    eps = 1e-5
    for k in range(6):
        v = f64(_rand(rng, args[k].shape))               # random direction
        plus = [a.copy() for a in args]
        minus = [a.copy() for a in args]
        plus[k] += eps * v
        minus[k] -= eps * v
        fd = (loss(plus) - loss(minus)) / (2 * eps)
        an = float((f64(grads[k]) * v).sum())
        assert abs(fd - an) <= 2e-5 * max(1.0, abs(an)), (k, fd, an)


def test_lstm_bf16_reading_against_an_explicit_float64_recurrence_with_torch_bf16_rounding():
    """oracle.lstm_fwd_bf16: h_t rounded to bf16 when stored and fed back rounded; cell state and gates not rounded.
    Pinned against the equations written out in torch float64 with torch's own bfloat16 cast as the quantiser."""
    import torch
    T, N, Cc, K = 5, 3, 16, 8
    rng = np.random.default_rng(77)
    d = orc.LstmShape(T, N, Cc, K, 16, 8, 4)
    q = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).float().numpy()
    x = q(rng.uniform(-1, 1, (T, N, Cc)))
    W = q(rng.uniform(-0.6, 0.6, (4, K, Cc)))
    R = q(rng.uniform(-0.6, 0.6, (4, K, K)))
    b = rng.uniform(-0.3, 0.3, (4, K)).astype(np.float32)
    h0 = q(rng.uniform(-0.5, 0.5, (N, K)))
    s0 = rng.uniform(-0.5, 0.5, (N, K)).astype(np.float32)
    W4 = np.stack([orc.w2_to_blocked(W[g], d.bc, d.bk) for g in range(4)])
    R4 = np.stack([orc.w2_to_blocked(R[g], d.bk, d.bk) for g in range(4)])
    h, s, g = orc.lstm_fwd_bf16(d, x, W4, R4, b, h0, s0)
    t64 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    hp, sp = t64(h0), t64(s0)
    flips = 0
    for t in range(T):
        z = [t64(x[t]) @ t64(W[k]).T + hp @ t64(R[k]).T + t64(b[k]) for k in range(4)]
        i, c, f, o = torch.sigmoid(z[0]), torch.tanh(z[1]), torch.sigmoid(z[2]), torch.sigmoid(z[3])
        st = f * sp + i * c
        ht = o * torch.tanh(st)
        hq = ht.float().to(torch.bfloat16).double()          # stored value: bf16
        assert np.array_equal(h[t], hq.numpy().astype(np.float32)), "h_t is the bf16 rounding of the step's result"
        assert np.allclose(s[t], st.numpy(), rtol=1e-6, atol=1e-7) and np.allclose(g[0, t], i.numpy(), rtol=1e-6, atol=1e-7)
        assert np.allclose(g[3, t], o.numpy(), rtol=1e-6, atol=1e-7) and np.allclose(g[1, t], c.numpy(), rtol=1e-6, atol=1e-7)
        flips += int((hq != ht).sum())
        hp, sp = hq, t64(s[t])                              # the rounded h and the fp32-stored state feed the next step
    assert flips > 0, "the rounding must matter in this test"
    # feeding the UNROUNDED h forward instead would give different later steps
    h_plain, _, _ = orc.lstm_fwd(d, x, W4, R4, b, h0, s0)
    assert not np.array_equal(orc.round_bf16(h_plain[-1]), h[-1])
