"""Pins for the oracle's recurrent core, heads and action selection."""
import math

import numpy as np
import pytest
import torch


def test_lstm_zero_weights_closed_form(orc64):
    """W = 0, b = 0: every gate pre-activation is 0, so i=f=o=1/2, tanh(g)=0:
    c' = c/2 and h' = tanh(c/2)/2."""
    F_, A, H = 3, 4, 5
    rng = np.random.default_rng(0)
    c = rng.standard_normal(H)
    h, cc = orc64.lstm_cell(rng.standard_normal(F_), 2, A, 0.7, rng.standard_normal(H), c,
                            np.zeros((F_ + A + 1 + H, 4 * H)), np.zeros(4 * H))
    np.testing.assert_allclose(cc, 0.5 * c, rtol=1e-15)
    np.testing.assert_allclose(h, 0.5 * np.tanh(0.5 * c), rtol=1e-15)


def test_lstm_gate_order_by_saturation(orc64):
    """Column blocks are [i|f|g|o].  Saturating one block at a time through
    the bias tells the blocks apart:
      f -> +inf, i -> -inf         : c' = c      (carry)
      i -> +inf, f -> -inf, g big  : c' = +1     (write)
      o -> -inf                    : h' = 0
    """
    F_, A, H = 2, 3, 4
    Wz = np.zeros((F_ + A + 1 + H, 4 * H))
    c = np.array([0.3, -1.2, 2.0, -0.1])
    feat, hin = np.ones(F_), np.ones(H)
    big = 50.0
    b = np.zeros(4 * H); b[0:H] = -big; b[H:2 * H] = big
    h, cc = orc64.lstm_cell(feat, 0, A, 0.0, hin, c, Wz, b)
    np.testing.assert_allclose(cc, c, rtol=1e-15)
    np.testing.assert_allclose(h, 0.5 * np.tanh(c), rtol=1e-15)
    b = np.zeros(4 * H); b[0:H] = big; b[H:2 * H] = -big; b[2 * H:3 * H] = big
    h, cc = orc64.lstm_cell(feat, 0, A, 0.0, hin, c, Wz, b)
    np.testing.assert_allclose(cc, np.ones(H), rtol=1e-12)
    b = np.zeros(4 * H); b[3 * H:] = -big
    h, cc = orc64.lstm_cell(feat, 0, A, 0.0, hin, c, Wz, b)
    assert np.all(np.abs(h) < 1e-20)


def test_lstm_hand_worked_single_unit(orc64):
    """H = 1, F = 1, A = 2, worked by hand from the definition."""
    feat, a_prev, r, h0, c0 = 0.5, 1, -2.0, 0.25, 0.75
    # rows: feat, onehot0, onehot1, reward, h ; columns i,f,g,o
    W = np.array([[0.1, 0.2, 0.3, 0.4],
                  [9.0, 9.0, 9.0, 9.0],      # action 0 row: must NOT be used
                  [0.5, -0.5, 0.25, -0.25],
                  [0.2, 0.1, -0.1, -0.2],
                  [1.0, -1.0, 0.5, 2.0]])
    b = np.array([0.01, 0.02, 0.03, 0.04])
    pre = feat * W[0] + W[2] + r * W[3] + h0 * W[4] + b
    sg = lambda v: 1 / (1 + math.exp(-v))
    c1 = sg(pre[1]) * c0 + sg(pre[0]) * math.tanh(pre[2])
    h1 = sg(pre[3]) * math.tanh(c1)
    h, c = orc64.lstm_cell([feat], a_prev, 2, r, [h0], [c0], W, b)
    assert abs(c[0] - c1) < 1e-15 and abs(h[0] - h1) < 1e-15


def test_lstm_matches_torch_cell_and_dense_onehot(orc64):
    """torch.nn.LSTMCell in fp64 uses the same gate order (i,f,g,o); feeding it
    the explicit dense [feat, one-hot, reward] vector pins the one-hot rows,
    the reward row and the h rows of the stacked matrix."""
    rng = np.random.default_rng(3)
    F_, A, H = 6, 5, 7
    Z = F_ + A + 1
    W = rng.standard_normal((Z + H, 4 * H)) * 0.4
    b = rng.standard_normal(4 * H) * 0.1
    feat, hin, cin = rng.standard_normal(F_), rng.standard_normal(H), rng.standard_normal(H)
    a_prev, r = 3, 1.7
    cell = torch.nn.LSTMCell(Z, H).double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(W[:Z].T))
        cell.weight_hh.copy_(torch.from_numpy(W[Z:].T))
        cell.bias_ih.copy_(torch.from_numpy(b))
        cell.bias_hh.zero_()
        z = np.concatenate([feat, np.eye(A)[a_prev], [r]])
        th, tc = cell(torch.from_numpy(z)[None], (torch.from_numpy(hin)[None], torch.from_numpy(cin)[None]))
    h, c = orc64.lstm_cell(feat, a_prev, A, r, hin, cin, W, b)
    np.testing.assert_allclose(h, th[0].numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(c, tc[0].numpy(), rtol=1e-12, atol=1e-13)
    # out-of-range previous action = all-zero one-hot
    h2, c2 = orc64.lstm_cell(feat, -1, A, r, hin, cin, W, b)
    with torch.no_grad():
        z0 = np.concatenate([feat, np.zeros(A), [r]])
        th0, tc0 = cell(torch.from_numpy(z0)[None], (torch.from_numpy(hin)[None], torch.from_numpy(cin)[None]))
    np.testing.assert_allclose(h2, th0[0].numpy(), rtol=1e-12, atol=1e-13)
    h3, _ = orc64.lstm_cell(feat, A, A, r, hin, cin, W, b)
    np.testing.assert_array_equal(h3, h2)


def test_policy_value_head(orc64):
    rng = np.random.default_rng(4)
    n, A = 9, 5
    wp, bp, wv, bv = rng.standard_normal((n, A)), rng.standard_normal(A), rng.standard_normal(n), rng.standard_normal(1)
    core = rng.standard_normal(n)
    logits, v = orc64.head_policy_value(core, A, np.concatenate([wp.ravel(), bp, wv, bv]))
    np.testing.assert_allclose(logits, core @ wp + bp, rtol=1e-12)
    assert abs(v - (core @ wv + bv[0])) < 1e-12


def _dueling_flat(rng, n, hid, A):
    parts = dict(w1v=rng.standard_normal((n, hid)), b1v=rng.standard_normal(hid), w2v=rng.standard_normal(hid),
                 b2v=rng.standard_normal(1), w1a=rng.standard_normal((n, hid)), b1a=rng.standard_normal(hid),
                 w2a=rng.standard_normal((hid, A)), b2a=rng.standard_normal(A))
    flat = np.concatenate([parts[k].ravel() for k in ("w1v", "b1v", "w2v", "b2v", "w1a", "b1a", "w2a", "b2a")])
    return parts, flat


def test_dueling_invariants(orc64):
    rng = np.random.default_rng(5)
    n, hid, A = 6, 8, 4
    p, flat = _dueling_flat(rng, n, hid, A)
    core = rng.standard_normal(n)
    q, v = orc64.head_dueling(core, hid, A, flat)
    # mean over actions of Q is the value stream
    assert abs(q.mean() - v) < 1e-13
    # explicit formula
    V = np.maximum(core @ p["w1v"] + p["b1v"], 0) @ p["w2v"] + p["b2v"][0]
    Adv = np.maximum(core @ p["w1a"] + p["b1a"], 0) @ p["w2a"] + p["b2a"]
    np.testing.assert_allclose(q, V + Adv - Adv.mean(), rtol=1e-12, atol=1e-13)
    assert abs(v - V) < 1e-13
    # a constant added to every advantage leaves Q unchanged
    p2 = dict(p); p2["b2a"] = p["b2a"] + 3.25
    flat2 = np.concatenate([p2[k].ravel() for k in ("w1v", "b1v", "w2v", "b2v", "w1a", "b1a", "w2a", "b2a")])
    q2, v2 = orc64.head_dueling(core, hid, A, flat2)
    np.testing.assert_allclose(q2, q, rtol=0, atol=1e-13)


def test_softmax_invariants(orc64):
    rng = np.random.default_rng(6)
    l = rng.standard_normal(19) * 4
    p = orc64.softmax(l)
    assert abs(p.sum() - 1) < 1e-14 and np.all(p > 0)
    np.testing.assert_allclose(orc64.softmax(l + 100.0), p, rtol=1e-12)
    np.testing.assert_allclose(orc64.softmax(np.full(6, 2.5)), np.full(6, 1 / 6), rtol=1e-15)
    np.testing.assert_allclose(p, torch.softmax(torch.from_numpy(l), 0).numpy(), rtol=1e-12)
    # large logits do not overflow
    assert np.isfinite(orc64.softmax(np.array([1000.0, 999.0]))).all()


def test_greedy_ties_lowest_index(orc):
    a, m = orc.select_greedy(np.array([0.1, 0.7, 0.7, 0.3], np.float32))
    assert a == 1 and m == 0
    a, m = orc.select_greedy(np.array([2.0, -1.0, 0.5], np.float32))
    assert a == 0 and abs(m - 1.5) < 1e-7
    a, m = orc.select_greedy(np.array([-3.0, -3.0], np.float32))
    assert a == 0


def test_gumbel_forced_and_formula(orc, orc64):
    l = np.array([0.0, 5.0, -1.0])
    # u -> 1 on one entry gives it a huge positive Gumbel term: that action wins
    a, pert, _ = orc64.select_gumbel(l, np.array([0.5, 0.5, 1.0]))
    assert a == 2
    # u -> 0 clamps to FLT_MIN: finite, very negative perturbation
    a, pert, _ = orc64.select_gumbel(l, np.array([0.0, 0.5, 0.5]))
    assert np.isfinite(pert).all() and a == 1
    u = np.array([0.3, 0.6, 0.9])
    a, pert, m = orc64.select_gumbel(l, u)
    np.testing.assert_allclose(pert, l - np.log(-np.log(u)), rtol=1e-14)
    srt = np.sort(pert)
    assert a == int(np.argmax(pert)) and abs(m - (srt[-1] - srt[-2])) < 1e-14
    # the f32 build does the same in single precision
    a32, pert32, _ = orc.select_gumbel(l.astype(np.float32), u.astype(np.float32))
    np.testing.assert_allclose(pert32, pert, rtol=1e-6)
    assert a32 == a


@pytest.mark.parametrize("logits", [[0.0, 1.0], [1.5, -0.5, 0.3], [0.2, 0.1, -2.0, 1.0]])
def test_gumbel_max_law_is_softmax(orc, logits):
    """The law of argmax(logit + Gumbel) is softmax(logits): the same law an
    inverse-CDF sampler has.  (The two samplers consume different numbers of
    uniforms per draw, so only the distribution can be compared, not paths.)
    For A = 2 this is the closed form P(a=0) = sigmoid(l0 - l1)."""
    l = np.array(logits, np.float32)
    A = len(l)
    rng = np.random.default_rng(11)
    u = rng.random((20000, A), dtype=np.float32)
    # the oracle itself is called per draw (a 1e6-draw version through the batched
    # forward pass lives in test_oracle_forward.py)
    sub = 20000
    counts = np.zeros(A)
    for i in range(sub):
        a, _, _ = orc.select_gumbel(l, u[i])
        counts[a] += 1
    p = np.exp(l - l.max()); p /= p.sum()
    sd = np.sqrt(p * (1 - p) / sub)
    assert np.all(np.abs(counts / sub - p) < 5 * sd), (counts / sub, p)
    if A == 2:
        assert abs(p[0] - 1 / (1 + math.exp(-(l[0] - l[1])))) < 1e-7
    # inverse-CDF sampler on an independent stream has the same frequencies
    v = rng.random(sub)
    inv = np.searchsorted(np.cumsum(p), v)
    inv_counts = np.bincount(np.minimum(inv, A - 1), minlength=A)
    assert np.all(np.abs(inv_counts / sub - counts / sub) < 5 * np.sqrt(2) * sd + 1e-9)
