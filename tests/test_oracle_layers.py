"""Pins for the oracle's torso layers: each check is something the
mathematics fixes (brute force in another formulation, closed forms, special
cases that reduce to a library routine), never the oracle against itself."""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F


def brute_conv_padded(x, w, b, stride, same):
    """Independent fp64 statement: build an explicitly zero-padded image, then
    sum products over every window with no range tests."""
    x = np.asarray(x, np.float64)
    w = np.asarray(w, np.float64)
    H, W, Cin = x.shape
    k, _, _, Cout = w.shape
    if same:
        OH, OW = -(-H // stride), -(-W // stride)
        th = max((OH - 1) * stride + k - H, 0)
        tw = max((OW - 1) * stride + k - W, 0)
        pt, pl = th // 2, tw // 2
        xp = np.zeros((H + th, W + tw, Cin))
        xp[pt:pt + H, pl:pl + W] = x
    else:
        OH, OW = (H - k) // stride + 1, (W - k) // stride + 1
        xp = x
    y = np.zeros((OH, OW, Cout))
    for oh, ow, co in itertools.product(range(OH), range(OW), range(Cout)):
        win = xp[oh * stride:oh * stride + k, ow * stride:ow * stride + k, :]
        y[oh, ow, co] = (win * w[:, :, :, co]).sum() + (0.0 if b is None else b[co])
    return y


@pytest.mark.parametrize("H,W,Cin,Cout,k,s,same", [
    (5, 6, 2, 3, 1, 1, 0), (5, 6, 2, 3, 3, 1, 0), (7, 9, 3, 2, 4, 2, 0), (9, 8, 1, 4, 3, 2, 0),
    (5, 6, 2, 3, 3, 1, 1), (4, 7, 3, 5, 3, 1, 1), (6, 6, 2, 2, 3, 2, 1), (12, 11, 4, 3, 8, 4, 0),
])
def test_conv_matches_brute_force(orc, orc64, H, W, Cin, Cout, k, s, same):
    rng = np.random.default_rng(H * 100 + W * 10 + k)
    x = rng.standard_normal((H, W, Cin))
    w = rng.standard_normal((k, k, Cin, Cout))
    b = rng.standard_normal(Cout)
    ref = brute_conv_padded(x, w, b, s, same)
    y64 = orc64.conv2d(x, w, b, s, same)
    assert y64.shape == ref.shape
    np.testing.assert_allclose(y64, ref, rtol=1e-12, atol=1e-12)
    # the f32 build sees fp32-rounded inputs; compare on those
    xf, wf, bf = (a.astype(np.float32) for a in (x, w, b))
    ref32 = brute_conv_padded(xf, wf, bf, s, same)
    np.testing.assert_allclose(orc.conv2d(xf, wf, bf, s, same), ref32, rtol=2e-6, atol=2e-6)


def test_conv_1x1_is_per_pixel_matmul(orc64):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((4, 5, 6))
    w = rng.standard_normal((1, 1, 6, 3))
    b = rng.standard_normal(3)
    y = orc64.conv2d(x, w, b, 1, 0)
    np.testing.assert_allclose(y, x @ w[0, 0] + b, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("kh,kw", [(0, 0), (0, 2), (1, 1), (2, 0), (2, 2)])
def test_conv_delta_kernel_is_shift(orc64, kh, kw):
    """A kernel that is 1 at one tap copies the input shifted by that tap
    (cross-correlation: tap (kh,kw) reads x[oh+kh-1, ow+kw-1]); a flipped
    (true convolution) kernel would shift the other way and fail here."""
    rng = np.random.default_rng(2)
    x = rng.standard_normal((6, 7, 2))
    w = np.zeros((3, 3, 2, 2))
    w[kh, kw, 0, 1] = 1.0    # input channel 0 -> output channel 1 (pins I/O order too)
    y = orc64.conv2d(x, w, None, 1, 1)
    exp = np.zeros((6, 7))
    for oh in range(6):
        for ow in range(7):
            ih, iw = oh + kh - 1, ow + kw - 1
            if 0 <= ih < 6 and 0 <= iw < 7:
                exp[oh, ow] = x[ih, iw, 0]
    np.testing.assert_array_equal(y[:, :, 1], exp)
    np.testing.assert_array_equal(y[:, :, 0], 0)


def test_conv_ones_counts_in_range_taps(orc64):
    """all-ones input and kernel: SAME output = number of in-range taps
    (9 inside, 6 on edges, 4 at corners); VALID output = k*k*Cin everywhere."""
    x = np.ones((5, 6, 2))
    w = np.ones((3, 3, 2, 1))
    y = orc64.conv2d(x, w, None, 1, 1)[:, :, 0] / 2
    assert y[0, 0] == 4 and y[0, 3] == 6 and y[2, 0] == 6 and y[2, 2] == 9 and y[4, 5] == 4
    yv = orc64.conv2d(x, w, None, 1, 0)
    assert yv.shape == (3, 4, 1) and np.all(yv == 18)


def test_output_size_closed_forms(orc):
    # Appendix A.3.1 stack on 84x84: 8/4 -> 20, 4/2 -> 9, 3/1 -> 7
    n = 84
    got = []
    for k, s in ((8, 4), (4, 2), (3, 1)):
        n = orc.out_size(n, k, s, 0)
        got.append(n)
    assert got == [20, 9, 7]
    # stride-2 SAME pooling halves with ceil: 72->36->18->9->5, 96->48->24->12->6
    h, w, hs, ws = 72, 96, [], []
    for _ in range(4):
        h, w = orc.out_size(h, 3, 2, 1), orc.out_size(w, 3, 2, 1)
        hs.append(h), ws.append(w)
    assert hs == [36, 18, 9, 5] and ws == [48, 24, 12, 6]


@pytest.mark.parametrize("k,s,same", [(8, 4, 0), (4, 2, 0), (3, 1, 0), (3, 1, 1)])
def test_conv_matches_torch_fp64(orc64, k, s, same):
    rng = np.random.default_rng(k)
    x = rng.standard_normal((17, 19, 5))
    w = rng.standard_normal((k, k, 5, 7))
    b = rng.standard_normal(7)
    y = orc64.conv2d(x, w, b, s, same)
    t = F.conv2d(torch.from_numpy(x).permute(2, 0, 1)[None], torch.from_numpy(w).permute(3, 2, 0, 1),
                 torch.from_numpy(b), stride=s, padding=1 if same else 0)
    np.testing.assert_allclose(y, t[0].permute(1, 2, 0).numpy(), rtol=1e-11, atol=1e-11)


def brute_pool(x):
    """TF-style SAME 3x3/2 pooling via explicit -inf padding (extra cell on
    the bottom/right when the total padding is odd)."""
    H, W, C = x.shape
    OH, OW = -(-H // 2), -(-W // 2)
    th, tw = max((OH - 1) * 2 + 3 - H, 0), max((OW - 1) * 2 + 3 - W, 0)
    xp = np.full((H + th, W + tw, C), -np.inf)
    xp[th // 2:th // 2 + H, tw // 2:tw // 2 + W] = x
    y = np.empty((OH, OW, C))
    for oh in range(OH):
        for ow in range(OW):
            y[oh, ow] = xp[2 * oh:2 * oh + 3, 2 * ow:2 * ow + 3].reshape(9, C).max(0)
    return y


@pytest.mark.parametrize("H,W", [(4, 6), (9, 12), (5, 5), (8, 7), (1, 1), (2, 3)])
def test_maxpool_brute_force(orc64, H, W):
    rng = np.random.default_rng(H * 10 + W)
    x = rng.standard_normal((H, W, 3))
    np.testing.assert_array_equal(orc64.maxpool(x), brute_pool(x))
    # all-negative input: a zero pad cell must never win
    xn = -np.abs(x) - 1.0
    y = orc64.maxpool(xn)
    assert np.all(y < 0)
    np.testing.assert_array_equal(y, brute_pool(xn))
    # shift equivariance
    np.testing.assert_allclose(orc64.maxpool(x + 3.5), orc64.maxpool(x) + 3.5, rtol=0, atol=1e-15)


def test_maxpool_window_alignment(orc64):
    """Even size (pad 0 before, 1 after): window of output 0 is rows 0..2;
    odd size 9 -> 5 (pad 1 before): window of output 0 is rows -1..1."""
    x = np.arange(8, dtype=np.float64)[::-1].reshape(8, 1, 1).copy()   # decreasing: max = first in-range row
    y = orc64.maxpool(np.broadcast_to(x, (8, 2, 1)).copy())
    assert y[:, 0, 0].tolist() == [7, 5, 3, 1]
    x9 = np.arange(9, dtype=np.float64).reshape(9, 1, 1)               # increasing: max = last in-range row
    y9 = orc64.maxpool(np.broadcast_to(x9, (9, 2, 1)).copy())
    assert y9[:, 0, 0].tolist() == [1, 3, 5, 7, 8]


def test_maxpool_matches_torch(orc64):
    rng = np.random.default_rng(5)
    for H, W in ((72, 96), (9, 12)):
        x = rng.standard_normal((H, W, 2))
        OH, OW = -(-H // 2), -(-W // 2)
        th, tw = (OH - 1) * 2 + 3 - H, (OW - 1) * 2 + 3 - W
        t = F.pad(torch.from_numpy(x).permute(2, 0, 1)[None], (tw // 2, tw - tw // 2, th // 2, th - th // 2),
                  value=float("-inf"))
        t = F.max_pool2d(t, 3, 2)[0].permute(1, 2, 0).numpy()
        np.testing.assert_array_equal(orc64.maxpool(x), t)


def test_relu(orc64):
    x = np.array([-2.0, -0.0, 0.0, 1e-30, 3.0])
    np.testing.assert_array_equal(orc64.relu(x), [0, 0, 0, 1e-30, 3.0])


def test_residual_block_zero_weights_is_identity(orc64):
    """With zero kernels and biases the block returns x itself, negative
    entries included: the skip adds the un-rectified input."""
    rng = np.random.default_rng(7)
    x = rng.standard_normal((5, 4, 3))
    w = np.zeros(2 * (9 * 9 + 3))
    np.testing.assert_array_equal(orc64.residual_block(x, w), x)


def test_residual_block_composition(orc64):
    """Against torch fp64: x + conv_b(relu(conv_a(relu(x))))."""
    rng = np.random.default_rng(8)
    Cc = 4
    x = rng.standard_normal((6, 7, Cc))
    wa, wb = rng.standard_normal((3, 3, Cc, Cc)), rng.standard_normal((3, 3, Cc, Cc))
    ba, bb = rng.standard_normal(Cc), rng.standard_normal(Cc)
    flat = np.concatenate([wa.ravel(), ba, wb.ravel(), bb])
    tx = torch.from_numpy(x).permute(2, 0, 1)[None]
    conv = lambda t, w, b: F.conv2d(t, torch.from_numpy(w).permute(3, 2, 0, 1), torch.from_numpy(b), padding=1)
    ty = tx + conv(F.relu(conv(F.relu(tx), wa, ba)), wb, bb)
    np.testing.assert_allclose(orc64.residual_block(x, flat), ty[0].permute(1, 2, 0).numpy(), rtol=1e-11, atol=1e-11)
    # a block whose second bias is the only non-zero parameter adds that bias
    flat0 = np.zeros_like(flat)
    flat0[-Cc:] = bb
    np.testing.assert_allclose(orc64.residual_block(x, flat0), x + bb, rtol=0, atol=1e-15)


def test_dense_selector_pins_row_major_in_out(orc64):
    x = np.arange(1.0, 7.0)
    w = np.zeros((6, 4))
    w[4, 2] = 1.0
    y = orc64.dense(x, w, np.array([0.5, 0.5, 0.5, 0.5]))
    np.testing.assert_array_equal(y, [0.5, 0.5, 5.5, 0.5])
    rng = np.random.default_rng(9)
    x, w, b = rng.standard_normal(33), rng.standard_normal((33, 9)), rng.standard_normal(9)
    np.testing.assert_allclose(orc64.dense(x, w, b), x @ w + b, rtol=1e-12, atol=1e-12)


def test_normalise(orc, orc64):
    obs = np.array([0, 1, 128, 255], np.uint8)
    np.testing.assert_array_equal(orc64.normalise(obs), np.array([0, 1, 128, 255]) / 255.0)
    np.testing.assert_array_equal(orc.normalise(obs), (np.array([0, 1, 128, 255], np.float32) / np.float32(255)))
    assert orc64.normalise(obs)[3] == 1.0
