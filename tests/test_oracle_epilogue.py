"""Pins for the fused-tail oracle (``oracle/epilogue.py``)."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import ConvShape
from oracle import epilogue as E


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_hand_example():
    # 1x1 convolution of one pixel: y_k = sum_c x_c w_kc + b_k, then the negative ones are cut
    s = ConvShape(1, 1, 1, 2, 3, 1, 1)
    x = np.array([1.0, -2.0]).reshape(1, 1, 1, 2)
    w = np.array([[1.0, 1.0], [3.0, 0.5], [0.0, 2.0]]).reshape(3, 1, 1, 2)
    b = np.array([0.5, -1.0, 10.0])
    assert np.array_equal(E.conv_fwd_bias_relu(s, x, w, b, False).ravel(), [-0.5, 1.0, 6.0])
    assert np.array_equal(E.conv_fwd_bias_relu(s, x, w, b, True).ravel(), [0.0, 1.0, 6.0])
    assert np.array_equal(E.conv_fwd_bias_relu(s, x, w, None, True).ravel(), [0.0, 2.0, 0.0])


def test_matches_library():
    for (g, relu) in [((2, 9, 11, 3, 4, 3, 3, 1, 1, 1), True), ((1, 12, 10, 4, 5, 3, 3, 2, 2, 2), True),
                      ((1, 8, 8, 6, 2, 1, 1, 1, 0, 1), False)]:
        s = ConvShape(*g)
        x, w, b = _rand(1, s.N, s.H, s.W, s.C), _rand(2, s.K, s.R, s.S, s.C), _rand(3, s.K)
        y = E.conv_fwd_bias_relu(s, x, w, b, relu)
        yt = F.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2), torch.from_numpy(w).permute(0, 3, 1, 2),
                      bias=torch.from_numpy(b), stride=s.stride, padding=s.pad, dilation=s.dil)
        if relu:
            yt = F.relu(yt)
        assert np.allclose(y, yt.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-12)


def test_properties_and_single_elements(oracle):
    s = ConvShape(2, 7, 9, 5, 6, 3, 3, 1, 1, 1)
    x, w, b = _rand(4, 2, 7, 9, 5), _rand(5, 6, 3, 3, 5), _rand(6, 6)
    plain = oracle.conv_fwd(s, x, w)
    assert np.array_equal(E.conv_fwd_bias_relu(s, x, w), plain)                     # no tail: the convolution itself
    y = E.conv_fwd_bias_relu(s, x, w, b, True)
    assert y.min() >= 0.0 and np.array_equal(y > 0, (plain + b) > 0)
    assert np.array_equal(E.conv_fwd_bias_relu(s, x, w, 1e9 * np.ones(6), True), plain + 1e9)   # nothing is cut
    assert not E.conv_fwd_bias_relu(s, x, w, -1e9 * np.ones(6), True).any()         # everything is cut
    idx = np.random.default_rng(7).integers(0, y.size, 300)
    x32, w32 = x.astype(np.float32), w.astype(np.float32)
    ref = E.conv_fwd_bias_relu(s, x32.astype(np.float64), w32.astype(np.float64), b, True).ravel()[idx]
    assert np.allclose(E.conv_fwd_bias_relu_at(s, x32, w32, b, True, idx), ref, rtol=0, atol=1e-13)


def test_tail_backward_hand_example():
    y = np.array([[1.0, 0.0, 2.0], [0.0, 3.0, 0.5]])
    dy = np.array([[10.0, 20.0, 30.0], [1.0, 2.0, 3.0]])
    dz, db = E.bias_relu_bwd(dy, y, True)
    assert np.array_equal(dz, [[10.0, 0.0, 30.0], [0.0, 2.0, 3.0]])
    assert np.array_equal(db, [10.0, 2.0, 33.0])
    dz, db = E.bias_relu_bwd(dy, y, False)
    assert np.array_equal(dz, dy) and np.array_equal(db, [11.0, 22.0, 33.0])


def test_tail_backward_against_autograd(oracle):
    s = ConvShape(2, 7, 9, 5, 6, 3, 3, 1, 1, 1)
    x, w, b = _rand(20, 2, 7, 9, 5), _rand(21, 6, 3, 3, 5), _rand(22, 6)
    dy = _rand(23, 2, 7, 9, 6)
    y = E.conv_fwd_bias_relu(s, x, w, b, True)
    dz, db = E.bias_relu_bwd(dy, y, True)
    xt = torch.from_numpy(x).permute(0, 3, 1, 2).requires_grad_(True)
    wt = torch.from_numpy(w).permute(0, 3, 1, 2).contiguous().requires_grad_(True)
    bt = torch.from_numpy(b).requires_grad_(True)
    yt = F.relu(F.conv2d(xt, wt, bias=bt, padding=1))
    yt.backward(torch.from_numpy(dy).permute(0, 3, 1, 2))
    assert np.allclose(db, bt.grad.numpy(), rtol=0, atol=1e-12)
    # dz is what the convolution's own gradients take: chain it through the oracle's data and filter gradients
    assert np.allclose(oracle.conv_bwd_data(s, dz, w), xt.grad.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-11)
    assert np.allclose(oracle.conv_bwd_filter(s, x, dz), wt.grad.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-11)


def test_residual_hand_example_and_library():
    # the hand example above with a residual of (1, -3, -20): sums (-0.5, 1, 6) + r = (0.5, -2, -14)
    s = ConvShape(1, 1, 1, 2, 3, 1, 1)
    x = np.array([1.0, -2.0]).reshape(1, 1, 1, 2)
    w = np.array([[1.0, 1.0], [3.0, 0.5], [0.0, 2.0]]).reshape(3, 1, 1, 2)
    b = np.array([0.5, -1.0, 10.0])
    r = np.array([1.0, -3.0, -20.0]).reshape(1, 1, 1, 3)
    assert np.array_equal(E.conv_fwd_bias_add_relu(s, x, w, b, r, False).ravel(), [0.5, -2.0, -14.0])
    assert np.array_equal(E.conv_fwd_bias_add_relu(s, x, w, b, r, True).ravel(), [0.5, 0.0, 0.0])
    assert np.array_equal(E.conv_fwd_bias_add_relu(s, x, w, None, r, True).ravel(), [0.0, 0.0, 0.0])    # (-1, 2, -4) + r
    # a ResNet block's tail against torch: relu(conv(x) + b + skip), float64
    s = ConvShape(2, 9, 11, 8, 12, 1, 1, 1, 0, 1)
    x, w, b = _rand(11, s.N, s.H, s.W, s.C), _rand(12, s.K, 1, 1, s.C), _rand(13, s.K)
    skip = _rand(14, s.N, s.H, s.W, s.K)
    y = E.conv_fwd_bias_add_relu(s, x, w, b, skip, True)
    yt = F.relu(F.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2), torch.from_numpy(w).permute(0, 3, 1, 2),
                         bias=torch.from_numpy(b)) + torch.from_numpy(skip).permute(0, 3, 1, 2))
    assert np.allclose(y, yt.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-12)
    # no residual: the plain fused tail; a huge negative residual cuts everything; single elements agree
    assert np.array_equal(E.conv_fwd_bias_add_relu(s, x, w, b, None, True), E.conv_fwd_bias_relu(s, x, w, b, True))
    assert not E.conv_fwd_bias_add_relu(s, x, w, b, -1e9 * np.ones_like(skip), True).any()
    idx = np.random.default_rng(15).integers(0, y.size, 200)
    x32, w32, r32 = x.astype(np.float32), w.astype(np.float32), skip.astype(np.float32)
    ref = E.conv_fwd_bias_add_relu(s, x32.astype(np.float64), w32.astype(np.float64), b, r32.astype(np.float64), True).ravel()[idx]
    assert np.allclose(E.conv_fwd_bias_add_relu_at(s, x32, w32, b, r32, True, idx), ref, rtol=0, atol=1e-13)
