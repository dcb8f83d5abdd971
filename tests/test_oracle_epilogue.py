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
