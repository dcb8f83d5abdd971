"""Pins for the transposed-convolution oracle (``oracle/transpose.py``): a
worked example, closed forms, a library routine, the scatter-form data
gradient written independently in C, adjoint and linearity identities.  None
of these call the GPU path."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import ConvShape
from oracle import transpose as T


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def _torch_transpose(s, x, w, P, Q):
    """torch's conv_transpose2d on the same data: NCHW, weight [in, out, R, S]."""
    st = (s.stride, s.stride if s.stride_w is None else s.stride_w)
    pad = (s.pad, s.pad if s.pad_w is None else s.pad_w)
    dil = (s.dil, s.dil if s.dil_w is None else s.dil_w)
    base = ((P - 1) * st[0] - 2 * pad[0] + dil[0] * (s.R - 1) + 1, (Q - 1) * st[1] - 2 * pad[1] + dil[1] * (s.S - 1) + 1)
    opad = (s.H - base[0], s.W - base[1])
    xt = torch.from_numpy(x).permute(0, 3, 1, 2).contiguous().requires_grad_(True)
    wt = torch.from_numpy(w).permute(0, 3, 1, 2).contiguous().requires_grad_(True)        # [K, C, R, S]
    y = F.conv_transpose2d(xt, wt, stride=st, padding=pad, output_padding=opad, dilation=dil)
    return xt, wt, y


# ---- 1. a worked example small enough to add up by hand ------------------------
def test_worked_example_stride_2_ones_filter(oracle):
    # each input value is stamped as a 3x3 block at (2p, 2q); overlapping stamps add
    s = ConvShape(1, 5, 5, 1, 1, 3, 3, 2, 0, 1)
    assert oracle.out_shape(s) == (2, 2)
    x = np.array([[1.0, 2.0], [3.0, 4.0]]).reshape(1, 2, 2, 1)
    y = T.conv_transpose_fwd(s, x, np.ones((1, 3, 3, 1)))[0, :, :, 0]
    expect = np.array([[1, 1, 3, 2, 2],
                       [1, 1, 3, 2, 2],
                       [4, 4, 10, 6, 6],
                       [3, 3, 7, 4, 4],
                       [3, 3, 7, 4, 4]], dtype=np.float64)
    assert np.array_equal(y, expect)


def test_worked_example_with_padding_crops_the_border(oracle):
    # pad 1 removes one ring of the unpadded result above
    s = ConvShape(1, 3, 3, 1, 1, 3, 3, 2, 1, 1)
    assert oracle.out_shape(s) == (2, 2)
    x = np.array([[1.0, 2.0], [3.0, 4.0]]).reshape(1, 2, 2, 1)
    y = T.conv_transpose_fwd(s, x, np.ones((1, 3, 3, 1)))[0, :, :, 0]
    assert np.array_equal(y, np.array([[1, 3, 2], [4, 10, 6], [3, 7, 4]], dtype=np.float64))


# ---- 2. closed forms -------------------------------------------------------------
def test_1x1_stride_2_places_scaled_inputs_on_even_pixels(oracle):
    s = ConvShape(2, 9, 12, 3, 4, 1, 1, 2, 0, 1)       # P = 5, Q = 6; H = 9 is the tight size, W = 12 one more
    P, Q = oracle.out_shape(s)
    assert (P, Q) == (5, 6)
    x, w = _rand(1, 2, P, Q, 4), _rand(2, 4, 1, 1, 3)
    y = T.conv_transpose_fwd(s, x, w)
    expect = np.zeros((2, 9, 12, 3))
    expect[:, ::2, ::2, :][:, :P, :Q, :] = np.einsum("npqk,kc->npqc", x, w[:, 0, 0, :])
    assert np.allclose(y, expect, rtol=0, atol=1e-14)


def test_delta_filter_tap_is_a_strided_shift(oracle):
    # only tap (r0, s0) non-zero: y[p*st - pad + r0*dil, q*st - pad + s0*dil] = x[p, q], nothing else
    for (st, pad, dil, r0, s0) in [(2, 1, 1, 0, 2), (2, 1, 1, 2, 1), (3, 2, 2, 1, 0), (1, 1, 1, 2, 2)]:
        s = ConvShape(1, 14, 15, 1, 1, 3, 3, st, pad, dil)
        P, Q = oracle.out_shape(s)
        x = _rand(3, 1, P, Q, 1)
        w = np.zeros((1, 3, 3, 1)); w[0, r0, s0, 0] = 1.0
        y = T.conv_transpose_fwd(s, x, w)[0, :, :, 0]
        expect = np.zeros((14, 15))
        for p in range(P):
            for q in range(Q):
                h, ww = p * st - pad + r0 * dil, q * st - pad + s0 * dil
                if 0 <= h < 14 and 0 <= ww < 15:
                    expect[h, ww] = x[0, p, q, 0]
        assert np.array_equal(y, expect)


def test_stride_1_is_a_correlation_with_the_mirrored_filter(oracle):
    # unit stride: no zeros are inserted, so the result is an ordinary convolution layer with the
    # filter mirrored, the channel roles exchanged and padding dil*(R-1) - pad
    for (R, pad, dil) in [(3, 1, 1), (3, 0, 1), (3, 2, 2), (5, 2, 1)]:
        s = ConvShape(2, 10, 11, 3, 4, R, R, 1, pad, dil)
        P, Q = oracle.out_shape(s)
        x, w = _rand(4, 2, P, Q, 4), _rand(5, 4, R, R, 3)
        y = T.conv_transpose_fwd(s, x, w)
        w_m = np.ascontiguousarray(w[:, ::-1, ::-1, :].transpose(3, 1, 2, 0))          # [C, R, S, K]
        plain = ConvShape(2, P, Q, 4, 3, R, R, 1, dil * (R - 1) - pad, dil)
        assert oracle.out_shape(plain) == (10, 11)
        assert np.allclose(y, oracle.conv_fwd(plain, x, w_m), rtol=0, atol=1e-12)


# ---- 3. the library routine and the independently written scatter form ----------
GRID = [
    # N, H, W, C, K, R, S, stride, pad, dil
    (2, 9, 11, 3, 4, 3, 3, 2, 1, 1),       # tight output size
    (2, 10, 12, 3, 4, 3, 3, 2, 1, 1),      # one more row and column ("output padding" 1)
    (1, 16, 18, 2, 5, 4, 4, 2, 1, 1),      # the 4x4 / stride 2 up-sampling layer
    (1, 13, 13, 2, 3, 3, 3, 3, 0, 1),
    (1, 15, 17, 3, 2, 3, 3, 2, 2, 2),
    (2, 8, 9, 4, 3, 2, 2, 2, 0, 1),
    (1, 12, 12, 2, 2, 5, 5, 1, 2, 1),
    (1, 11, 14, 3, 3, 3, 3, 2, 3, 1),      # padding beyond the filter's reach: the border is cropped
    (1, 7, 7, 8, 8, 1, 1, 1, 0, 1),
]


@pytest.mark.parametrize("g", GRID, ids=[str(g) for g in GRID])
def test_matches_library_and_scatter_form(oracle, g):
    s = ConvShape(*g)
    P, Q = oracle.out_shape(s)
    x, w = _rand(10, s.N, P, Q, s.K), _rand(11, s.K, s.R, s.S, s.C)
    y = T.conv_transpose_fwd(s, x, w)
    assert y.shape == (s.N, s.H, s.W, s.C)
    # (a) the scatter loop nest in oracle.c (adjoint of the forward convolution)
    assert np.allclose(y, oracle.conv_bwd_data(s, x, w), rtol=0, atol=1e-12)
    # (b) torch's conv_transpose2d in float64, where it can express the case
    base_h = (P - 1) * s.stride - 2 * s.pad + s.dil * (s.R - 1) + 1
    if 0 <= s.H - base_h < max(s.stride, s.dil):
        _, _, yt = _torch_transpose(s, x, w, P, Q)
        assert np.allclose(y, yt.detach().permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-12)
    # (c) single elements
    idx = np.random.default_rng(12).integers(0, y.size, 200)
    got = T.conv_transpose_fwd_at(s, x.astype(np.float32), w.astype(np.float32), idx)
    ref = T.conv_transpose_fwd(s, x.astype(np.float32).astype(np.float64), w.astype(np.float32).astype(np.float64))
    assert np.allclose(got, ref.ravel()[idx], rtol=0, atol=1e-12)


def test_rectangular_strides(oracle):
    s = ConvShape(1, 12, 13, 2, 3, 3, 2, 2, 1, 1, stride_w=3, pad_w=0, dil_w=2)
    P, Q = oracle.out_shape(s)
    x, w = _rand(20, 1, P, Q, 3), _rand(21, 3, 3, 2, 2)
    y = T.conv_transpose_fwd(s, x, w)
    assert np.allclose(y, oracle.conv_bwd_data(s, x, w), rtol=0, atol=1e-12)


# ---- 4. adjoint of the forward convolution ---------------------------------------
@pytest.mark.parametrize("g", GRID[:6], ids=[str(g) for g in GRID[:6]])
def test_is_the_adjoint_of_the_convolution(oracle, g):
    s = ConvShape(*g)
    P, Q = oracle.out_shape(s)
    u, v, w = _rand(30, s.N, s.H, s.W, s.C), _rand(31, s.N, P, Q, s.K), _rand(32, s.K, s.R, s.S, s.C)
    lhs = np.vdot(oracle.conv_fwd(s, u, w), v)
    rhs = np.vdot(u, T.conv_transpose_fwd(s, v, w))
    assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(lhs))


# ---- 5. gradients -----------------------------------------------------------------
@pytest.mark.parametrize("g", GRID[:5], ids=[str(g) for g in GRID[:5]])
def test_gradients_against_autograd_and_linearity(oracle, g):
    s = ConvShape(*g)
    P, Q = oracle.out_shape(s)
    x, w, dy = _rand(40, s.N, P, Q, s.K), _rand(41, s.K, s.R, s.S, s.C), _rand(42, s.N, s.H, s.W, s.C)
    dx = T.conv_transpose_bwd_data(s, dy, w)
    dw = T.conv_transpose_bwd_filter(s, x, dy)
    assert dx.shape == x.shape and dw.shape == w.shape
    # y = A(w) x is bilinear: <y, dy> = <x, dx> = <w, dw>
    inner = np.vdot(T.conv_transpose_fwd(s, x, w), dy)
    assert abs(np.vdot(x, dx) - inner) <= 1e-10 * max(1.0, abs(inner))
    assert abs(np.vdot(w, dw) - inner) <= 1e-10 * max(1.0, abs(inner))
    # library autograd
    xt, wt, yt = _torch_transpose(s, x, w, P, Q)
    yt.backward(torch.from_numpy(dy).permute(0, 3, 1, 2))
    assert np.allclose(dx, xt.grad.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-11)
    assert np.allclose(dw, wt.grad.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-11)


def test_filter_gradient_by_finite_differences(oracle):
    s = ConvShape(1, 8, 9, 2, 2, 3, 3, 2, 1, 1)
    P, Q = oracle.out_shape(s)
    x, w, dy = _rand(50, 1, P, Q, 2), _rand(51, 2, 3, 3, 2), _rand(52, 1, 8, 9, 2)
    dw = T.conv_transpose_bwd_filter(s, x, dy)
    for (k, r, s_, c) in [(0, 0, 0, 0), (1, 2, 1, 0), (0, 1, 2, 1)]:
        e = np.zeros_like(w); e[k, r, s_, c] = 1.0
        fd = np.vdot(T.conv_transpose_fwd(s, x, w + e) - T.conv_transpose_fwd(s, x, w - e), dy) / 2.0
        assert abs(fd - dw[k, r, s_, c]) <= 1e-10 * max(1.0, abs(fd))
