"""Pins for the convolution oracle: closed forms, brute force written a
different way, adjoint identities, GEMM special case, finite differences and
a textbook library routine.  None of these call the GPU path."""
import itertools

import numpy as np
import pytest

from oracle import ConvShape


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


# ---- 1. all-ones closed form: counts the taps that land inside the image ----
def _taps_in_bounds(P, H, R, st, pad, dil):
    p = np.arange(P)[:, None] * st - pad + np.arange(R)[None, :] * dil
    return ((p >= 0) & (p < H)).sum(axis=1)


@pytest.mark.parametrize("R,st,pad,dil", [(3, 1, 1, 1), (3, 1, 2, 2), (3, 1, 6, 6), (3, 1, 12, 12),
                                          (3, 1, 18, 18), (3, 2, 1, 1), (3, 2, 2, 2), (7, 2, 3, 1),
                                          (1, 1, 0, 1), (1, 2, 0, 1)])
def test_all_ones_counts_valid_taps(oracle, R, st, pad, dil):
    s = ConvShape(2, 20, 27, 3, 2, R, R, st, pad, dil)
    y = oracle.conv_fwd(s, np.ones((2, 20, 27, 3)), np.ones((2, R, R, 3)))
    P, Q = oracle.out_shape(s)
    expect = 3 * np.outer(_taps_in_bounds(P, 20, R, st, pad, dil), _taps_in_bounds(Q, 27, R, st, pad, dil))
    assert y.shape == (2, P, Q, 2)
    assert np.array_equal(y, np.broadcast_to(expect[None, :, :, None], y.shape))


def test_all_ones_3x3_same_padding_formula(oracle):
    # pad = dil = d on a 3x3: (3 - [p<d] - [p>=H-d]) * (3 - [q<d] - [q>=W-d]) * C
    for d in (1, 2, 6):
        H, W, C = 17, 23, 4
        s = ConvShape(1, H, W, C, 1, 3, 3, 1, d, d)
        y = oracle.conv_fwd(s, np.ones((1, H, W, C)), np.ones((1, 3, 3, C)))[0, :, :, 0]
        p, q = np.arange(H), np.arange(W)
        fp = 3 - (p < d) - (p >= H - d)
        fq = 3 - (q < d) - (q >= W - d)
        assert np.array_equal(y, C * np.outer(fp, fq))


def test_output_extent(oracle):
    assert oracle.out_shape(ConvShape(2, 768, 1152, 16, 64, 7, 7, 2, 3, 1)) == (384, 576)
    assert oracle.out_shape(ConvShape(1, 96, 144, 16, 64, 3, 3, 1, 2, 2)) == (96, 144)
    assert oracle.out_shape(ConvShape(2, 192, 288, 256, 512, 1, 1, 2, 0, 1)) == (96, 144)
    assert oracle.out_shape(ConvShape(2, 48, 72, 2048, 256, 3, 3, 1, 18, 18)) == (48, 72)
    assert oracle.out_shape(ConvShape(1, 5, 5, 1, 1, 3, 3, 1, 0, 1)) == (3, 3)
    assert oracle.out_shape(ConvShape(1, 5, 5, 1, 1, 3, 3, 1, 0, 2)) == (1, 1)
    with pytest.raises(ValueError):
        oracle.out_shape(ConvShape(1, 4, 4, 1, 1, 3, 3, 1, 0, 2))


# ---- 2. a delta filter shifts (and subsamples) the input ---------------------
@pytest.mark.parametrize("st,dil", [(1, 1), (1, 2), (2, 1), (2, 3)])
def test_delta_filter_is_a_shift(oracle, st, dil):
    H, W, C, K, R = 11, 13, 3, 2, 3
    pad = dil
    x = _rand(1, 1, H, W, C)
    s = ConvShape(1, H, W, C, K, R, R, st, pad, dil)
    P, Q = oracle.out_shape(s)
    for r0, s0, c0, k0 in [(0, 0, 0, 0), (2, 1, 1, 1), (1, 2, 2, 0)]:
        w = np.zeros((K, R, R, C))
        w[k0, r0, s0, c0] = 1.0
        y = oracle.conv_fwd(s, x, w)
        expect = np.zeros((1, P, Q, K))
        for p in range(P):
            for q in range(Q):
                h, ww = p * st - pad + r0 * dil, q * st - pad + s0 * dil
                if 0 <= h < H and 0 <= ww < W:
                    expect[0, p, q, k0] = x[0, h, ww, c0]
        assert np.array_equal(y, expect)


# ---- 3. brute force, written as padded shifted slices -----------------------
def _conv_by_slices(x, w, st, pad, dil):
    N, H, W, C = x.shape
    K, R, S, _ = w.shape
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, C))
    xp[:, pad:pad + H, pad:pad + W] = x
    P = (H + 2 * pad - dil * (R - 1) - 1) // st + 1
    Q = (W + 2 * pad - dil * (S - 1) - 1) // st + 1
    y = np.zeros((N, P, Q, K))
    for r in range(R):
        for s in range(S):
            win = xp[:, r * dil: r * dil + (P - 1) * st + 1: st, s * dil: s * dil + (Q - 1) * st + 1: st, :]
            y += win @ w[:, r, s, :].T
    return y


@pytest.mark.parametrize("st,dil,pad", list(itertools.product((1, 2), (1, 2), (0, 1, 2))))
def test_brute_force_tiny(oracle, st, dil, pad):
    x, w = _rand(2, 1, 7, 8, 2), _rand(3, 3, 3, 3, 2)
    s = ConvShape(1, 7, 8, 2, 3, 3, 3, st, pad, dil)
    np.testing.assert_allclose(oracle.conv_fwd(s, x, w), _conv_by_slices(x, w, st, pad, dil), rtol=0, atol=1e-13)


def test_brute_force_stem_like_and_rect_filter(oracle):
    x, w = _rand(4, 2, 12, 10, 3), _rand(5, 4, 7, 7, 3)
    s = ConvShape(2, 12, 10, 3, 4, 7, 7, 2, 3, 1)
    np.testing.assert_allclose(oracle.conv_fwd(s, x, w), _conv_by_slices(x, w, 2, 3, 1), rtol=0, atol=1e-12)
    # non-square filter and per-axis stride / pad / dilation: a hand-expanded single output
    s = ConvShape(1, 9, 11, 2, 1, 2, 3, stride=2, pad=1, dil=3, stride_w=1, pad_w=2, dil_w=2)
    x, w = _rand(6, 1, 9, 11, 2), _rand(7, 1, 2, 3, 2)
    y = oracle.conv_fwd(s, x, w)
    p, q = 2, 4
    acc = 0.0
    for r in range(2):
        for t in range(3):
            h, ww = p * 2 - 1 + r * 3, q * 1 - 2 + t * 2
            if 0 <= h < 9 and 0 <= ww < 11:
                acc += float(x[0, h, ww] @ w[0, r, t])
    assert abs(y[0, p, q, 0] - acc) < 1e-13


# ---- 4. adjoint identities ---------------------------------------------------
@pytest.mark.parametrize("R,st,pad,dil", [(3, 1, 1, 1), (3, 1, 2, 2), (3, 2, 1, 1), (7, 2, 3, 1),
                                          (1, 2, 0, 1), (3, 2, 3, 3), (3, 1, 6, 6)])
def test_adjoint_identities(oracle, R, st, pad, dil):
    s = ConvShape(2, 13, 14, 5, 4, R, R, st, pad, dil)
    P, Q = oracle.out_shape(s)
    x, w, dy = _rand(8, 2, 13, 14, 5), _rand(9, 4, R, R, 5), _rand(10, 2, P, Q, 4)
    lhs = np.vdot(dy, oracle.conv_fwd(s, x, w))
    via_dx = np.vdot(oracle.conv_bwd_data(s, dy, w), x)
    via_dw = np.vdot(oracle.conv_bwd_filter(s, x, dy), w)
    assert abs(lhs - via_dx) <= 1e-12 * abs(lhs)
    assert abs(lhs - via_dw) <= 1e-12 * abs(lhs)


# ---- 5. 1x1 convolution is a matrix product ---------------------------------
def test_1x1_is_gemm(oracle):
    x, w = _rand(11, 2, 6, 7, 16), _rand(12, 8, 1, 1, 16)
    s = ConvShape(2, 6, 7, 16, 8, 1, 1)
    np.testing.assert_allclose(oracle.conv_fwd(s, x, w),
                               (x.reshape(-1, 16) @ w.reshape(8, 16).T).reshape(2, 6, 7, 8), rtol=0, atol=1e-13)
    dy = _rand(13, 2, 6, 7, 8)
    np.testing.assert_allclose(oracle.conv_bwd_data(s, dy, w),
                               (dy.reshape(-1, 8) @ w.reshape(8, 16)).reshape(2, 6, 7, 16), rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.conv_bwd_filter(s, x, dy),
                               (dy.reshape(-1, 8).T @ x.reshape(-1, 16)).reshape(8, 1, 1, 16), rtol=0, atol=1e-12)
    # stride 2: the same product on the subsampled rows
    s2 = ConvShape(2, 6, 7, 16, 8, 1, 1, 2, 0, 1)
    xs = x[:, ::2, ::2, :]
    np.testing.assert_allclose(oracle.conv_fwd(s2, x, w),
                               (xs.reshape(-1, 16) @ w.reshape(8, 16).T).reshape(2, 3, 4, 8), rtol=0, atol=1e-13)


# ---- 6. finite differences ---------------------------------------------------
@pytest.mark.parametrize("R,st,pad,dil", [(3, 1, 2, 2), (3, 2, 1, 1), (7, 2, 3, 1)])
def test_finite_differences(oracle, R, st, pad, dil):
    s = ConvShape(1, 10, 9, 3, 2, R, R, st, pad, dil)
    P, Q = oracle.out_shape(s)
    x, w, dy = _rand(14, 1, 10, 9, 3), _rand(15, 2, R, R, 3), _rand(16, 1, P, Q, 2)
    dw = oracle.conv_bwd_filter(s, x, dy)
    dx = oracle.conv_bwd_data(s, dy, w)
    f = lambda xx, ww: float(np.vdot(dy, oracle.conv_fwd(s, xx, ww)))
    g = np.random.default_rng(17)
    eps = 1e-4
    for _ in range(12):
        i = tuple(g.integers(0, n) for n in w.shape)
        e = np.zeros_like(w); e[i] = eps
        fd = (f(x, w + e) - f(x, w - e)) / (2 * eps)
        assert abs(fd - dw[i]) <= 1e-7 * max(1.0, abs(dw[i]))
        j = tuple(g.integers(0, n) for n in x.shape)
        e = np.zeros_like(x); e[j] = eps
        fd = (f(x + e, w) - f(x - e, w)) / (2 * eps)
        assert abs(fd - dx[j]) <= 1e-7 * max(1.0, abs(dx[j]))


# ---- 7. textbook library routine (float64 torch on the CPU) -----------------
@pytest.mark.parametrize("R,st,pad,dil", [(3, 1, 1, 1), (3, 1, 2, 2), (3, 2, 1, 1), (7, 2, 3, 1), (1, 2, 0, 1),
                                          (3, 1, 6, 6)])
def test_against_torch_float64(oracle, R, st, pad, dil):
    import torch
    import torch.nn.functional as F
    s = ConvShape(2, 12, 15, 4, 6, R, R, st, pad, dil)
    P, Q = oracle.out_shape(s)
    x, w, dy = _rand(18, 2, 12, 15, 4), _rand(19, 6, R, R, 4), _rand(20, 2, P, Q, 6)
    xt = torch.tensor(x).permute(0, 3, 1, 2).requires_grad_(True)
    wt = torch.tensor(w).permute(0, 3, 1, 2).requires_grad_(True)
    yt = F.conv2d(xt, wt, stride=st, padding=pad, dilation=dil)
    yt.backward(torch.tensor(dy).permute(0, 3, 1, 2))
    np.testing.assert_allclose(oracle.conv_fwd(s, x, w), yt.detach().permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.conv_bwd_data(s, dy, w), xt.grad.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.conv_bwd_filter(s, x, dy), wt.grad.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-11)


# ---- 8. single-element variants agree with the full tensors -----------------
@pytest.mark.parametrize("R,st,pad,dil", [(3, 1, 2, 2), (3, 2, 1, 1), (7, 2, 3, 1), (1, 1, 0, 1), (1, 2, 0, 1)])
def test_point_evaluation_matches_full(oracle, R, st, pad, dil):
    s = ConvShape(2, 11, 12, 8, 5, R, R, st, pad, dil)
    P, Q = oracle.out_shape(s)
    x = _rand(21, 2, 11, 12, 8).astype(np.float32)
    w = _rand(22, 5, R, R, 8).astype(np.float32)
    dy = _rand(23, 2, P, Q, 5).astype(np.float32)
    y = oracle.conv_fwd(s, x, w).ravel()
    dx = oracle.conv_bwd_data(s, dy, w).ravel()
    dw = oracle.conv_bwd_filter(s, x, dy).ravel()
    np.testing.assert_allclose(oracle.conv_fwd_at(s, x, w, np.arange(y.size)), y, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.conv_bwd_data_at(s, dy, w, np.arange(dx.size)), dx, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.conv_bwd_filter_at(s, x, dy, np.arange(dw.size)), dw, rtol=0, atol=1e-12)


# ---- 9. stride-2 data gradient leaves untouched pixels at zero --------------
def test_strided_1x1_dgrad_is_zero_off_grid(oracle):
    s = ConvShape(1, 6, 6, 2, 3, 1, 1, 2, 0, 1)
    dy, w = _rand(24, 1, 3, 3, 3), _rand(25, 3, 1, 1, 2)
    dx = oracle.conv_bwd_data(s, dy, w)
    assert np.all(dx[:, 1::2] == 0) and np.all(dx[:, :, 1::2] == 0)
    np.testing.assert_allclose(dx[:, ::2, ::2], dy @ w.reshape(3, 2), rtol=0, atol=1e-14)
