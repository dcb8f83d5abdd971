"""Pins of the fused logits + loss oracle (``oracle/fused.py``) against things other
than itself: float64 autograd of torch through an independently written forward
(linear layer + torch's own cross-entropy), central finite differences, a hand
example, and invariants."""
import numpy as np
import pytest
import torch

from oracle.fused import logits_ce_fused


def _case(seed, n, C):
    rng = np.random.default_rng(seed)
    x = rng.normal(size=(n, C))
    w = rng.normal(size=(3, C)) / np.sqrt(C)
    labels = rng.integers(0, 3, size=n).astype(np.uint8)
    cw = np.array([1.0, 7.5, 31.0])
    return x, w, labels, cw


def test_hand_example():
    # one pixel, two channels: z = (1, 0, -1); label 0, weight 2, scale 0.5
    x = np.array([[1.0, 2.0]])
    w = np.array([[1.0, 0.0], [0.0, 0.0], [-1.0, 0.0]])
    z, loss, dz, dx, dw = logits_ce_fused(x, w, np.array([0], dtype=np.uint8), np.array([2.0, 1.0, 1.0]), 0.5)
    e = np.exp([1.0, 0.0, -1.0])
    p = e / e.sum()
    assert np.allclose(z, [[1.0, 0.0, -1.0]])
    assert np.isclose(loss, 0.5 * 2.0 * -np.log(p[0]))
    g = 0.5 * 2.0 * (p - np.array([1.0, 0.0, 0.0]))
    assert np.allclose(dz, [g])
    assert np.allclose(dx, [[g[0] - g[2], 0.0]])                 # W^T g
    assert np.allclose(dw, np.outer(g, [1.0, 2.0]))


@pytest.mark.parametrize("n,C", [(1, 8), (37, 16), (200, 40)])
def test_against_torch_autograd(n, C):
    x, w, labels, cw = _case(n + C, n, C)
    scale = 1.0 / n
    z, loss, dz, dx, dw = logits_ce_fused(x, w, labels, cw, scale)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    zt = torch.nn.functional.linear(xt, wt)
    zt.retain_grad()
    per = torch.nn.functional.cross_entropy(zt, torch.tensor(labels.astype(np.int64)), reduction="none")
    lt = scale * (torch.tensor(cw)[torch.tensor(labels.astype(np.int64))] * per).sum()
    lt.backward()
    assert np.allclose(z, zt.detach().numpy(), rtol=1e-12, atol=1e-12)
    assert np.isclose(loss, lt.item(), rtol=1e-12)
    assert np.allclose(dz, zt.grad.numpy(), rtol=1e-10, atol=1e-14)
    assert np.allclose(dx, xt.grad.numpy(), rtol=1e-10, atol=1e-14)
    assert np.allclose(dw, wt.grad.numpy(), rtol=1e-10, atol=1e-14)


def test_finite_differences():
    x, w, labels, cw = _case(5, 6, 8)
    scale = 0.25
    _, loss, _, dx, dw = logits_ce_fused(x, w, labels, cw, scale)
    h = 1e-6
    for (i, j) in [(0, 0), (3, 5), (5, 7)]:
        xp, xm = x.copy(), x.copy()
        xp[i, j] += h
        xm[i, j] -= h
        fd = (logits_ce_fused(xp, w, labels, cw, scale)[1] - logits_ce_fused(xm, w, labels, cw, scale)[1]) / (2 * h)
        assert np.isclose(fd, dx[i, j], rtol=1e-6, atol=1e-9)
    for (k, j) in [(0, 0), (1, 4), (2, 7)]:
        wp, wm = w.copy(), w.copy()
        wp[k, j] += h
        wm[k, j] -= h
        fd = (logits_ce_fused(x, wp, labels, cw, scale)[1] - logits_ce_fused(x, wm, labels, cw, scale)[1]) / (2 * h)
        assert np.isclose(fd, dw[k, j], rtol=1e-6, atol=1e-9)


def test_invariants():
    x, w, labels, cw = _case(9, 50, 24)
    z, loss, dz, dx, dw = logits_ce_fused(x, w, labels, cw, 1.0)
    assert np.allclose(dz.sum(axis=1), 0.0, atol=1e-12)          # softmax - onehot sums to zero per pixel
    assert np.allclose(dw.sum(axis=0), 0.0, atol=1e-10)          # hence so do the rows of dW
    # a class whose weight is zero contributes nothing from its pixels
    cw0 = cw.copy()
    cw0[1] = 0.0
    _, _, dz0, dx0, _ = logits_ce_fused(x, w, labels, cw0, 1.0)
    assert np.all(dz0[labels == 1] == 0.0) and np.all(dx0[labels == 1] == 0.0)
    # the scale is a factor of everything but the logits
    _, loss2, dz2, dx2, dw2 = logits_ce_fused(x, w, labels, cw, 0.5)
    assert np.isclose(loss2, 0.5 * loss) and np.allclose(dx2, 0.5 * dx) and np.allclose(dw2, 0.5 * dw)
    # no pixels: zero loss and zero filter gradient
    z, loss, dz, dx, dw = logits_ce_fused(np.zeros((0, 8)), np.ones((3, 8)), np.zeros(0, dtype=np.uint8), cw, 1.0)
    assert loss == 0.0 and dw.shape == (3, 8) and np.all(dw == 0.0) and dx.shape == (0, 8)
