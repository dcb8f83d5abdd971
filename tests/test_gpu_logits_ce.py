"""GPU parity of logits_ce_fused_fwd_bwd (the logits layer fused with the loss) through the C
boundary against the fp64 oracle (``oracle/fused.py``), and against the four separate entry
points it replaces."""
import sys

import numpy as np
import pytest
import torch

from oracle.fused import logits_ce_fused
from paper_1810_01993_amd import synth

import gpu_util as U

pytestmark = pytest.mark.gpu

LOSS_RTOL = 1e-5          # fp32 log-sum-exp and an fp32 sum over the pixels (as for the loss alone)
DW_TOL = {"f16": 2e-3, "bf16": 8e-3, "f32": 2e-5}


@pytest.fixture(scope="module")
def api():
    from paper_1810_01993_amd import api as _api
    assert torch.cuda.is_available()
    return _api


def _inputs(n, C, dtype, seed):
    x32, xb = synth.quantize(synth.half_normal(seed, (n, C)), dtype)
    w32, wb = synth.quantize(synth.he_filter(seed + 1, 3, 1, 1, C), dtype)
    labels = synth.rng(seed + 2).choice(3, size=n, p=synth.CLASS_FREQ).astype(np.uint8)
    return x32, xb, w32.reshape(3, C), wb.reshape(3, C), labels


def _check(api, n, C, dtype, seed, scale=None, dw_f32=False, sample=None):
    print(f"[case] logits_ce_fused n={n} C={C} {dtype} seed={seed} dw_f32={dw_f32}", flush=True)
    sys.stdout.flush()
    x32, xb, w32, wb, labels = _inputs(n, C, dtype, seed)
    cw = np.asarray(synth.CLASS_WEIGHTS, dtype=np.float32)
    scale = (1.0 / max(n, 1)) if scale is None else scale
    logits, loss, dlogits, dx, dw = api.logits_ce_fused_fwd_bwd(
        U.to_device(xb, dtype), U.to_device(wb, dtype), torch.from_numpy(labels).cuda(), torch.from_numpy(cw).cuda(),
        scale, dw_f32=dw_f32)
    torch.cuda.synchronize()
    rz, rloss, rdz, rdx, rdw = logits_ce_fused(x32, w32, labels, cw.astype(np.float64), float(np.float32(scale)))
    tol = U.TOL[dtype]
    if n:
        assert U.rel_err(U.to_host_f64(logits), rz) <= tol
        assert U.rel_err(U.to_host_f64(dlogits), rdz) <= tol
        got_dx = U.to_host_f64(dx)
        if sample:
            idx = U.sample_indices(got_dx.shape, sample, seed)
            assert U.rel_err(got_dx.ravel()[idx], rdx.ravel()[idx]) <= tol
        else:
            assert U.rel_err(got_dx, rdx) <= tol
    assert abs(float(loss.item()) - rloss) <= LOSS_RTOL * max(abs(rloss), 1e-30) + 1e-12
    got_dw = dw.double().cpu().numpy().reshape(3, C)
    assert np.all(np.isfinite(got_dw))
    if n:
        assert U.rel_err(got_dw, rdw) <= DW_TOL["f32" if dw_f32 else dtype]
    else:
        assert np.all(got_dw == 0.0)
    return logits, loss, dlogits, dx, dw


@pytest.mark.parametrize("n,C", [(1, 32), (7, 40), (333, 256), (1000, 240), (4097, 64), (130, 2048), (5000, 304)])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_small_cases(api, n, C, dtype):
    # a single pixel, fewer pixels than a trip, ragged last trips, channel counts that do not divide the
    # workgroup (40, 240, 304 channels: idle threads), the widest supported row; gradients large enough for fp16
    _check(api, n, C, dtype, synth.seed_for(7, n + C), scale=1.0 / 64)


def test_no_pixels(api):
    _check(api, 0, 256, "f16", synth.seed_for(7, 1), scale=1.0)


def test_fp32_filter_gradient_and_optional_outputs(api):
    _check(api, 20000, 256, "f16", synth.seed_for(7, 2), scale=1.0 / 1024, dw_f32=True)
    x32, xb, w32, wb, labels = _inputs(3000, 256, "f16", synth.seed_for(7, 3))
    cw = torch.tensor(synth.CLASS_WEIGHTS, dtype=torch.float32, device="cuda")
    args = (U.to_device(xb, "f16"), U.to_device(wb, "f16"), torch.from_numpy(labels).cuda(), cw, 1.0 / 256)
    full = api.logits_ce_fused_fwd_bwd(*args)
    bare = api.logits_ce_fused_fwd_bwd(*args, want_logits=False, want_dlogits=False)
    assert bare[0] is None and bare[2] is None
    assert torch.equal(full[1], bare[1]) and torch.equal(full[3], bare[3]) and torch.equal(full[4], bare[4])


def test_network_size_and_determinism(api):
    # the network's logits layer: 2 x 768 x 1152 pixels, 256 channels; scale 2^-10 keeps fp16 gradients normal
    n = 2 * 768 * 1152
    a = _check(api, n, 256, "f16", synth.seed_for(7, 4), scale=2.0 ** -10, sample=20000)
    b = _check(api, n, 256, "f16", synth.seed_for(7, 4), scale=2.0 ** -10, sample=20000)
    for t, u in zip(a, b):
        assert torch.equal(t, u)


def test_agrees_with_the_separate_entry_points(api):
    """Same inputs through conv2d_fwd -> weighted_pixel_ce_fwd_bwd -> conv2d_bwd_data / conv2d_bwd_filter.  The
    chain rounds the logits and their gradient to 16 bits in between, the fused call does not: they agree to
    that rounding."""
    N, H, W, C = 1, 96, 130, 256
    n = N * H * W
    x32, xb, w32, wb, labels = _inputs(n, C, "f16", synth.seed_for(7, 5))
    cw = torch.tensor(synth.CLASS_WEIGHTS, dtype=torch.float32, device="cuda")
    x = U.to_device(xb, "f16").view(N, H, W, C)
    w = U.to_device(wb, "f16").view(3, 1, 1, C)
    lab = torch.from_numpy(labels).cuda()
    scale = 1.0 / 64
    d = api.ConvDesc(N=N, H=H, W=W, C=C, K=3, R=1, S=1, stride_h=1, stride_w=1, pad_h=0, pad_w=0, dil_h=1, dil_w=1,
                     dtype=api.DL_F16)
    z = api.conv2d_fwd(d, x, w)
    loss, dz = api.weighted_pixel_ce_fwd_bwd(z.view(n, 3), lab, cw, scale)
    dx = api.conv2d_bwd_data(d, dz.view(N, H, W, 3), w)
    dw = api.conv2d_bwd_filter(d, x, dz.view(N, H, W, 3))
    fz, floss, fdz, fdx, fdw = api.logits_ce_fused_fwd_bwd(x, w, lab, cw, scale)
    torch.cuda.synchronize()
    assert U.rel_err(U.to_host_f64(fz), U.to_host_f64(z).reshape(n, 3)) <= 1e-3
    assert abs(floss.item() - loss.item()) <= 2e-3 * abs(loss.item())
    assert U.rel_err(U.to_host_f64(fdz), U.to_host_f64(dz)) <= 4e-3
    assert U.rel_err(U.to_host_f64(fdx), U.to_host_f64(dx)) <= 4e-3
    assert U.rel_err(fdw.double().cpu().numpy().ravel(), dw.double().cpu().numpy().ravel()) <= 4e-3


def test_argument_errors(api):
    x = torch.zeros((10, 24), dtype=torch.float16, device="cuda")             # fewer than 32 channels
    w = torch.zeros((3, 24), dtype=torch.float16, device="cuda")
    lab = torch.zeros(10, dtype=torch.uint8, device="cuda")
    cw = torch.ones(3, dtype=torch.float32, device="cuda")
    with pytest.raises(api.DlError):
        api.logits_ce_fused_fwd_bwd(x, w, lab, cw, 1.0)
    x = torch.zeros((10, 36), dtype=torch.float16, device="cuda")             # not a multiple of 8
    w = torch.zeros((3, 36), dtype=torch.float16, device="cuda")
    with pytest.raises(api.DlError):
        api.logits_ce_fused_fwd_bwd(x, w, lab, cw, 1.0)
    with pytest.raises(ValueError):
        api.logits_ce_fused_fwd_bwd(torch.zeros((10, 64), dtype=torch.float16, device="cuda"), w, lab, cw, 1.0)


def test_labels_outside_the_classes_have_weight_zero(api):
    """Pixels with a label other than 0, 1, 2 drop out: zero dlogits and dx rows, and loss and dW are
    those of the remaining pixels alone (the oracle on the good pixels with the same scale)."""
    for n, C, dtype in ((5000, 256, "f16"), (3001, 304, "bf16")):
        seed = synth.seed_for(7, 60 + C)
        print(f"[case] logits_ce_fused bad labels n={n} C={C} {dtype}", flush=True)
        x32, xb, w32, wb, labels = _inputs(n, C, dtype, seed)
        bad = np.zeros(n, dtype=bool)
        bad[synth.rng(seed + 9).integers(0, n, n // 20)] = True
        bad[[0, n - 1]] = True
        labels_bad = labels.copy()
        labels_bad[bad] = 200
        cw = np.asarray(synth.CLASS_WEIGHTS, dtype=np.float32)
        scale = 1.0 / 64
        _, loss, dlogits, dx, dw = api.logits_ce_fused_fwd_bwd(
            U.to_device(xb, dtype), U.to_device(wb, dtype), torch.from_numpy(labels_bad).cuda(),
            torch.from_numpy(cw).cuda(), scale)
        torch.cuda.synchronize()
        good = ~bad
        _, rloss, rdz, rdx, rdw = logits_ce_fused(x32[good], w32, labels[good], cw.astype(np.float64),
                                                  float(np.float32(scale)))
        gdz, gdx = U.to_host_f64(dlogits), U.to_host_f64(dx)
        assert np.all(gdz[bad] == 0.0) and np.all(gdx[bad] == 0.0)
        assert U.rel_err(gdz[good], rdz) <= U.TOL[dtype]
        assert U.rel_err(gdx[good], rdx) <= U.TOL[dtype]
        assert abs(float(loss.item()) - rloss) <= LOSS_RTOL * abs(rloss)
        assert U.rel_err(dw.double().cpu().numpy().reshape(3, C), rdw) <= DW_TOL[dtype]
