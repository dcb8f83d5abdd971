"""GPU parity: weighted_pixel_ce_fwd_bwd through the C boundary against the oracle."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_1810_01993_amd import synth

import gpu_util as U

pytestmark = pytest.mark.gpu

# fp32 evaluation of log-sum-exp and an fp32 tree sum over the pixels: the
# relative error of the scalar is a few fp32 ulps times log2(n) -- 1e-5 leaves
# an order of magnitude of room at 1.8 M pixels.
LOSS_RTOL = 1e-5


@pytest.fixture(scope="module")
def api():
    from paper_1810_01993_amd import api as _api
    assert torch.cuda.is_available()
    return _api


def _run(api, n, dtype, seed, labels=None, sigma=1.0, scale=None):
    print(f"[case] weighted_ce n={n} {dtype} seed={seed} sigma={sigma}", flush=True)
    sys.stdout.flush()
    z32, zb = synth.quantize(synth.normal(seed, (n, 3), sigma=sigma), dtype)
    if labels is None:
        labels = synth.rng(seed + 1).choice(3, size=n, p=synth.CLASS_FREQ).astype(np.uint8)
    scale = (1.0 / max(n, 1)) if scale is None else scale
    cw = np.asarray(synth.CLASS_WEIGHTS, dtype=np.float32)
    loss, dz = api.weighted_pixel_ce_fwd_bwd(U.to_device(zb, dtype), torch.from_numpy(labels).cuda(),
                                             torch.from_numpy(cw).cuda(), scale)
    torch.cuda.synchronize()
    ref_loss, ref_dz = oracle.weighted_ce(z32, labels, cw.astype(np.float64), float(np.float32(scale)))
    got_loss = float(loss.item())
    if n:
        assert abs(got_loss - ref_loss) <= LOSS_RTOL * abs(ref_loss), (got_loss, ref_loss)
        err = U.rel_err(U.to_host_f64(dz), ref_dz)
        assert err <= U.TOL[dtype], f"dlogits max|err|/max|ref| = {err:.3e}"
        # the gradient of the labelled class is negative, the others positive
        g = U.to_host_f64(dz)
        assert np.all(g[np.arange(n), labels] <= 0)
    else:
        assert got_loss == 0.0
    return got_loss


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 1000, 8 * 257 + 3, 8 * 256 * 9 + 5])
def test_sizes_and_ragged_tails(api, n, dtype):
    _run(api, n, dtype, synth.seed_for(0, 900 + n % 97))


def test_large_logits(api):
    _run(api, 4099, "f16", synth.seed_for(0, 950), sigma=40.0)
    _run(api, 4099, "bf16", synth.seed_for(0, 951), sigma=300.0)


def test_config5_full_mask(api):
    """N=2 full-resolution logits with the ellipse label mask, 1/(N*H*W) scale."""
    labels = synth.ellipse_labels(synth.seed_for(5, 990), 2, 768, 1152).ravel()
    got = _run(api, labels.size, "f16", synth.seed_for(5, 991), labels=labels)
    assert got > 0


def test_determinism_and_redzones(api):
    n = 8 * 300 + 5
    _, zb = synth.quantize(synth.normal(3, (n, 3)), "f16")
    labels = synth.rng(4).integers(0, 3, n).astype(np.uint8)
    cw = torch.tensor(synth.CLASS_WEIGHTS, dtype=torch.float32, device="cuda")
    z, lab = U.to_device(zb, "f16"), torch.from_numpy(labels).cuda()
    guard = 64
    res = []
    for _ in range(2):
        buf = torch.full((3 * n + 2 * guard,), 77.0, dtype=torch.float16, device="cuda")
        dz = buf[guard:guard + 3 * n].view(n, 3)
        loss, _ = api.weighted_pixel_ce_fwd_bwd(z, lab, cw, 0.5, dlogits=dz)
        torch.cuda.synchronize()
        assert torch.all(buf[:guard] == 77.0) and torch.all(buf[-guard:] == 77.0)
        res.append((loss.clone(), dz.clone()))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])


def test_more_pixels_than_one_trip_per_wavefront(api):
    # above 1024 workgroups x 4 wavefronts x 512 pixels a wavefront makes several trips (the
    # loads of the next trip are in flight while the current one is worked on)
    # (scale 2^-10 rather than 1/n: with 4 M pixels 1/n would put every gradient in fp16's
    # subnormal range, where the spacing of 6e-8 is 4e-3 of the largest gradient)
    n = 2 * 1024 * 4 * 512 + 8 * 70 + 3
    _run(api, n, "f16", synth.seed_for(0, 960), scale=2.0 ** -10)


# ---- per-pixel weight map --------------------------------------------------------
def _run_map(api, n, dtype, seed, from_table=False):
    print(f"[case] weighted_ce_map n={n} {dtype} seed={seed} from_table={from_table}", flush=True)
    sys.stdout.flush()
    z32, zb = synth.quantize(synth.normal(seed, (n, 3)), dtype)
    labels = synth.rng(seed + 1).choice(3, size=n, p=synth.CLASS_FREQ).astype(np.uint8)
    if from_table:
        wm = np.asarray(synth.CLASS_WEIGHTS, dtype=np.float32)[labels]
    else:
        wm = synth.rng(seed + 2).uniform(0.0, 40.0, n).astype(np.float32)
        wm[::5] = 0.0                                   # masked-out pixels
    scale = 1.0 / max(n, 1)
    zd, ld, wd = U.to_device(zb, dtype), torch.from_numpy(labels).cuda(), torch.from_numpy(wm).cuda()
    loss, dz = api.weighted_pixel_ce_map_fwd_bwd(zd, ld, wd, scale)
    torch.cuda.synchronize()
    ref_loss, ref_dz = oracle.weighted_ce_map(z32, labels, wm.astype(np.float64), float(np.float32(scale)))
    got_loss = float(loss.item())
    if n == 0:
        assert got_loss == 0.0
        return
    assert abs(got_loss - ref_loss) <= LOSS_RTOL * abs(ref_loss), (got_loss, ref_loss)
    g = U.to_host_f64(dz)
    assert U.rel_err(g, ref_dz) <= U.TOL[dtype]
    if not from_table:
        assert np.all(g[::5] == 0.0)
    else:
        # the class-table entry point must give the very same bits
        cw = torch.tensor(synth.CLASS_WEIGHTS, dtype=torch.float32, device="cuda")
        loss2, dz2 = api.weighted_pixel_ce_fwd_bwd(zd, ld, cw, scale)
        assert torch.equal(dz, dz2) and torch.equal(loss, loss2)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("n", [0, 1, 7, 9, 1000, 8 * 257 + 3, 8 * 256 * 9 + 5])
def test_weight_map_sizes_and_ragged_tails(api, n, dtype):
    _run_map(api, n, dtype, synth.seed_for(0, 970 + n % 89))


def test_weight_map_full_mask_and_class_table_equivalence(api):
    _run_map(api, 2 * 768 * 1152, "f16", synth.seed_for(5, 995), from_table=True)
    _run_map(api, 2 * 1024 * 4 * 512 + 8 * 70 + 3, "bf16", synth.seed_for(0, 996))


def test_labels_outside_the_classes_have_weight_zero(api):
    """A corrupted mask (label 3 or 255) must not train silently on class 2: such pixels add
    nothing to the loss and get a zero gradient, in whole-wavefront trips, in the left-over groups
    of 8 and in the ragged tail, with the class table and with the weight map."""
    n = 2 * 1024 * 4 * 512 + 8 * 70 + 5
    seed = synth.seed_for(0, 980)
    for dtype in ("f16", "bf16"):
        print(f"[case] weighted_ce bad labels n={n} {dtype}", flush=True)
        z32, zb = synth.quantize(synth.normal(seed, (n, 3)), dtype)
        labels = synth.rng(seed + 1).choice(3, size=n, p=synth.CLASS_FREQ).astype(np.uint8)
        bad = np.zeros(n, dtype=bool)
        bad[synth.rng(seed + 2).integers(0, n, 5000)] = True
        bad[[0, 511, 512, n - 600, n - 9, n - 5, n - 1]] = True      # first trip, trip boundary, groups of 8, tail
        labels_bad = labels.copy()
        labels_bad[bad] = np.where(np.arange(n)[bad] % 2 == 0, 3, 255).astype(np.uint8)
        cw = np.asarray(synth.CLASS_WEIGHTS, dtype=np.float32)
        scale = 2.0 ** -10
        wm = cw[labels].astype(np.float32)
        wm[bad] = 0.0
        ref_loss, ref_dz = oracle.weighted_ce_map(z32, labels, wm.astype(np.float64), float(np.float32(scale)))
        zd, ld = U.to_device(zb, dtype), torch.from_numpy(labels_bad).cuda()
        for which in ("table", "map"):
            if which == "table":
                loss, dz = api.weighted_pixel_ce_fwd_bwd(zd, ld, torch.from_numpy(cw).cuda(), scale)
            else:
                loss, dz = api.weighted_pixel_ce_map_fwd_bwd(zd, ld, torch.from_numpy(cw[labels]).cuda(), scale)
            torch.cuda.synchronize()
            g = U.to_host_f64(dz)
            assert np.all(g[bad] == 0.0), which
            assert U.rel_err(g, ref_dz) <= U.TOL[dtype], which
            assert abs(float(loss.item()) - ref_loss) <= LOSS_RTOL * abs(ref_loss), (which, loss.item(), ref_loss)
