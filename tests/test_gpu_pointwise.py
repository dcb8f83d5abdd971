"""GPU parity of bias_relu_bwd (backward of the fused point-wise tail: ReLU mask
on dy and bias gradient in one pass) against the fp64 oracle."""
import sys

import numpy as np
import pytest
import torch

from oracle import epilogue as E
from paper_1810_01993_amd import synth

import gpu_util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    from paper_1810_01993_amd import api as _api
    assert torch.cuda.is_available()
    return _api


def _run(api, n, K, dtype, seed, relu=True, alias=False):
    print(f"[case] bias_relu_bwd n={n} K={K} {dtype} relu={relu} alias={alias} seed={seed}", flush=True)
    sys.stdout.flush()
    dy32, dyb = synth.quantize(synth.normal(seed, (n, K)), dtype)
    # a forward output: about half of it cut to exactly zero (also -0 never appears after a ReLU)
    y32, yb = synth.quantize(np.maximum(synth.normal(seed + 1, (n, K)), 0.0), dtype)
    dyd, yd = U.to_device(dyb, dtype), U.to_device(yb, dtype)
    dz, db = api.bias_relu_bwd(dyd, yd if relu else None, relu, dz=dyd if (alias and relu) else None)
    torch.cuda.synchronize()
    ref_dz, ref_db = E.bias_relu_bwd(dy32, y32, relu)
    got_dz = U.to_host_f64(dz)
    assert np.array_equal(got_dz, ref_dz)                       # masking copies bits: exact
    got_db = db.double().cpu().numpy()
    # fp32 running sums over up to n terms: error bounded by a few ulps of the sum of magnitudes
    bound = 1e-5 * np.abs(ref_dz).sum(axis=0) + 1e-30
    assert np.all(np.abs(got_db - ref_db) <= bound), float(np.max(np.abs(got_db - ref_db) / bound))
    return db


CASES = [(1, 8), (5, 8), (1000, 64), (777, 48), (4099, 256), (300, 304), (2500, 3), (911, 5), (64, 2048), (33, 4096),
         (70000, 16)]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("n,K", CASES, ids=[f"{n}x{K}" for n, K in CASES])
def test_mask_and_bias_gradient(api, n, K, dtype):
    _run(api, n, K, dtype, synth.seed_for(0, 1500 + (n * 7 + K) % 91))


def test_without_relu_in_place_and_repeatable(api):
    _run(api, 3001, 72, "f16", synth.seed_for(0, 1590), relu=False)
    a = _run(api, 3001, 72, "bf16", synth.seed_for(0, 1591), alias=True)
    b = _run(api, 3001, 72, "bf16", synth.seed_for(0, 1591), alias=True)
    assert torch.equal(a, b)


def test_decoder_sized_tensor(api):
    # one image of the full-resolution decoder output: 884 736 pixels x 256 channels
    _run(api, 768 * 1152, 256, "f16", synth.seed_for(0, 1595))


def test_empty(api):
    dy = torch.empty((0, 16), dtype=torch.float16, device="cuda")
    dz, db = api.bias_relu_bwd(dy, dy.clone(), True)
    torch.cuda.synchronize()
    assert dz.numel() == 0 and torch.count_nonzero(db).item() == 0
