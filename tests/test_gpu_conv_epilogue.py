"""GPU parity of conv2d_fwd_bias_relu (bias and ReLU fused into the store of the
forward convolution) against the fp64 oracle, on shapes that reach every
forward kernel: the 3x3 halo-tile kernel with each column-tile width, the
general halo-tile kernel, every tile of the plain engine, the split reduction,
the element-wise kernel for odd channel counts, the 3-column logits layer."""
import sys

import numpy as np
import pytest
import torch

from oracle import epilogue as E
from paper_1810_01993_amd import layers, synth
from paper_1810_01993_amd.layers import ConvLayer

import gpu_util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    from paper_1810_01993_amd import api as _api
    assert torch.cuda.is_available(), "a GPU is required for -m gpu tests"
    return _api


def check(api, layer: ConvLayer, dtype: str, seed: int, bias=True, relu=True, n_samples=6000):
    (x32, xb), (w32, wb), _ = U.conv_inputs(layer, dtype, seed, "normal")
    # biases of the size of the sums, so that a good part of the outputs is cut and a good part is not
    b = (synth.normal(seed + 7, (layer.K,)) * 0.7).astype(np.float32) if bias else None
    desc = api.desc_from_layer(layer, dtype)
    s = U.shape_of(layer)
    full = layer.flops() <= U.FULL_ORACLE_FLOPS
    print(f"[case] bias_relu {layer.name} {dtype} bias={bias} relu={relu} N{layer.N} {layer.H}x{layer.W}x{layer.C}->"
          f"{layer.K} {layer.R}x{layer.S} s{layer.stride} p{layer.pad} d{layer.dil} seed={seed} full={full}", flush=True)
    sys.stdout.flush()
    bd = torch.from_numpy(b).cuda() if bias else None
    got = U.to_host_f64(api.conv2d_fwd_bias_relu(desc, U.to_device(xb, dtype), U.to_device(wb, dtype), bd, relu))
    torch.cuda.synchronize()
    if full:
        ref = E.conv_fwd_bias_relu(s, x32, w32, b, relu)
    else:
        idx = np.union1d(U.sample_indices(got.shape, n_samples, seed), U.border_indices(got.shape, 256, seed))
        ref = E.conv_fwd_bias_relu_at(s, x32, w32, b, relu, idx)
        got = got.ravel()[idx]
    assert np.all(np.isfinite(got))
    if relu:
        assert got.min() >= 0.0
        cut = float(np.mean(ref == 0.0))
        assert 0.05 < cut < 0.95, f"degenerate case: {cut:.2f} of the outputs cut"
        # where the sum is clearly negative the output is exactly zero
        assert np.all(got[ref == 0.0] <= U.TOL[dtype] * np.max(np.abs(ref)))
    err = U.rel_err(got, ref)
    assert err <= U.TOL[dtype], f"{layer.name} {dtype}: max|err|/max|ref| = {err:.3e}"


L = ConvLayer
CASES = [
    (L("e.halo3x3.k256", 1, 200, 230, 40, 256, 3, 3, 1, 1, 1), "f16"),            # two 128-wide column tiles
    (L("e.halo3x3.k304", 1, 150, 260, 32, 304, 3, 3, 1, 1, 1), "bf16"),           # two 160-wide tiles, ragged
    (L("e.halo3x3.k192", 1, 210, 300, 24, 192, 3, 3, 1, 1, 1), "f16"),            # 128 + a 64-wide tile (bias offset)
    (L("e.halo.d2.k192", 1, 230, 250, 32, 192, 3, 3, 1, 2, 2), "bf16"),           # general halo kernel + remainder launch
    (L("e.dma.256x256", 2, 192, 288, 16, 256, 3, 3, 1, 1, 1), "f16"),
    (L("e.dma.k304.remainder", 2, 150, 200, 64, 304, 1, 1, 1, 0, 1), "f16"),      # 256 + 48 columns in two launches
    (L("e.dma.small", 2, 19, 23, 24, 40, 3, 3, 1, 1, 1), "bf16"),
    (L("e.dma.s2", 2, 21, 26, 32, 48, 3, 3, 2, 1, 1), "f16"),
    (L("e.dma.1x1.k136", 2, 17, 19, 72, 136, 1, 1, 1, 0, 1), "f16"),
    (L("e.ksplit.3x3.c1000", 1, 20, 24, 1000, 256, 3, 3, 1, 1, 1), "f16"),        # split reduction: tail in the reduce kernel
    (L("e.scalar.odd-channels", 2, 9, 11, 3, 5, 3, 3, 1, 1, 1), "f16"),
    (L("e.logits.k3", 1, 33, 47, 256, 3, 1, 1, 1, 0, 1), "bf16"),
    (L("e.thin.c4", 1, 40, 50, 4, 64, 1, 1, 1, 0, 1), "f16"),                     # 4 input channels: the streaming kernel
    (L("e.stem7x7", 2, 30, 44, 16, 64, 7, 7, 2, 3, 1), "bf16"),
    (L("e.narrow5x5.k32", 4, 75, 200, 16, 32, 5, 5, 1, 2, 1), "f16"),             # 5x5 kernel for <= 32 output channels
    (L("e.narrow5x5.k24", 3, 100, 230, 40, 24, 5, 5, 1, 2, 1), "bf16"),
    (L("e.narrow5x5.ksplit", 4, 50, 70, 96, 32, 5, 5, 1, 2, 1), "f16"),             # its split reduction: tail in the reduce kernel
]


@pytest.mark.parametrize("layer,dtype", CASES, ids=[l.name for l, _ in CASES])
def test_bias_and_relu(api, layer, dtype):
    check(api, layer, dtype, synth.seed_for(0, 1400 + CASES.index((layer, dtype))))


def test_bias_only_and_relu_only(api):
    layer = CASES[0][0]
    check(api, layer, "f16", synth.seed_for(0, 1450), bias=True, relu=False)
    check(api, layer, "f16", synth.seed_for(0, 1451), bias=False, relu=True)
    small = CASES[6][0]
    check(api, small, "bf16", synth.seed_for(0, 1452), bias=True, relu=False)
    check(api, small, "bf16", synth.seed_for(0, 1453), bias=False, relu=True)


def test_no_tail_gives_the_bits_of_conv2d_fwd(api):
    for layer, dtype in (CASES[0], CASES[6], CASES[9]):
        (_, xb), (_, wb), _ = U.conv_inputs(layer, dtype, 5, "normal")
        desc = api.desc_from_layer(layer, dtype)
        xd, wd = U.to_device(xb, dtype), U.to_device(wb, dtype)
        a = api.conv2d_fwd(desc, xd, wd)
        b = api.conv2d_fwd_bias_relu(desc, xd, wd, None, False)
        z = api.conv2d_fwd_bias_relu(desc, xd, wd, torch.zeros(layer.K, dtype=torch.float32, device="cuda"), False)
        assert torch.equal(a, b) and torch.equal(a, z)


def test_full_resolution_decoder_layer(api):
    layer = [l for l in layers.config5()[1] if l.name == "dec.3x3.256-256"][0]
    check(api, layer, "f16", synth.seed_for(0, 1460), n_samples=3000)


def check_residual(api, layer: ConvLayer, dtype: str, seed: int, bias=True, relu=True, n_samples=6000):
    """y = act(conv + bias + residual) against the oracle; the residual is of the size of the sums."""
    (x32, xb), (w32, wb), _ = U.conv_inputs(layer, dtype, seed, "normal")
    b = (synth.normal(seed + 7, (layer.K,)) * 0.7).astype(np.float32) if bias else None
    r32, rb = synth.quantize(synth.normal(seed + 8, (layer.N, layer.P, layer.Q, layer.K)), dtype)
    desc = api.desc_from_layer(layer, dtype)
    s = U.shape_of(layer)
    full = layer.flops() <= U.FULL_ORACLE_FLOPS
    print(f"[case] bias_add_relu {layer.name} {dtype} bias={bias} relu={relu} N{layer.N} {layer.H}x{layer.W}x{layer.C}->"
          f"{layer.K} {layer.R}x{layer.S} s{layer.stride} p{layer.pad} d{layer.dil} seed={seed} full={full}", flush=True)
    sys.stdout.flush()
    bd = torch.from_numpy(b).cuda() if bias else None
    got = U.to_host_f64(api.conv2d_fwd_bias_add_relu(desc, U.to_device(xb, dtype), U.to_device(wb, dtype), bd,
                                                     U.to_device(rb, dtype), relu))
    torch.cuda.synchronize()
    if full:
        ref = E.conv_fwd_bias_add_relu(s, x32, w32, b, r32, relu)
    else:
        idx = np.union1d(U.sample_indices(got.shape, n_samples, seed), U.border_indices(got.shape, 256, seed))
        ref = E.conv_fwd_bias_add_relu_at(s, x32, w32, b, r32, relu, idx)
        got = got.ravel()[idx]
    assert np.all(np.isfinite(got))
    if relu:
        assert got.min() >= 0.0
        cut = float(np.mean(ref == 0.0))
        assert 0.05 < cut < 0.95, f"degenerate case: {cut:.2f} of the outputs cut"
    err = U.rel_err(got, ref)
    assert err <= U.TOL[dtype], f"{layer.name} {dtype}: max|err|/max|ref| = {err:.3e}"


# every kernel a launch with a residual can take: the plain engine's staged store (several tile shapes, strided,
# a remainder launch with offset pointers, output channels not a multiple of 4 or 8), its split reduction, the
# general halo-tile kernel (+ remainder), the element-wise kernel, the streaming kernel for few input channels;
# and the shapes that would take the 3x3 or 5x5 patch kernels without one
RESIDUAL_CASES = [
    (L("r.res-block.1x1.64-256", 2, 40, 56, 64, 256, 1, 1, 1, 0, 1), "f16"),        # a ResNet block's last convolution
    (L("r.res-block.1x1.512-2048", 1, 20, 24, 512, 2048, 1, 1, 1, 0, 1), "bf16"),
    (L("r.dma.k304.remainder", 2, 150, 200, 64, 304, 1, 1, 1, 0, 1), "f16"),
    (L("r.dma.s2.k48", 2, 21, 26, 32, 48, 3, 3, 2, 1, 1), "bf16"),
    (L("r.dma.k136", 2, 17, 19, 72, 136, 1, 1, 1, 0, 1), "f16"),
    (L("r.dma.k20", 1, 14, 15, 16, 20, 5, 5, 1, 2, 1), "f16"),                       # 8-byte alignment of rows varies
    (L("r.ksplit.3x3.c1000", 1, 20, 24, 1000, 256, 3, 3, 1, 1, 1), "f16"),
    (L("r.halo.d2.k192", 1, 230, 250, 32, 192, 3, 3, 1, 2, 2), "bf16"),
    (L("r.scalar.odd-channels", 2, 9, 11, 3, 5, 3, 3, 1, 1, 1), "f16"),
    (L("r.thin.c4", 1, 40, 50, 4, 64, 1, 1, 1, 0, 1), "bf16"),
    (L("r.logits.k3", 1, 33, 47, 256, 3, 1, 1, 1, 0, 1), "f16"),                      # would take the streaming forward kernel
    (L("r.would-be-halo3x3.k256", 1, 200, 230, 40, 256, 3, 3, 1, 1, 1), "f16"),
    (L("r.would-be-narrow5x5.k32", 4, 75, 200, 16, 32, 5, 5, 1, 2, 1), "f16"),
    (L("r.would-be-wide5x5.c32.k80", 3, 100, 230, 32, 80, 5, 5, 1, 2, 1), "bf16"),
]


@pytest.mark.parametrize("layer,dtype", RESIDUAL_CASES, ids=[l.name for l, _ in RESIDUAL_CASES])
def test_bias_residual_relu(api, layer, dtype):
    check_residual(api, layer, dtype, synth.seed_for(0, 1500 + RESIDUAL_CASES.index((layer, dtype))))


def test_residual_only_and_null_residual(api):
    layer, dtype = RESIDUAL_CASES[0]
    check_residual(api, layer, dtype, synth.seed_for(0, 1550), bias=False, relu=False)
    check_residual(api, layer, dtype, synth.seed_for(0, 1551), bias=False, relu=True)
    # without a residual the entry point is conv2d_fwd_bias_relu, bit for bit (same kernels)
    for layer, dtype in (CASES[0], CASES[6]):
        (_, xb), (_, wb), _ = U.conv_inputs(layer, dtype, 6, "normal")
        desc = api.desc_from_layer(layer, dtype)
        xd, wd = U.to_device(xb, dtype), U.to_device(wb, dtype)
        bias = torch.randn(layer.K, dtype=torch.float32, device="cuda")
        assert torch.equal(api.conv2d_fwd_bias_relu(desc, xd, wd, bias, True),
                           api.conv2d_fwd_bias_add_relu(desc, xd, wd, bias, None, True))
