"""GPU parity: conv2d_fwd / conv2d_bwd_data / conv2d_bwd_filter through the C
boundary against the fp64 oracle, element by element on the same seeded
inputs (full tensors for small cases, sampled outputs at full size)."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_1810_01993_amd import layers, synth
from paper_1810_01993_amd.layers import ConvLayer

import gpu_util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    from paper_1810_01993_amd import api as _api
    assert torch.cuda.is_available(), "a GPU is required for -m gpu tests"
    return _api


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def check_layer(api, layer: ConvLayer, dtype: str, seed: int, x_kind="half_normal", n_samples=8192,
                dw_f32=False, passes=("fwd", "dgrad", "wgrad"), full_passes=(), dw_per_cell=0):
    """Run the requested passes on the GPU and compare with the oracle: on the whole tensor where the
    oracle's cost allows (U.FULL_LIMIT; always for the passes named in `full_passes`), otherwise on
    n_samples uniformly drawn outputs plus every element of the first and last two rows and columns
    (activations) or, with dw_per_cell > 0, that many elements of every 32 x 32-channel block of every
    tap (filter gradient).  Every output and every workspace lies between marked guard zones, which
    must survive the call.  Returns {pass: rel_err}."""
    (x32, xb), (w32, wb), (dy32, dyb) = U.conv_inputs(layer, dtype, seed, x_kind)
    desc = api.desc_from_layer(layer, dtype, dw_f32=dw_f32)
    s = U.shape_of(layer)
    xd, wd, dyd = U.to_device(xb, dtype), U.to_device(wb, dtype), U.to_device(dyb, dtype)
    tdt = U.TORCH_DTYPE[dtype]
    errs = {}
    for which in passes:
        full = which in full_passes or layer.flops() <= U.FULL_LIMIT[which]
        _say(f"[case] {layer.name} {dtype} {which} N{layer.N} {layer.H}x{layer.W}x{layer.C}->{layer.K} "
             f"{layer.R}x{layer.S} s{layer.stride} p{layer.pad} d{layer.dil} seed={seed} full={full}")
        pass_id = {"fwd": api.PASS_FWD, "dgrad": api.PASS_BWD_DATA, "wgrad": api.PASS_BWD_FILTER}[which]
        ws_bytes = api.dl_conv_workspace_bytes(desc, pass_id)
        ws_buf, ws = U.guarded_workspace(ws_bytes)
        if which == "fwd":
            out_buf, out = U.guarded((layer.N, layer.P, layer.Q, layer.K), tdt)
            api.conv2d_fwd(desc, xd, wd, y=out, workspace=ws)
        elif which == "dgrad":
            out_buf, out = U.guarded((layer.N, layer.H, layer.W, layer.C), tdt)
            api.conv2d_bwd_data(desc, dyd, wd, dx=out, workspace=ws)
        else:
            out_buf, out = U.guarded((layer.K, layer.R, layer.S, layer.C), torch.float32 if dw_f32 else tdt)
            api.conv2d_bwd_filter(desc, xd, dyd, dw=out, workspace=ws)
        torch.cuda.synchronize()
        assert U.guards_intact(out_buf), f"{layer.name} {which}: write outside the output tensor"
        assert U.workspace_guards_intact(ws_buf, ws_bytes), f"{layer.name} {which}: write outside the workspace"
        got = U.to_host_f64(out)
        del out, out_buf, ws, ws_buf
        if which == "fwd":
            if full:
                ref = oracle.conv_fwd(s, x32, w32)
            else:
                idx = np.union1d(U.sample_indices(got.shape, n_samples, seed), U.all_border_indices(got.shape, seed))
                ref = oracle.conv_fwd_at(s, x32, w32, idx)
                got = got.ravel()[idx]
        elif which == "dgrad":
            if full:
                ref = oracle.conv_bwd_data(s, dy32, w32)
            else:
                idx = np.union1d(U.sample_indices(got.shape, n_samples, seed), U.all_border_indices(got.shape, seed))
                ref = oracle.conv_bwd_data_at(s, dy32, w32, idx)
                got = got.ravel()[idx]
        else:
            if full:
                ref = oracle.conv_bwd_filter(s, x32, dy32)
            else:
                npix = layer.N * layer.P * layer.Q
                if dw_per_cell > 0:
                    idx = U.stratified_filter_indices(got.shape, dw_per_cell, seed)
                else:
                    idx = U.sample_indices(got.shape, max(16, min(n_samples, int(4e9 // npix))), seed)
                ref = oracle.conv_bwd_filter_at(s, x32, dy32, idx)
                got = got.ravel()[idx]
        assert np.all(np.isfinite(got)), f"{layer.name} {which}: non-finite output"
        if dtype == "f16" and ref.size:
            assert float(np.max(np.abs(ref))) < U.FP16_MAX_REF, f"{layer.name} {which}: the exact result leaves fp16's range"
        errs[which] = U.rel_err(got, ref)
        tol = U.TOL[dtype]
        assert errs[which] <= tol, f"{layer.name} {dtype} {which}: max|err|/max|ref| = {errs[which]:.3e} > {tol}"
    return errs


# ---- small shapes: several tiles, ragged tails, every index path ------------
L = ConvLayer
SMALL = [
    L("3x3.d2.c16k64", 1, 24, 36, 16, 64, 3, 3, 1, 2, 2),
    L("3x3.ragged", 2, 19, 23, 24, 40, 3, 3, 1, 1, 1),
    L("3x3.s2", 2, 21, 26, 32, 48, 3, 3, 2, 1, 1),
    L("3x3.s2.d2", 1, 22, 25, 16, 32, 3, 3, 2, 2, 2),
    L("3x3.s3.d2", 1, 25, 22, 8, 16, 3, 3, 3, 2, 2),
    L("7x7.s2.c16", 2, 30, 44, 16, 64, 7, 7, 2, 3, 1),
    L("1x1", 2, 17, 19, 72, 136, 1, 1, 1, 0, 1),
    L("1x1.s2", 2, 18, 20, 64, 160, 1, 1, 2, 0, 1),
    L("1x1.k3", 1, 33, 47, 256, 3, 1, 1, 1, 0, 1),
    L("1x1.k3.many-slices", 1, 150, 250, 64, 3, 1, 1, 1, 0, 1),   # 147 pixel slices x 192 outputs: the 32-group reduce; ragged row ranges
    L("1x1.k48", 1, 20, 30, 256, 48, 1, 1, 1, 0, 1),
    L("1x1.k4.c304", 2, 21, 30, 304, 4, 1, 1, 1, 0, 1),
    L("1x1.k2.c8", 1, 9, 10, 8, 2, 1, 1, 1, 0, 1),
    # 256 input channels and 1..4 output channels: the streaming forward kernel (runs of 16 pixels per wavefront)
    L("1x1.c256.k1.one-pixel", 1, 1, 1, 256, 1, 1, 1, 1, 0, 1),
    L("1x1.c256.k2.ragged-run", 1, 5, 7, 256, 2, 1, 1, 1, 0, 1),
    L("1x1.c256.k4", 2, 9, 7, 256, 4, 1, 1, 1, 0, 1),
    L("1x1.c256.k3.many-runs", 1, 301, 171, 256, 3, 1, 1, 1, 0, 1),            # more runs than wavefronts in the grid
    L("3x3.c304", 1, 12, 40, 304, 256, 3, 3, 1, 1, 1),
    L("3x3.d6.small-map", 2, 10, 14, 64, 32, 3, 3, 1, 6, 6),
    L("3x3.d12.small-map", 1, 12, 18, 32, 64, 3, 3, 1, 12, 12),
    L("3x3.d18.taps-in-padding", 1, 12, 20, 32, 32, 3, 3, 1, 18, 18),
    L("3x3.odd-channels", 2, 9, 11, 3, 5, 3, 3, 1, 1, 1),
    L("3x3.odd-c.s2", 1, 13, 10, 5, 8, 3, 3, 2, 1, 1),
    L("5x5.c12k20", 1, 14, 15, 12, 20, 5, 5, 1, 2, 1),
    L("pool.1x1.map", 2, 1, 1, 2048, 256, 1, 1, 1, 0, 1),
    L("nopad.3x3", 1, 9, 9, 8, 8, 3, 3, 1, 0, 1),
    L("single-pixel-out", 1, 3, 3, 8, 8, 3, 3, 1, 0, 1),
    L("wide.n-tiles", 1, 16, 24, 32, 328, 3, 3, 1, 1, 1),
    # few output pixels, long reduction: the reduction is split over workgroups (ragged last chunk, ragged columns)
    L("ksplit.3x3.c1000", 1, 20, 24, 1000, 256, 3, 3, 1, 1, 1),
    L("ksplit.1x1.c8200", 2, 12, 20, 8200, 256, 1, 1, 1, 0, 1),
]


@pytest.mark.parametrize("layer", SMALL, ids=[l.name for l in SMALL])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_small_shapes(api, layer, dtype):
    check_layer(api, layer, dtype, synth.seed_for(0, 7 * SMALL.index(layer)), x_kind="normal")


def _random_layers(seed, count):
    """Seeded random layer shapes: filter sizes 1..7, strides 1..3, dilations 1..6, paddings 0..half the
    dilated filter, channel counts with and without the 8- and 32-alignment the fast paths want."""
    import random
    rng = random.Random(seed)
    out = []
    while len(out) < count:
        R = rng.choice([1, 1, 3, 3, 3, 5, 7])
        S = R if rng.random() < 0.8 else rng.choice([1, 3])
        st = rng.choice([1, 1, 1, 2, 2, 3])
        dil = rng.choice([1, 1, 2, 3, 6])
        pad = rng.choice([0, dil * (R // 2), dil * (R // 2), 1, 2])
        C = rng.choice([3, 8, 16, 24, 32, 40, 64, 72, 128, 136, 256, 304, 520])
        K = rng.choice([3, 5, 8, 16, 32, 48, 64, 72, 128, 160, 256, 264, 304])
        N, H, W = rng.choice([1, 2]), rng.randint(6, 70), rng.randint(6, 90)
        if rng.random() < 0.2:                   # some maps large enough for the halo-tile kernels
            H, W, C, K = rng.randint(150, 260), rng.randint(150, 300), min(C, 72), min(K, 264)
        layer = L(f"rand{len(out)}.{H}x{W}x{C}-{K}.{R}x{S}.s{st}p{pad}d{dil}", N, H, W, C, K, R, S, st, pad, dil)
        if layer.P >= 1 and layer.Q >= 1:
            out.append((layer, rng.choice(["f16", "bf16"])))
    return out


RANDOM = _random_layers(20181001, 48)


@pytest.mark.parametrize("layer,dtype", RANDOM, ids=[l.name for l, _ in RANDOM])
def test_random_shapes(api, layer, dtype):
    check_layer(api, layer, dtype, synth.seed_for(0, 900 + RANDOM.index((layer, dtype))), x_kind="normal",
                n_samples=3000)


def test_big_tile_path(api):
    # enough 256-row tiles that the wide configuration is selected (8.2 GFLOP: whole tensors)
    check_layer(api, L("bigtile", 2, 192, 288, 16, 256, 3, 3, 1, 1, 1), "f16", synth.seed_for(0, 501))


# Shapes that take the halo-tile kernels (stride 1, several taps, >= 200
# tiles): the 3x3 unit-dilation kernel and the general one; ragged patches,
# ragged channel chunk, ragged column tile, dilation 2, a column remainder
# handed to the plain engine, no padding, both data types, every column-tile
# width of the 3x3 kernel (128, 160, <= 64) alone and mixed.
HALO = [
    (L("halo.ragged", 2, 150, 170, 40, 256, 3, 3, 1, 1, 1), "f16"),
    (L("halo.d2.n192", 1, 230, 250, 32, 192, 3, 3, 1, 2, 2), "bf16"),
    (L("halo.dgrad.c304", 1, 230, 250, 304, 32, 3, 3, 1, 1, 1), "f16"),
    (L("halo.5x5.nopad", 1, 240, 260, 16, 160, 5, 5, 1, 0, 1), "bf16"),
    (L("halo.3x3.n224.c72", 1, 200, 333, 72, 224, 3, 3, 1, 1, 1), "bf16"),
    (L("halo.3x3.nopad", 2, 130, 140, 48, 128, 3, 3, 1, 0, 1), "f16"),
    (L("halo.3x3.k192.narrow-tile", 1, 210, 300, 24, 192, 3, 3, 1, 1, 1), "f16"),
    (L("halo.3x3.k152.one-160-tile", 1, 200, 280, 24, 152, 3, 3, 1, 1, 1), "bf16"),
    (L("halo.3x3.k288.128+160", 1, 150, 250, 40, 288, 3, 3, 1, 1, 1), "f16"),
]


@pytest.mark.parametrize("layer,dtype", HALO, ids=[l.name for l, _ in HALO])
def test_halo_tile_kernel(api, layer, dtype):
    check_layer(api, layer, dtype, synth.seed_for(0, 600 + len(layer.name)), x_kind="normal", n_samples=8192)


# 7x7 / stride 2 / padding 3 with 8 or 16 input channels: the data gradient takes the kernel that
# keeps the filter and a dy patch resident in LDS; odd and even image sizes (ragged patches, the
# last output row belonging to one parity class only), one and two chunks of K, ragged K chunk.
STEM = [
    (L("stem.c16.k64", 2, 61, 75, 16, 64, 7, 7, 2, 3, 1), "f16"),
    (L("stem.c16.k40.even", 1, 64, 96, 16, 40, 7, 7, 2, 3, 1), "bf16"),
    (L("stem.c8.k24", 1, 33, 130, 8, 24, 7, 7, 2, 3, 1), "f16"),
    (L("stem.c16.k8.tiny", 3, 5, 7, 16, 8, 7, 7, 2, 3, 1), "bf16"),
]


@pytest.mark.parametrize("layer,dtype", STEM, ids=[l.name for l, _ in STEM])
def test_stem_data_gradient_kernel(api, layer, dtype):
    check_layer(api, layer, dtype, synth.seed_for(0, 650 + len(layer.name)), x_kind="normal", passes=("dgrad",))


def test_wgrad_3x3_fused_taps(api):
    # large-image 3x3 filter gradient (all taps per workgroup): ragged strip, ragged channel block, ragged k
    check_layer(api, L("wgrad3x3.ragged", 1, 330, 1000, 40, 72, 3, 3, 1, 1, 1), "bf16", synth.seed_for(0, 700),
                x_kind="normal", passes=("wgrad",))
    check_layer(api, L("wgrad3x3.k264", 2, 400, 416, 32, 264, 3, 3, 1, 1, 1), "f16", synth.seed_for(0, 701),
                x_kind="normal", passes=("wgrad",))


def test_fp32_filter_gradient(api):
    layer = L("dw32", 2, 19, 23, 24, 40, 3, 3, 1, 1, 1)
    (x32, xb), _, (dy32, dyb) = U.conv_inputs(layer, "bf16", 77, "normal")
    desc = api.desc_from_layer(layer, "bf16", dw_f32=True)
    got = api.conv2d_bwd_filter(desc, U.to_device(xb, "bf16"), U.to_device(dyb, "bf16"))
    assert got.dtype == torch.float32
    ref = oracle.conv_bwd_filter(U.shape_of(layer), x32, dy32)
    assert U.rel_err(U.to_host_f64(got), ref) <= 1e-5       # fp32 accumulate, no output rounding


def test_run_to_run_determinism_and_redzones(api):
    layer = L("det", 2, 21, 26, 32, 48, 3, 3, 2, 1, 1)
    (_, xb), (_, wb), (_, dyb) = U.conv_inputs(layer, "f16", 99, "normal")
    desc = api.desc_from_layer(layer, "f16")
    xd, wd, dyd = U.to_device(xb, "f16"), U.to_device(wb, "f16"), U.to_device(dyb, "f16")
    guard = 64

    def guarded(shape):
        n = int(np.prod(shape))
        buf = torch.full((n + 2 * guard,), 123.0, dtype=torch.float16, device="cuda")
        return buf, buf[guard:guard + n].view(shape)

    outs = []
    for _ in range(2):
        by, y = guarded((layer.N, layer.P, layer.Q, layer.K))
        bdx, dx = guarded((layer.N, layer.H, layer.W, layer.C))
        bdw, dw = guarded((layer.K, layer.R, layer.S, layer.C))
        api.conv2d_fwd(desc, xd, wd, y=y)
        api.conv2d_bwd_data(desc, dyd, wd, dx=dx)
        api.conv2d_bwd_filter(desc, xd, dyd, dw=dw)
        torch.cuda.synchronize()
        for b in (by, bdx, bdw):
            assert torch.all(b[:guard] == 123.0) and torch.all(b[-guard:] == 123.0), "write outside the output"
        outs.append((y.clone(), dx.clone(), dw.clone()))
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b), "results differ between two identical runs"


# ---- the benchmark configurations -------------------------------------------
def test_config1(api):
    dtype, ls = layers.config1()
    check_layer(api, ls[0], dtype, synth.seed_for(1, 0), x_kind="normal")


def test_config2_stem(api):
    dtype, ls = layers.config2()
    check_layer(api, ls[0], dtype, synth.seed_for(2, 0), x_kind="fields", n_samples=16384)


@pytest.mark.parametrize("i", range(3))
def test_config3_bottleneck(api, i):
    dtype, ls = layers.config3()
    check_layer(api, ls[i], dtype, synth.seed_for(3, 10 * i))


@pytest.mark.parametrize("i", range(5))
def test_config4_aspp(api, i):
    dtype, ls = layers.config4()
    check_layer(api, ls[i], dtype, synth.seed_for(4, 10 * i), n_samples=8192)


_, CFG5 = layers.config5()


FULL_RES = ("dec.3x3.304-256", "dec.3x3.256-256", "logits.256-3")       # 87 % of the step's FLOPs


@pytest.mark.parametrize("layer", CFG5, ids=[l.name for l in CFG5])
def test_config5_full_size_layers(api, layer):
    """Every distinct layer shape of the network at its real size, fp16.  Whole tensors wherever the
    oracle's cost allows; the three full-resolution layers: 65536 uniformly drawn outputs plus every
    element of the first and last two rows and columns (forward, data gradient), and the filter
    gradient in full (1.1-1.2 T multiply-adds in the oracle, about a minute each)."""
    kind = "fields" if layer.name == "stem7x7" else "half_normal"
    big = layer.name in FULL_RES
    check_layer(api, layer, "f16", synth.seed_for(5, 10 * CFG5.index(layer)), x_kind=kind,
                n_samples=65536 if big else 16384, full_passes=("wgrad",) if big else ())
    torch.cuda.empty_cache()


def test_decoder_layer_bf16_full_size(api):
    """The dominant layer at its benchmark size in bfloat16: 3x3 halo kernel (forward, data gradient) on
    65536 outputs plus all border elements, the fused-tap filter-gradient kernel on 8 elements of every
    (32 output channels, tap, 32 input channels) block."""
    layer = [l for l in CFG5 if l.name == "dec.3x3.256-256"][0]
    check_layer(api, layer, "bf16", synth.seed_for(5, 777), n_samples=65536, dw_per_cell=8)
    torch.cuda.empty_cache()


# Whole-tensor comparisons for the two kernels that carry the decoder: cases small enough for the full
# oracle that still meet the kernels' selection rules (3x3 halo-tile kernel: >= 200 tiles; fused-tap
# filter gradient: >= 300 000 pixels).  Each column-tile width of the halo kernel (128, 160, <= 64
# channels) is reached from the forward pass (K) and from the data gradient (C); several channel chunks
# with a ragged last one; ragged patches on both image axes; both dtypes.
DOMINANT = [
    (L("full.halo3x3.k128", 2, 160, 320, 8, 128, 3, 3, 1, 1, 1), "f16", ("fwd", "dgrad")),
    (L("full.halo3x3.k160", 2, 160, 320, 8, 160, 3, 3, 1, 1, 1), "bf16", ("fwd", "dgrad")),
    (L("full.halo3x3.k64", 2, 160, 320, 8, 64, 3, 3, 1, 1, 1), "f16", ("fwd", "dgrad")),
    (L("full.halo3x3.c128", 2, 160, 320, 128, 8, 3, 3, 1, 1, 1), "bf16", ("fwd", "dgrad")),
    (L("full.halo3x3.c160", 2, 160, 320, 160, 8, 3, 3, 1, 1, 1), "f16", ("fwd", "dgrad")),
    (L("full.halo3x3.c64", 2, 160, 320, 64, 8, 3, 3, 1, 1, 1), "bf16", ("fwd", "dgrad")),
    (L("full.halo3x3.chunks.c72k128", 1, 170, 630, 72, 128, 3, 3, 1, 1, 1), "f16", ("fwd",)),
    (L("full.halo3x3.chunks.c128k72", 1, 170, 630, 128, 72, 3, 3, 1, 1, 1), "f16", ("dgrad",)),
    (L("full.halo3x3.k304.c40", 1, 165, 650, 40, 304, 3, 3, 1, 1, 1), "bf16", ("fwd",)),
    (L("full.halo3x3.c304.k16", 1, 165, 650, 304, 16, 3, 3, 1, 1, 1), "f16", ("dgrad",)),
    (L("full.wgrad3x3.c8k16", 1, 512, 608, 8, 16, 3, 3, 1, 1, 1), "f16", ("wgrad",)),
    (L("full.wgrad3x3.c40k72", 1, 515, 611, 40, 72, 3, 3, 1, 1, 1), "bf16", ("wgrad",)),
    (L("full.wgrad3x3.c304k256", 1, 400, 768, 304, 256, 3, 3, 1, 1, 1), "f16", ("wgrad",)),
]


@pytest.mark.parametrize("layer,dtype,passes", DOMINANT, ids=[l.name for l, _, _ in DOMINANT])
def test_dominant_kernels_whole_tensors(api, layer, dtype, passes):
    for which in passes:                       # keeps the oracle's share of the run to seconds per case
        assert layer.flops() <= {"fwd": 100e9, "dgrad": 25e9, "wgrad": 500e9}[which], (layer.name, which)
    check_layer(api, layer, dtype, synth.seed_for(0, 800 + [l.name for l, _, _ in DOMINANT].index(layer.name)),
                x_kind="normal", passes=passes, full_passes=passes)


def test_determinism_of_the_large_layer_kernels(api):
    """Two runs of the halo-tile, fused-tap filter-gradient and split-reduction paths give identical bits."""
    cases = [L("det.halo3x3", 2, 150, 170, 40, 256, 3, 3, 1, 1, 1),          # 3x3 halo kernel, ragged everything
             L("det.wgrad3x3", 1, 330, 1000, 40, 72, 3, 3, 1, 1, 1),         # fused-tap filter gradient
             L("det.ksplit", 1, 20, 24, 1000, 256, 3, 3, 1, 1, 1)]           # split reduction + ordered reduce
    for layer in cases:
        (_, xb), (_, wb), (_, dyb) = U.conv_inputs(layer, "f16", 4242, "normal")
        desc = api.desc_from_layer(layer, "f16")
        xd, wd, dyd = U.to_device(xb, "f16"), U.to_device(wb, "f16"), U.to_device(dyb, "f16")
        outs = []
        for _ in range(2):
            _say(f"[case] {layer.name} determinism run")
            y = api.conv2d_fwd(desc, xd, wd)
            dx = api.conv2d_bwd_data(desc, dyd, wd)
            dw = api.conv2d_bwd_filter(desc, xd, dyd)
            torch.cuda.synchronize()
            outs.append((y.clone(), dx.clone(), dw.clone()))
        for a, b in zip(outs[0], outs[1]):
            assert torch.equal(a, b), f"{layer.name}: results differ between two identical runs"


# ---- host-forceable errors on a GPU machine --------------------------------------
def test_argument_errors(api):
    layer = L("err", 1, 8, 8, 8, 8, 3, 3, 1, 1, 1)
    desc = api.desc_from_layer(layer, "f16")
    x = torch.zeros((1, 8, 8, 8), dtype=torch.float16, device="cuda")
    w = torch.zeros((8, 3, 3, 8), dtype=torch.float16, device="cuda")
    tiny = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(api.DlError) as e:
        api.conv2d_bwd_filter(desc, x, x, workspace=tiny)
    assert e.value.code == 5
    with pytest.raises(api.DlError) as e:
        api.conv2d_bwd_data(desc, x, w, workspace=tiny)
    assert e.value.code == 5
