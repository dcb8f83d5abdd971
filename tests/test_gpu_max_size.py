"""GPU parity at the largest tensors the boundary accepts (just under 2^31
elements, 4.3 GB per activation tensor): the kernels' 32-bit byte offsets and
the out-of-range marker are exercised at the far end of the address range.
Inputs are drawn on the device (seeded) and copied to the host for the
single-element oracle; sampled outputs concentrate on the last rows."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_1810_01993_amd.layers import ConvLayer

import gpu_util as U

pytestmark = pytest.mark.gpu

MAX_ELEMS = 0x7FF00000          # the boundary rejects tensors of this many elements or more


@pytest.fixture(scope="module")
def api():
    from paper_1810_01993_amd import api as _api
    assert torch.cuda.is_available(), "a GPU is required for -m gpu tests"
    return _api


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _device_inputs(layer, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    x = torch.randn((layer.N, layer.H, layer.W, layer.C), generator=g, device="cuda", dtype=torch.float16)
    sigma = float(np.sqrt(2.0 / (layer.R * layer.S * layer.C)))
    w = (torch.randn((layer.K, layer.R, layer.S, layer.C), generator=g, device="cuda") * sigma).half()
    dy = torch.randn((layer.N, layer.P, layer.Q, layer.K), generator=g, device="cuda", dtype=torch.float16)
    return x, w, dy


def _host32(t):
    return t.cpu().numpy().astype(np.float32)


def _tail_heavy_indices(shape, n, seed):
    """Half of the samples uniform, half from the last 1/1024 of the tensor."""
    total = int(np.prod(shape))
    g = np.random.default_rng(seed)
    tail = total - total // 1024
    return np.unique(np.concatenate([g.integers(0, total, n // 2), g.integers(tail, total, n // 2),
                                     np.array([0, total - 1])]))


def _check(layer, api, seed, n_samples, n_dw):
    assert layer.N * layer.H * layer.W * layer.C < MAX_ELEMS
    s = U.shape_of(layer)
    desc = api.desc_from_layer(layer, "f16")
    _say(f"[case] max-size {layer.name}: x {layer.N}x{layer.H}x{layer.W}x{layer.C} "
         f"({layer.N * layer.H * layer.W * layer.C} elements) -> K {layer.K}, {layer.R}x{layer.S}: drawing inputs")
    x, w, dy = _device_inputs(layer, seed)
    _say("[step] forward")
    y = api.conv2d_fwd(desc, x, w)
    torch.cuda.synchronize()
    x32, w32 = _host32(x), _host32(w)
    idx = _tail_heavy_indices(y.shape, n_samples, seed)
    got = y.view(-1)[torch.from_numpy(idx).cuda()].double().cpu().numpy()
    assert U.rel_err(got, oracle.conv_fwd_at(s, x32, w32, idx)) <= U.TOL["f16"]
    del y
    _say("[step] filter gradient")
    dw = api.conv2d_bwd_filter(desc, x, dy)
    torch.cuda.synchronize()
    dy32 = _host32(dy)
    idw = np.unique(np.random.default_rng(seed + 1).integers(0, dw.numel(), n_dw))
    got = dw.view(-1)[torch.from_numpy(idw).cuda()].double().cpu().numpy()
    assert U.rel_err(got, oracle.conv_bwd_filter_at(s, x32, dy32, idw)) <= U.TOL["f16"]
    del x, x32, dw
    _say("[step] data gradient")
    dx = api.conv2d_bwd_data(desc, dy, w)
    torch.cuda.synchronize()
    idx = _tail_heavy_indices(dx.shape, n_samples, seed + 2)
    got = dx.view(-1)[torch.from_numpy(idx).cuda()].double().cpu().numpy()
    assert U.rel_err(got, oracle.conv_bwd_data_at(s, dy32, w32, idx)) <= U.TOL["f16"]


def test_largest_1x1_activation_tensor(api):
    # 4093 x 4096 pixels x 128 channels = 2 145 910 784 elements (limit 2 146 435 072)
    _check(ConvLayer("max.1x1.c128k8", 1, 4093, 4096, 128, 8, 1, 1, 1, 0, 1), api, 4101, 4000, 64)


def test_largest_3x3_image(api):
    # 16376 x 16380 pixels x 8 channels on both sides: the 3x3 halo-tile and fused-tap kernels
    # at the far end of their 32-bit offsets
    _check(ConvLayer("max.3x3.c8k8", 1, 16376, 16380, 8, 8, 3, 3, 1, 1, 1), api, 4102, 4000, 24)
