"""Host-only checks of the C boundary: the library loads without a GPU,
exports every symbol the header declares, and rejects bad arguments before
touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def api():
    from paper_1810_01993_amd import build
    if not os.path.exists(build.LIB):
        build.build_library()
    from paper_1810_01993_amd import api as _api
    return _api


def test_every_declared_symbol_is_exported(api):
    header = open(os.path.join(ROOT, "include", "dlconv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(\w+)\s*\([^;{]*\)\s*;", header))
    assert {"conv2d_fwd", "conv2d_bwd_data", "conv2d_bwd_filter", "weighted_pixel_ce_fwd_bwd"} <= declared
    lib = ctypes.CDLL(api.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in dlconv.h but not exported"
    assert declared == set(api.EXPORTS)
    # the measurement aids have a header of their own
    probe = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "dlprobe.h")).read(), flags=re.S)
    declared_probe = set(re.findall(r"\b(\w+)\s*\([^;{]*\)\s*;", probe))
    assert declared_probe == set(api.PROBE_EXPORTS)
    for name in declared_probe:
        assert hasattr(lib, name), f"{name} is declared in dlprobe.h but not exported"
    assert set(os.listdir(os.path.join(ROOT, "include"))) == {"dlconv.h", "dlprobe.h"}


def test_out_shape_and_workspace_queries(api):
    d = api.ConvDesc(2, 768, 1152, 16, 64, 7, 7, 2, 2, 3, 3, 1, 1, api.DL_BF16)
    assert api.dl_conv_out_shape(d) == (384, 576)
    assert api.dl_conv_workspace_bytes(d, api.PASS_FWD) == 0
    # data gradient: room for the re-laid-out filter (every tap lands in exactly one parity class)
    assert api.dl_conv_workspace_bytes(d, api.PASS_BWD_DATA) >= 64 * 7 * 7 * 16 * 2
    ws = api.dl_conv_workspace_bytes(d, api.PASS_BWD_FILTER)
    assert ws >= 64 * 7 * 7 * 16 * 4 and ws % (64 * 7 * 7 * 16 * 4) == 0
    assert api.dl_ce_workspace_bytes(0) >= 4
    assert api.dl_ce_workspace_bytes(2 * 768 * 1152) >= 4


def _code(fn, *a):
    with pytest.raises(Exception) as e:
        fn(*a)
    return e.value.code


def test_descriptor_validation(api):
    ok = dict(N=1, H=8, W=8, C=8, K=8, R=3, S=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1, dil_h=1, dil_w=1,
              dtype=api.DL_F16)
    assert api.dl_conv_out_shape(api.ConvDesc(**ok)) == (8, 8)
    for field, bad in [("N", 0), ("C", -1), ("K", 0), ("R", 0), ("stride_h", 0), ("dil_w", 0), ("pad_h", -1)]:
        assert _code(api.dl_conv_out_shape, api.ConvDesc(**{**ok, field: bad})) == 2, field
    assert _code(api.dl_conv_out_shape, api.ConvDesc(**{**ok, "H": 2, "pad_h": 0, "dil_h": 2})) == 2   # empty output
    assert _code(api.dl_conv_out_shape, api.ConvDesc(**{**ok, "dtype": api.DL_F32})) == 3
    assert _code(api.dl_conv_out_shape, api.ConvDesc(**{**ok, "dtype": api.DL_F16, "dw_dtype": api.DL_BF16})) == 3
    assert _code(api.dl_conv_out_shape, api.ConvDesc(**{**ok, "N": 4096, "H": 4096, "W": 4096})) == 2  # index overflow
    assert _code(api.dl_conv_workspace_bytes, api.ConvDesc(**ok), 7) == 6


def test_pointer_checks_happen_before_any_launch(api):
    lib = api._lib
    d = api.ConvDesc(1, 8, 8, 8, 8, 3, 3, 1, 1, 1, 1, 1, 1, api.DL_F16).c_struct()
    ref = ctypes.byref(d)
    for fn in (lib.conv2d_fwd, lib.conv2d_bwd_data, lib.conv2d_bwd_filter):
        assert fn(ref, None, None, None, None, 0, None) == 1           # null
        assert fn(None, 16, 16, 16, None, 0, None) == 1
        assert fn(ref, 16, 16, 24, None, 0, None) == 4                 # misaligned
    assert lib.conv2d_bwd_data(ref, 16, 16, 16, None, 0, None) == 5    # workspace missing
    assert lib.conv2d_bwd_filter(ref, 16, 16, 16, 32, 8, None) == 5    # workspace too small
    assert lib.weighted_pixel_ce_fwd_bwd(None, 0, None, None, 1.0, 8, None, None, None, 0, None) == 1
    assert lib.weighted_pixel_ce_fwd_bwd(16, 2, 16, 16, 1.0, 8, 16, 16, 16, 64, None) == 3
    assert lib.weighted_pixel_ce_fwd_bwd(16, 0, 16, 16, 1.0, -1, 16, 16, 16, 64, None) == 2
    assert lib.weighted_pixel_ce_fwd_bwd(16, 0, 16, 16, 1.0, 8, 16, 16, None, 0, None) == 5
    assert lib.weighted_pixel_ce_fwd_bwd(16, 0, 16, 16, 1.0, 8, 16, 24, 16, 64, None) == 4
    # the entry point without a workspace: same checks, plus its size limit, all before the first HIP call
    assert lib.weighted_pixel_ce_fwd_bwd_static(16, 0, 16, 16, 1.0, api.CE_STATIC_MAX_PIXELS + 1, 16, 16, None) == 2
    assert lib.weighted_pixel_ce_fwd_bwd_static(16, 0, 16, 16, 1.0, 8, None, 16, None) == 1
    assert lib.weighted_pixel_ce_map_fwd_bwd(16, 0, 16, None, 1.0, 8, 16, 16, 16, 64, None) == 1   # no weight map
    assert lib.weighted_pixel_ce_map_fwd_bwd(16, 0, 16, 24, 1.0, 8, 16, 16, 16, 64, None) == 4     # map misaligned
    assert lib.weighted_pixel_ce_map_fwd_bwd(16, 0, 16, 16, 1.0, 8, 16, 16, None, 0, None) == 5
    for fn in (lib.conv2d_transpose_fwd, lib.conv2d_transpose_bwd_data, lib.conv2d_transpose_bwd_filter):
        assert fn(ref, None, None, None, None, 0, None) == 1
        assert fn(ref, 16, 16, 24, None, 0, None) == 4
    assert lib.conv2d_fwd_bias_relu(ref, None, 16, None, 1, 16, None, 0, None) == 1
    assert lib.conv2d_fwd_bias_relu(ref, 16, 16, 18, 1, 16, None, 0, None) == 4                    # bias not 4-byte aligned
    assert lib.bias_relu_bwd(16, 16, 0, 8, 8, 1, 16, None, 16, 4096, None) == 1            # no dbias
    assert lib.bias_relu_bwd(16, None, 0, 8, 8, 1, 16, 16, 16, 4096, None) == 1            # ReLU needs y
    assert lib.bias_relu_bwd(16, 16, 2, 8, 8, 1, 16, 16, 16, 4096, None) == 3
    assert lib.bias_relu_bwd(16, 16, 0, 8, 0, 1, 16, 16, 16, 4096, None) == 2
    assert lib.bias_relu_bwd(16, 16, 0, 8, 8, 1, 16, 16, None, 0, None) == 5
    t = (api._LarcTensor * 2)(api._LarcTensor(16, 16, None, 8), api._LarcTensor(16, None, None, 8))
    tp = ctypes.cast(t, ctypes.c_void_p)
    f = ctypes.c_float
    assert lib.larc_sgd_step(tp, 2, 0, f(.1), f(.02), f(0), f(0), f(0), 1, None, 16, 1 << 20, None) == 1   # tensor 1 has no gradient
    assert lib.larc_sgd_step(tp, 1, 0, f(.1), f(.02), f(0), f(.9), f(0), 1, None, 16, 1 << 20, None) == 1  # momentum needs v
    assert lib.larc_sgd_step(tp, 1, 7, f(.1), f(.02), f(0), f(0), f(0), 1, None, 16, 1 << 20, None) == 3
    assert lib.larc_sgd_step(tp, 1, 0, f(.1), f(.02), f(0), f(0), f(0), 1, None, 16, 8, None) == 5
    assert lib.larc_sgd_step(None, 0, 0, f(.1), f(.02), f(0), f(0), f(0), 1, None, None, 0, None) == 0     # nothing to do
    assert lib.dl_status_string(0) == b"ok" and b"workspace" in lib.dl_status_string(5)
    flop = ctypes.c_double()
    assert lib.dl_probe_mfma(0, 0, 10, None, 16, ctypes.byref(flop), None) == 1
    assert lib.dl_probe_mfma(2, 0, 10, 16, 16, ctypes.byref(flop), None) == 2
    assert lib.dl_probe_stream(1, 16, None, 16, 3073, 16, None) == 2
    assert lib.dl_probe_stream(3, 16, None, 16, 3072, 16, None) == 1


_DISPATCH_PROBE = r"""
import sys
sys.path.insert(0, %r)
from paper_1810_01993_amd import api
out = []
shapes = [(2, 768, 1152, 256, 256, 3, 1, 1, 1),     # decoder 3x3: halo-tile kernel, fused-tap filter gradient
          (2, 48, 72, 2048, 256, 3, 1, 6, 6),       # ASPP 3x3: split reduction
          (2, 48, 72, 1024, 256, 1, 1, 0, 1),       # 1x1
          (2, 192, 288, 128, 128, 3, 2, 1, 1),      # stride 2: parity classes in one launch
          (2, 768, 1152, 16, 64, 7, 2, 3, 1),       # stem
          (2, 768, 1152, 208, 32, 5, 1, 2, 1)]      # 5x5 with 32 output channels
for (N, H, W, C, K, R, st, pad, dil) in shapes:
    d = api.ConvDesc(N, H, W, C, K, R, R, st, st, pad, pad, dil, dil, api.DL_F16)
    out.append([api.dl_conv_workspace_bytes(d, p) for p in (0, 1, 2)])
out.append(api.dl_ce_workspace_bytes(2 * 768 * 1152))
print(out)
"""


def test_dispatch_does_not_read_the_environment(api):
    """The library has no run-time knobs: the sweep variables of the tuning build change nothing (the
    workspace sizes follow the kernel choice, the split of reductions and the slice plans), no source
    file calls getenv outside the tuning build's helper, and the built library does not import it."""
    import subprocess
    import sys
    knobs = {"DLCONV_HALO": "0", "DLCONV_KSPLIT": "0", "DLCONV_WGRAD_CFG": "1", "DLCONV_WGRAD3X3": "0",
             "DLCONV_WGRAD5X5": "0", "DLCONV_NARROW": "0", "DLCONV_WIDE5X5": "0", "DLCONV_DGRAD_STEM": "0",
             "DLCONV_IGEMM_CFG": "103", "DLCONV_BATCH": "0", "DLCONV_BT": "0", "DLCONV_CE_BLOCKS": "7",
             "DLCONV_WGRAD_TARGET": "64", "DLCONV_C_OUTER": "0", "DLCONV_CFG128_MIN": "1", "DLCONV_REDUCE4": "0"}
    clean = {k: v for k, v in os.environ.items() if not k.startswith("DLCONV_")}
    code = _DISPATCH_PROBE % ROOT
    plain = subprocess.run([sys.executable, "-c", code], env=clean, capture_output=True, text=True, check=True).stdout
    steered = subprocess.run([sys.executable, "-c", code], env={**clean, **knobs}, capture_output=True, text=True,
                             check=True).stdout
    assert plain == steered and plain.strip().startswith("[[")
    csrc = os.path.join(ROOT, "paper_1810_01993_amd", "csrc")
    for name in os.listdir(csrc):
        if name.endswith(".hip"):
            assert "getenv" not in open(os.path.join(csrc, name)).read(), name
    syms = subprocess.run(["nm", "-D", "--undefined-only", api.LIB_PATH], capture_output=True, text=True, check=True).stdout
    assert "getenv" not in syms


def test_describe_names_the_kernels_of_the_decoder_layers(api):
    """dl_conv_describe runs the entry points' own dispatch with launches logged instead of issued
    (no GPU needed): the layers that carry 87 % of the FLOPs must reach the kernels built for them."""
    dec = api.ConvDesc(2, 768, 1152, 256, 256, 3, 3, 1, 1, 1, 1, 1, 1, api.DL_F16)
    assert "igemm_halo3x3_kernel<4>[6912]" in api.dl_conv_describe(dec, api.PASS_FWD)
    assert "igemm_halo3x3_kernel<4>[6912]" in api.dl_conv_describe(dec, api.PASS_BWD_DATA)
    assert api.dl_conv_describe(dec, api.PASS_BWD_FILTER).startswith("wgrad3x3_kernel[")
    dec304 = api.ConvDesc(2, 768, 1152, 304, 256, 3, 3, 1, 1, 1, 1, 1, 1, api.DL_BF16)
    assert "igemm_halo3x3_kernel<5>[6912]" in api.dl_conv_describe(dec304, api.PASS_BWD_DATA)
    stem = api.ConvDesc(2, 768, 1152, 16, 64, 7, 7, 2, 2, 3, 3, 1, 1, api.DL_F16)
    assert "dgrad_stem_kernel" in api.dl_conv_describe(stem, api.PASS_BWD_DATA)
    logits = api.ConvDesc(2, 768, 1152, 256, 3, 1, 1, 1, 1, 0, 0, 1, 1, api.DL_F16)
    assert api.dl_conv_describe(logits, api.PASS_FWD) == "thin_cols_kernel[2048]"
    assert "thin_rows_kernel" in api.dl_conv_describe(logits, api.PASS_BWD_DATA)
    assert "thin_wgrad_kernel" in api.dl_conv_describe(logits, api.PASS_BWD_FILTER)
    # the query leaves nothing behind: a call after it still validates and reports as before
    assert api._lib.conv2d_fwd(ctypes.byref(dec.c_struct()), None, None, None, None, 0, None) == 1
    assert _code(api.dl_conv_describe, api.ConvDesc(2, 8, 8, 8, 8, 3, 3, 1, 1, 1, 1, 1, 1, api.DL_F16), 5) == 6
