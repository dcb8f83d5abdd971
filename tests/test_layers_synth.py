"""Host-side checks: FLOP convention, layer table, seeded generators."""
import numpy as np

from paper_1810_01993_amd import layers, synth
from test_oracle_loss import _golden


def test_flop_example_from_the_paper():
    g = _golden()
    n = layers.conv_flops(int(g["flop_example_R"]), int(g["flop_example_S"]), int(g["flop_example_H"]),
                          int(g["flop_example_W"]), int(g["flop_example_C"]), int(g["flop_example_K"]),
                          int(g["flop_example_N"]))
    assert n == 48_922_361_856
    assert abs(n - g["flop_example_total"]) / g["flop_example_total"] < 1e-3


def test_backward_counts_twice_forward():
    g = _golden()
    assert abs(g["deeplab_fp16_bwd_conv_TF"] / g["deeplab_fp16_fwd_conv_TF"] - 2) < 1e-2
    assert abs(g["deeplab_fp32_bwd_conv_TF"] / g["deeplab_fp32_fwd_conv_TF"] - 2) < 1e-2
    L = layers.deeplab_layers()
    fwd = sum(l.flops() * l.count for l in L)
    assert layers.total_flops(L, passes=3) == 3 * fwd


def test_layer_table_shapes_chain():
    L = {l.name: l for l in layers.deeplab_layers()}
    assert sum(l.count for l in L.values()) == 63
    assert (L["stem7x7"].P, L["stem7x7"].Q) == (384, 576)
    assert (L["res3.3x3.128.s2"].P, L["res3.3x3.128.s2"].Q) == (96, 144)
    assert (L["res4.short.512-1024.s2"].P, L["res4.short.512-1024.s2"].Q) == (48, 72)
    for n in ("aspp.3x3.d6", "aspp.3x3.d12", "aspp.3x3.d18", "res5.3x3.512.d2"):
        assert (L[n].P, L[n].Q) == (48, 72)
    assert L["dec.3x3.304-256"].C == 256 + L["dec.low.256-48"].K
    assert (L["logits.256-3"].P, L["logits.256-3"].Q, L["logits.256-3"].K) == (768, 1152, 3)
    fwd = sum(l.flops() * l.count for l in L.values())
    assert abs(fwd / 2 / 1e12 - 2.63) < 0.01          # TF per sample, forward
    dec = L["dec.3x3.304-256"].flops() + L["dec.3x3.256-256"].flops()
    assert 0.86 < dec / fwd < 0.88


def test_quantize_roundtrip_and_ties():
    a = np.array([1.0, 1.0 + 2 ** -9, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -9, -2.5, 0.0, 3.0e38], dtype=np.float32)
    v, bits = synth.quantize(a, "bf16")
    # bf16 has 8 significand bits: spacing 2^-7 at 1.0; 1+2^-8 is a tie -> even (1.0); 1+3*2^-9 rounds up
    assert v[0] == 1.0 and v[1] == 1.0 and v[2] == 1.0 and v[3] == np.float32(1.0 + 2 ** -7)
    assert v[4] == -2.5 and v[5] == 0.0 and np.isfinite(v[6])
    assert np.array_equal(synth.bits_to_f32(bits, "bf16"), v)
    v16, b16 = synth.quantize(a[:6], "f16")
    assert np.array_equal(synth.bits_to_f32(b16, "f16"), v16)
    assert v16[1] == 1.0 + 2 ** -9 and v16[4] == -2.5
    # values survive a second rounding unchanged
    assert np.array_equal(synth.quantize(v, "bf16")[0], v)


def test_generators_are_seeded_and_have_the_stated_statistics():
    a, b = synth.normal(5, (1000, 64)), synth.normal(5, (1000, 64))
    assert np.array_equal(a, b) and not np.array_equal(a, synth.normal(6, (1000, 64)))
    assert abs(a.mean()) < 0.02 and abs(a.std() - 1) < 0.02
    h = synth.half_normal(7, (1000, 64))
    assert h.min() >= 0 and abs(h.mean() - np.sqrt(2 / np.pi)) < 0.02
    w = synth.he_filter(8, 64, 3, 3, 16)
    assert w.shape == (64, 3, 3, 16) and abs(w.std() - np.sqrt(2 / 144)) < 0.005


def test_smooth_fields_are_normalised_and_smooth():
    f = synth.smooth_fields(9, 1, 96, 144, 4)
    assert f.shape == (1, 96, 144, 4)
    np.testing.assert_allclose(f.mean(axis=(0, 1, 2)), 0, atol=1e-4)
    np.testing.assert_allclose(f.std(axis=(0, 1, 2)), 1, atol=1e-4)
    # neighbouring pixels are strongly correlated (sigma = 8 px), and longitude wraps
    assert np.corrcoef(f[0, :, :-1, 0].ravel(), f[0, :, 1:, 0].ravel())[0, 1] > 0.98
    assert np.corrcoef(f[0, :, 0, 0], f[0, :, -1, 0])[0, 1] > 0.98


def test_ellipse_labels_match_class_balance():
    lab = synth.ellipse_labels(10, 2, 192, 288)
    assert lab.dtype == np.uint8 and lab.shape == (2, 192, 288) and lab.max() == 2
    frac = np.bincount(lab.ravel(), minlength=3) / lab.size
    assert abs(frac[1] - 0.017) < 5e-4 and abs(frac[2] - 0.001) < 5e-4
    assert np.array_equal(lab, synth.ellipse_labels(10, 2, 192, 288))
