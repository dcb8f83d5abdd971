"""Host-side checks of the layer tables (no GPU): shapes, counts and FLOP totals
of the reading of the paper's second network."""
from paper_1810_01993_amd import layers


def test_tiramisu_table_shapes():
    convs, deconvs = layers.tiramisu_layers(2, 768, 1152)
    # 2+2+2+4+5 down and 4+2+2+2 up dense layers, the first convolution, four transitions down, the logits
    # layer; four transitions up
    assert len(convs) == 15 + 10 + 1 + 4 + 1 and len(deconvs) == 4
    dense = [l for l in convs if ".5x5." in l.name]
    assert len(dense) == 25 and all(l.K == 32 and l.R == 5 and l.S == 5 and l.pad == 2 and l.stride == 1 for l in dense)
    assert [l.C for l in convs if "down1" in l.name] == [48, 80]
    assert [l.C for l in convs if "down5" in l.name] == [368, 400, 432, 464, 496]
    assert [l.C for l in convs if "up4" in l.name] == [528, 560, 592, 624]       # 160 up-sampled + 368 skipped
    assert [l.C for l in convs if "up1" in l.name] == [176, 208]                  # 64 up-sampled + 112 skipped
    assert [(l.C, l.K, l.stride) for l in convs if ".td" in l.name] == [(c, c, 2) for c in (112, 176, 240, 368)]
    assert [(l.C, l.H) for l in deconvs] == [(160, 96), (128, 192), (64, 384), (64, 768)]
    assert all((l.P, l.Q) == (l.H // 2, l.W // 2) for l in deconvs)
    assert convs[-1].C == 240 and convs[-1].K == 3
    per_sample = sum(l.flops() for l in convs + deconvs) / 2
    assert abs(per_sample - 1.238e12) < 2e9                                       # forward; x3 with both gradients


def test_deeplab_table_totals():
    dtype, table = layers.config5()
    assert dtype == "f16" and sum(l.count for l in table) == 63
    fwd = sum(l.flops() * l.count for l in table)
    assert abs(fwd - 5.2528e12) < 1e9                                             # N = 2: 2.63 TFLOP per sample
