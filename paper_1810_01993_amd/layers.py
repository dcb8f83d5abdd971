"""Layer shapes of the workload and the FLOP-count convention.

The network is the paper's modified DeepLabv3+ (Sec. "Segmentation
Architecture" and the caption of its network schematic): ResNet-50 encoder at
output stride 16, atrous spatial pyramid pooling, and a decoder that runs at
full resolution, on 16-channel 1152x768 fields with a per-GPU batch of 2 in
half precision (Sec. "Single GPU Performance").  The schematic itself does not
list every layer, so the table below is the standard ResNet-50 / ASPP layout
with the decoder's 3x3 convolutions and the 3-class logits at full resolution.

FLOPs follow Sec. "Performance Measurement": a convolution costs
2*R*S*P*Q*C*K*N (multiply and add both counted); the data gradient and the
filter gradient each cost the same as the forward pass.
"""
from __future__ import annotations

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class ConvLayer:
    name: str
    N: int
    H: int
    W: int
    C: int
    K: int
    R: int
    S: int
    stride: int = 1
    pad: int = 0
    dil: int = 1
    count: int = 1          # how many times this shape occurs in the network

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.dil * (self.R - 1) - 1) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.dil * (self.S - 1) - 1) // self.stride + 1

    def flops(self) -> int:
        """FLOPs of ONE pass (forward, or data gradient, or filter gradient)."""
        return conv_flops(self.R, self.S, self.P, self.Q, self.C, self.K, self.N)

    def bytes_fwd(self, elt: int = 2) -> int:
        """Compulsory bytes of one pass: every tensor touched once."""
        return elt * (self.N * self.H * self.W * self.C + self.K * self.R * self.S * self.C
                      + self.N * self.P * self.Q * self.K)


def conv_flops(R: int, S: int, P: int, Q: int, C: int, K: int, N: int) -> int:
    return 2 * R * S * P * Q * C * K * N


def deeplab_layers(N: int = 2, H: int = 768, W: int = 1152, full_res_decoder: bool = True):
    """The 30 distinct convolution shapes (63 layers) of the network."""
    h4, w4 = H // 4, W // 4        # after the stride-2 stem and the stride-2 max-pool
    h8, w8 = H // 8, W // 8
    h16, w16 = H // 16, W // 16
    hd, wd = (H, W) if full_res_decoder else (h4, w4)
    L = ConvLayer
    return [
        L("stem7x7", N, H, W, 16, 64, 7, 7, 2, 3, 1, 1),
        L("res2.1x1.64-64", N, h4, w4, 64, 64, 1, 1, 1, 0, 1, 1),
        L("res2.3x3.64", N, h4, w4, 64, 64, 3, 3, 1, 1, 1, 3),
        L("res2.1x1.64-256", N, h4, w4, 64, 256, 1, 1, 1, 0, 1, 4),
        L("res2.1x1.256-64", N, h4, w4, 256, 64, 1, 1, 1, 0, 1, 2),
        L("res3.1x1.256-128", N, h4, w4, 256, 128, 1, 1, 1, 0, 1, 1),
        L("res3.3x3.128.s2", N, h4, w4, 128, 128, 3, 3, 2, 1, 1, 1),
        L("res3.1x1.128-512", N, h8, w8, 128, 512, 1, 1, 1, 0, 1, 4),
        L("res3.short.256-512.s2", N, h4, w4, 256, 512, 1, 1, 2, 0, 1, 1),
        L("res3.1x1.512-128", N, h8, w8, 512, 128, 1, 1, 1, 0, 1, 3),
        L("res3.3x3.128", N, h8, w8, 128, 128, 3, 3, 1, 1, 1, 3),
        L("res4.1x1.512-256", N, h8, w8, 512, 256, 1, 1, 1, 0, 1, 1),
        L("res4.3x3.256.s2", N, h8, w8, 256, 256, 3, 3, 2, 1, 1, 1),
        L("res4.1x1.256-1024", N, h16, w16, 256, 1024, 1, 1, 1, 0, 1, 6),
        L("res4.short.512-1024.s2", N, h8, w8, 512, 1024, 1, 1, 2, 0, 1, 1),
        L("res4.1x1.1024-256", N, h16, w16, 1024, 256, 1, 1, 1, 0, 1, 5),
        L("res4.3x3.256", N, h16, w16, 256, 256, 3, 3, 1, 1, 1, 5),
        L("res5.1x1.1024-512", N, h16, w16, 1024, 512, 1, 1, 1, 0, 1, 1),
        L("res5.3x3.512.d2", N, h16, w16, 512, 512, 3, 3, 1, 2, 2, 3),
        L("res5.1x1.512-2048", N, h16, w16, 512, 2048, 1, 1, 1, 0, 1, 3),
        L("res5.short.1024-2048", N, h16, w16, 1024, 2048, 1, 1, 1, 0, 1, 1),
        L("res5.1x1.2048-512", N, h16, w16, 2048, 512, 1, 1, 1, 0, 1, 2),
        L("aspp.1x1.2048-256", N, h16, w16, 2048, 256, 1, 1, 1, 0, 1, 1),
        L("aspp.3x3.d6", N, h16, w16, 2048, 256, 3, 3, 1, 6, 6, 1),
        L("aspp.3x3.d12", N, h16, w16, 2048, 256, 3, 3, 1, 12, 12, 1),
        L("aspp.3x3.d18", N, h16, w16, 2048, 256, 3, 3, 1, 18, 18, 1),
        L("aspp.pool.1x1", N, 1, 1, 2048, 256, 1, 1, 1, 0, 1, 1),
        L("aspp.proj.1280-256", N, h16, w16, 1280, 256, 1, 1, 1, 0, 1, 1),
        L("dec.low.256-48", N, h4, w4, 256, 48, 1, 1, 1, 0, 1, 1),
        L("dec.3x3.304-256", N, hd, wd, 304, 256, 3, 3, 1, 1, 1, 1),
        L("dec.3x3.256-256", N, hd, wd, 256, 256, 3, 3, 1, 1, 1, 1),
        L("logits.256-3", N, hd, wd, 256, 3, 1, 1, 1, 0, 1, 1),
    ]


def total_flops(layers, passes: int = 3) -> int:
    return passes * sum(l.flops() * l.count for l in layers)


# ---- the five benchmark / parity configurations ---------------------------
def config1():
    """Single atrous 3x3, fp16."""
    return "f16", [ConvLayer("cfg1.3x3.d2", 1, 96, 144, 16, 64, 3, 3, 1, 2, 2)]


def config2():
    """Encoder stem, bf16."""
    return "bf16", [ConvLayer("cfg2.stem7x7", 2, 768, 1152, 16, 64, 7, 7, 2, 3, 1)]


def config3():
    """ResNet-50 bottleneck at output stride 16, bf16."""
    return "bf16", [
        ConvLayer("cfg3.1x1.1024-256", 2, 48, 72, 1024, 256, 1, 1, 1, 0, 1),
        ConvLayer("cfg3.3x3.256.d2", 2, 48, 72, 256, 256, 3, 3, 1, 2, 2),
        ConvLayer("cfg3.1x1.256-1024", 2, 48, 72, 256, 1024, 1, 1, 1, 0, 1),
    ]


def config4():
    """ASPP block, bf16."""
    return "bf16", [
        ConvLayer("cfg4.aspp.1x1", 2, 48, 72, 2048, 256, 1, 1, 1, 0, 1),
        ConvLayer("cfg4.aspp.3x3.d6", 2, 48, 72, 2048, 256, 3, 3, 1, 6, 6),
        ConvLayer("cfg4.aspp.3x3.d12", 2, 48, 72, 2048, 256, 3, 3, 1, 12, 12),
        ConvLayer("cfg4.aspp.3x3.d18", 2, 48, 72, 2048, 256, 3, 3, 1, 18, 18),
        ConvLayer("cfg4.aspp.proj", 2, 48, 72, 1280, 256, 1, 1, 1, 0, 1),
    ]


def deconv_layers(N: int = 2, H: int = 768, W: int = 1152):
    """The decoder's up-sampling path as transposed convolutions (the network
    schematic's caption names deconvolutional layers in the full-resolution
    decoder; it does not give their shapes).  Reading: 3x3, stride 2, padding 1,
    256 -> 256 channels, each doubling the resolution, from the encoder's
    output stride 16 up to full resolution.  Each entry is the UNDERLYING
    convolution (the layer is its adjoint): (H, W, C) is the layer's output,
    K its input channels, (P, Q) = (H/2, W/2) its input size."""
    L = ConvLayer
    return [L(f"deconv.3x3.s2.256.to-{H // f}x{W // f}", N, H // f, W // f, 256, 256, 3, 3, 2, 1, 1, 1)
            for f in (8, 4, 2, 1)]


def tiramisu_layers(N: int = 2, H: int = 768, W: int = 1152):
    """The paper's other segmentation network (Sec. "Segmentation Architecture" and
    "Modifications to the neural network architectures"): a Tiramisu (fully
    convolutional DenseNet) with five dense blocks in each direction of 2, 2, 2, 4
    and 5 layers (top to bottom), growth rate 32 and 5x5 convolutions.  The paper
    gives no layer list; this reading fills the rest in from the network the paper
    modifies: a 3x3 first convolution to 48 channels; every dense-block layer sees
    the block's input concatenated with the outputs of the layers before it and adds
    32 channels; a transition down is a 1x1 convolution of all channels with stride 2
    (the paper's schematic caption says transitions down use stride-2 convolutions);
    a transition up is a 3x3 stride-2 transposed convolution of the channels the
    block below has added; the up blocks see that concatenated with the skip
    connection; a 1x1 convolution maps the last 240 channels to the 3 classes.
    That is 1.24 TFLOP per sample forward, 3.7 with both gradients, against the
    4.19 TFLOP per sample the paper counts for its network.

    Returns (convolutions, transposed convolutions); a transposed entry is the
    UNDERLYING convolution, as in deconv_layers()."""
    L = ConvLayer
    growth, first = 32, 48
    per_block = (2, 2, 2, 4, 5)
    convs, deconvs = [L("tira.first.3x3", N, H, W, 16, first, 3, 3, 1, 1, 1)], []
    ch, skips = first, []
    for b, n_layers in enumerate(per_block):                       # down path, block b at 1 / 2^b resolution
        h, w = H >> b, W >> b
        for i in range(n_layers):
            convs.append(L(f"tira.down{b + 1}.5x5.{ch + i * growth}-32", N, h, w, ch + i * growth, growth, 5, 5, 1, 2, 1))
        added = n_layers * growth
        ch += added
        if b + 1 < len(per_block):
            skips.append(ch)
            convs.append(L(f"tira.td{b + 1}.1x1.s2.{ch}", N, h, w, ch, ch, 1, 1, 2, 0, 1))
    for b in range(len(per_block) - 2, -1, -1):                    # up path, block b at 1 / 2^b resolution
        h, w = H >> b, W >> b
        deconvs.append(L(f"tira.tu{b + 1}.3x3.s2.{added}", N, h, w, added, added, 3, 3, 2, 1, 1))
        ch = added + skips[b]
        n_layers = per_block[b]
        for i in range(n_layers):
            convs.append(L(f"tira.up{b + 1}.5x5.{ch + i * growth}-32", N, h, w, ch + i * growth, growth, 5, 5, 1, 2, 1))
        added = n_layers * growth
    convs.append(L("tira.logits.1x1", N, H, W, ch + added, 3, 1, 1, 1, 0, 1))
    return convs, deconvs


def config5():
    """Whole conv stack + loss, one GPU's share, fp16."""
    return "f16", deeplab_layers(2, 768, 1152, True)


def scaled(layer: ConvLayer, **kw) -> ConvLayer:
    return replace(layer, **kw)
