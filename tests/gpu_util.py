"""Helpers shared by the GPU parity tests: seeded inputs -> device tensors,
oracle evaluation (full or sampled), and the max|err|/max|ref| measure."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_1810_01993_amd import synth

TOL = {"f16": 2e-3, "bf16": 8e-3}          # max|err| / max|ref|
TORCH_DTYPE = {"f16": torch.float16, "bf16": torch.bfloat16}
FULL_ORACLE_FLOPS = 3e9                    # the fused / transposed variants: above this, sampled outputs
# Convolution passes (check_layer): whole tensors up to these sizes.  The forward and filter-gradient
# oracles run ~30 GFLOP/s on the test box's 16 cores (about 3 s at the limit), the scatter-form data
# gradient about 3.6 GFLOP/s; above the limit the sampled comparison below takes over.
FULL_LIMIT = {"fwd": 100e9, "wgrad": 100e9, "dgrad": 12e9}
BORDER_CAP = 6_000_000                     # every border element up to this many, a random subset beyond
FP16_MAX_REF = 6e4                         # an fp16 case whose exact result leaves fp16's range is a bad case, not a bad kernel


def to_device(bits: np.ndarray, dtype: str) -> torch.Tensor:
    """uint16 storage bits -> device tensor of the matching 16-bit float type."""
    return torch.from_numpy(bits.view(np.int16)).view(TORCH_DTYPE[dtype]).cuda()


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def shape_of(layer) -> oracle.ConvShape:
    return oracle.ConvShape(layer.N, layer.H, layer.W, layer.C, layer.K, layer.R, layer.S,
                            layer.stride, layer.pad, layer.dil)


def conv_inputs(layer, dtype: str, seed: int, x_kind: str = "half_normal"):
    """(values32, bits) for x, w, dy of one layer, rounded once to dtype."""
    xs = (layer.N, layer.H, layer.W, layer.C)
    if x_kind == "normal":
        x = synth.normal(seed, xs)
    elif x_kind == "half_normal":
        x = synth.half_normal(seed, xs)
    elif x_kind == "fields":
        x = synth.smooth_fields(seed, *xs)
    else:
        raise ValueError(x_kind)
    w = synth.he_filter(seed + 1, layer.K, layer.R, layer.S, layer.C)
    dy = synth.normal(seed + 2, (layer.N, layer.P, layer.Q, layer.K))
    return synth.quantize(x, dtype), synth.quantize(w, dtype), synth.quantize(dy, dtype)


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    denom = float(np.max(np.abs(ref))) if ref.size else 0.0
    if ref.size == 0:
        return 0.0
    if denom == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref))) / denom


def sample_indices(shape, n_random: int, seed: int) -> np.ndarray:
    """n_random uniformly drawn flat indices into a tensor of this shape (sorted, duplicates removed)."""
    total = int(np.prod(shape))
    g = np.random.default_rng(seed)
    return np.unique(g.integers(0, total, size=min(n_random, total)))


def border_indices(shape, per_edge: int, seed: int) -> np.ndarray:
    """Random elements restricted to the outermost two rows / columns of an
    [N, H, W, C] tensor, where padding taps matter."""
    N, H, W, C = shape
    g = np.random.default_rng(seed)
    out = []
    rows = np.unique(np.clip(np.array([0, 1, H - 2, H - 1]), 0, H - 1))
    cols = np.unique(np.clip(np.array([0, 1, W - 2, W - 1]), 0, W - 1))
    n = g.integers(0, N, per_edge); c = g.integers(0, C, per_edge)
    out.append(((n * H + g.choice(rows, per_edge)) * W + g.integers(0, W, per_edge)) * C + c)
    out.append(((n * H + g.integers(0, H, per_edge)) * W + g.choice(cols, per_edge)) * C + c)
    return np.unique(np.concatenate(out))


def all_border_indices(shape, seed: int, cap: int = BORDER_CAP) -> np.ndarray:
    """Every element of an [N, H, W, C] tensor whose pixel lies in the first or last two rows or
    columns (all images, all channels); a seeded random subset of `cap` of them if there are more."""
    N, H, W, C = shape
    edge = np.zeros((H, W), dtype=bool)
    edge[:2, :] = True
    edge[-2:, :] = True
    edge[:, :2] = True
    edge[:, -2:] = True
    pix = np.flatnonzero(edge)                                      # h * W + w
    idx = ((np.arange(N, dtype=np.int64)[:, None] * (H * W) + pix[None, :]).reshape(-1, 1) * C
           + np.arange(C, dtype=np.int64)[None, :]).ravel()
    if idx.size > cap:
        idx = np.sort(np.random.default_rng(seed).choice(idx, size=cap, replace=False))
    return idx


def stratified_filter_indices(shape, per_cell: int, seed: int, block: int = 32) -> np.ndarray:
    """Flat indices into a filter tensor [K, R, S, C]: `per_cell` random elements in every
    (block of 32 output channels, tap, block of 32 input channels) cell, so that no tile of a
    filter-gradient kernel goes unvisited."""
    K, R, S, C = shape
    g = np.random.default_rng(seed)
    out = []
    for k0 in range(0, K, block):
        for c0 in range(0, C, block):
            kn, cn = min(block, K - k0), min(block, C - c0)
            for r in range(R):
                for s_ in range(S):
                    k = k0 + g.integers(0, kn, per_cell)
                    c = c0 + g.integers(0, cn, per_cell)
                    out.append(((k * R + r) * S + s_) * C + c)
    return np.unique(np.concatenate(out))


def guarded(shape, torch_dtype, guard: int = 128, fill: float = 123.0):
    """(buffer, view): an output tensor of this shape with `guard` elements of a known value on
    either side (the view stays 16-byte aligned)."""
    n = int(np.prod(shape))
    buf = torch.full((n + 2 * guard,), fill, dtype=torch_dtype, device="cuda")
    return buf, buf[guard:guard + n].view(shape)


def guards_intact(buf: torch.Tensor, guard: int = 128, fill: float = 123.0) -> bool:
    return bool(torch.all(buf[:guard] == fill)) and bool(torch.all(buf[-guard:] == fill))


def guarded_workspace(nbytes: int, guard: int = 256):
    """(buffer, view or None): a workspace of exactly nbytes with marked bytes on either side."""
    buf = torch.full((nbytes + 2 * guard,), 0xA5, dtype=torch.uint8, device="cuda")
    return buf, (buf[guard:guard + nbytes] if nbytes > 0 else None)


def workspace_guards_intact(buf: torch.Tensor, nbytes: int, guard: int = 256) -> bool:
    return bool(torch.all(buf[:guard] == 0xA5)) and bool(torch.all(buf[guard + nbytes:] == 0xA5))
