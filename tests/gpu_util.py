"""Helpers shared by the GPU parity tests: seeded inputs -> device tensors,
oracle evaluation (full or sampled), and the max|err|/max|ref| measure."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_1810_01993_amd import synth

TOL = {"f16": 2e-3, "bf16": 8e-3}          # max|err| / max|ref|
TORCH_DTYPE = {"f16": torch.float16, "bf16": torch.bfloat16}
FULL_ORACLE_FLOPS = 3e9                    # above this, spot-check sampled outputs instead


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
    """Flat indices: n_random uniform ones plus every element whose spatial
    position lies in the first / last two rows or columns (for a 4-d
    activation tensor [N, H, W, C]); for a filter [K, R, S, C] uniform only."""
    total = int(np.prod(shape))
    g = np.random.default_rng(seed)
    idx = [g.integers(0, total, size=min(n_random, total))]
    return np.unique(np.concatenate(idx))


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
