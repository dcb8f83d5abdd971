"""Seeded synthetic inputs that stand in for the CAM5 climate fields and the
TECA / flood-fill label masks (paper, Sec. "Climate Dataset and Ground Truth
Labels"), which are not available offline.

This module holds none of the method's arithmetic (no convolution, no loss):
it only draws random tensors with the shapes, value distributions and class
balance of the workload and rounds them once to the storage type.  Both the
CPU oracle's tests and the GPU path's tests / benchmark take their inputs
from here, so the two sides always see the same bits.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 18100199300

# Class ids: 0 background, 1 atmospheric river, 2 tropical cyclone.  Nominal
# pixel frequencies from Sec. "Weighted loss" (98.2 %, 1.7 %, "<0.1 %" taken
# as 0.1 %), and the inverse-square-root-of-frequency class weights.
CLASS_FREQ = (0.982, 0.017, 0.001)
CLASS_WEIGHTS = tuple(1.0 / np.sqrt(f) for f in CLASS_FREQ)


def rng(seed: int) -> np.random.Generator:
    """Counter-based Philox stream keyed by ``seed``."""
    return np.random.Generator(np.random.Philox(key=int(seed)))


def seed_for(config: int, tensor: int) -> int:
    return BASE_SEED + 1000 * int(config) + int(tensor)


# ---- storage rounding -----------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(a: np.ndarray, dtype: str):
    """Round ``a`` once to ``dtype`` ('f16' or 'bf16').

    Returns ``(values, bits)``: the rounded values as float32 (exact) and the
    16-bit storage pattern as uint16, same shape.
    """
    a = np.asarray(a)
    if dtype == "f16":
        h = a.astype(np.float16)
        return h.astype(np.float32), h.view(np.uint16)
    if dtype == "bf16":
        bits = f32_to_bf16_bits(a.astype(np.float32))
        return bf16_bits_to_f32(bits), bits
    raise ValueError(f"dtype must be 'f16' or 'bf16', got {dtype!r}")


def bits_to_f32(bits: np.ndarray, dtype: str) -> np.ndarray:
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(bits)
    raise ValueError(dtype)


# ---- tensors --------------------------------------------------------------
def normal(seed: int, shape, sigma: float = 1.0) -> np.ndarray:
    """N(0, sigma^2), float32."""
    a = rng(seed).standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        a *= np.float32(sigma)
    return a


def half_normal(seed: int, shape) -> np.ndarray:
    """|N(0,1)|: non-negative, like the output of a ReLU."""
    a = rng(seed).standard_normal(size=shape, dtype=np.float32)
    np.abs(a, out=a)
    return a


def he_filter(seed: int, K: int, R: int, S: int, C: int) -> np.ndarray:
    """KRSC filter ~ N(0, 2 / (R*S*C))."""
    return normal(seed, (K, R, S, C), sigma=float(np.sqrt(2.0 / (R * S * C))))


def smooth_fields(seed: int, N: int, H: int, W: int, C: int, sigma_px: float = 8.0) -> np.ndarray:
    """Smooth, per-channel normalised fields shaped like climate variables on a
    lat-lon grid: white noise blurred with a Gaussian of ``sigma_px`` pixels
    (periodic in W = longitude, reflecting in H = latitude, truncated at
    4 sigma), then each channel shifted and scaled to zero mean, unit variance
    over the batch.  NHWC float32."""
    from scipy.ndimage import gaussian_filter1d

    a = rng(seed).standard_normal(size=(N, H, W, C), dtype=np.float32)
    a = gaussian_filter1d(a, sigma_px, axis=2, mode="wrap", truncate=4.0)
    a = gaussian_filter1d(a, sigma_px, axis=1, mode="reflect", truncate=4.0)
    mean = a.mean(axis=(0, 1, 2), keepdims=True, dtype=np.float64)
    std = a.std(axis=(0, 1, 2), keepdims=True, dtype=np.float64)
    return ((a - mean) / std).astype(np.float32)


def _paint_ellipse(mask, cy, cx, a, b, theta):
    H, W = mask.shape
    ext = int(np.ceil(max(a, b))) + 1
    y0, y1 = max(0, int(cy) - ext), min(H, int(cy) + ext + 1)
    x0, x1 = max(0, int(cx) - ext), min(W, int(cx) + ext + 1)
    if y0 >= y1 or x0 >= x1:
        return
    yy, xx = np.mgrid[y0:y1, x0:x1]
    dy, dx = yy - cy, xx - cx
    ct, st = np.cos(theta), np.sin(theta)
    u = (dx * ct + dy * st) / a
    v = (-dx * st + dy * ct) / b
    mask[y0:y1, x0:x1] |= (u * u + v * v) <= 1.0


def _fill_to_fraction(g, H, W, target_px, axes, blocked=None):
    """Paint random ellipses into a fresh mask until exactly ``target_px``
    unblocked pixels are painted: ellipses never larger than 80 % of what is
    still missing, and single pixels for the last few."""
    mask = np.zeros((H, W), dtype=bool)
    free = np.ones((H, W), dtype=bool) if blocked is None else ~blocked

    for _ in range(100000):
        missing = target_px - int((mask & free).sum())
        if missing <= 0:
            break
        if missing < 12:
            cand = np.flatnonzero((~mask & free).ravel())
            mask.ravel()[g.choice(cand, size=missing, replace=False)] = True
            break
        (a_lo, a_hi), (b_lo, b_hi) = axes
        a, b = g.uniform(a_lo, a_hi), g.uniform(b_lo, b_hi)
        area = np.pi * a * b
        if area > 0.8 * missing:                 # late patches shrink to what is left
            f = np.sqrt(0.8 * missing / area)
            a, b = max(a * f, 0.6), max(b * f, 0.6)
        trial = mask.copy()
        _paint_ellipse(trial, g.uniform(0, H), g.uniform(0, W), a, b, g.uniform(0, np.pi))
        if int((trial & free).sum()) <= target_px:
            mask = trial
    return mask


def ellipse_labels(seed: int, N: int, H: int, W: int, freq=CLASS_FREQ, tol: float = 5e-4) -> np.ndarray:
    """uint8 label mask [N, H, W]: background everywhere, elongated randomly
    oriented ellipses for atmospheric rivers (class 1), small near-circular
    blobs for tropical cyclones (class 2, painted last).  Each image's class
    fractions are within ``tol`` (absolute) of ``freq``; this is asserted."""
    g = rng(seed)
    out = np.zeros((N, H, W), dtype=np.uint8)
    npx = H * W
    scale = np.sqrt(npx / (768.0 * 1152.0))     # ellipse sizes follow the grid size
    for n in range(N):
        tc = _fill_to_fraction(g, H, W, round(freq[2] * npx),
                               ((6 * scale, 12 * scale), (5 * scale, 10 * scale)))
        ar = _fill_to_fraction(g, H, W, round(freq[1] * npx),
                               ((60 * scale, 200 * scale), (8 * scale, 25 * scale)), blocked=tc)
        out[n][ar] = 1
        out[n][tc] = 2
        got = np.bincount(out[n].ravel(), minlength=3) / npx
        assert abs(got[1] - freq[1]) <= tol and abs(got[2] - freq[2]) <= tol, got
    return out
