"""fp64 CPU oracle for the forward convolution with the point-wise tail fused
into it: y = act(conv(x, w) + bias).

TEST INFRASTRUCTURE ONLY, like the rest of this package.

The paper counts bias layers among the point-wise operations around the
convolutions and names fusing point-wise operations, so that tensors are read
and written fewer times, as the optimisation being pursued (Sec. "Single GPU
Performance").  The definition is the convolution of ``oracle.c`` followed by
  y[n,p,q,k] <- y[n,p,q,k] + bias[k]            (bias: one value per output channel)
  y          <- max(y, 0)                        (if relu)
applied to the un-rounded fp64 sums.  With a residual input (the skip
connection of a ResNet block, which is added to the block's last convolution
before the activation) the middle line is
  y[n,p,q,k] <- y[n,p,q,k] + bias[k] + residual[n,p,q,k].
"""
from __future__ import annotations

import numpy as np

from . import ConvShape, conv_fwd, conv_fwd_at


def conv_fwd_bias_relu(s: ConvShape, x, w, bias=None, relu: bool = False) -> np.ndarray:
    y = conv_fwd(s, x, w)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64)
        if b.shape != (s.K,):
            raise ValueError("bias must have one entry per output channel")
        y = y + b[None, None, None, :]
    if relu:
        y = np.maximum(y, 0.0)
    return y


def conv_fwd_bias_add_relu(s: ConvShape, x, w, bias=None, residual=None, relu: bool = False) -> np.ndarray:
    """act(conv(x, w) + bias + residual); residual has the shape of the output."""
    y = conv_fwd_bias_relu(s, x, w, bias, False)
    if residual is not None:
        r = np.asarray(residual, dtype=np.float64)
        if r.shape != y.shape:
            raise ValueError("the residual must have the shape of the output")
        y = y + r
    if relu:
        y = np.maximum(y, 0.0)
    return y


def conv_fwd_bias_add_relu_at(s: ConvShape, x32, w32, bias, residual32, relu: bool, flat_idx) -> np.ndarray:
    """Single output elements (float32 storage, double arithmetic)."""
    idx = np.asarray(flat_idx, dtype=np.int64)
    y = conv_fwd_bias_relu_at(s, x32, w32, bias, False, idx)
    if residual32 is not None:
        y = y + np.asarray(residual32).ravel()[idx].astype(np.float64)
    if relu:
        y = np.maximum(y, 0.0)
    return y


def conv_fwd_bias_relu_at(s: ConvShape, x32, w32, bias, relu: bool, flat_idx) -> np.ndarray:
    """Single output elements (float32 storage, double arithmetic)."""
    idx = np.asarray(flat_idx, dtype=np.int64)
    y = conv_fwd_at(s, x32, w32, idx)
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[idx % s.K]
    if relu:
        y = np.maximum(y, 0.0)
    return y


def bias_relu_bwd(dy, y, relu: bool = True):
    """Backward of the point-wise tail y = act(s + bias[k]) given dy = dL/dy and the forward
    output y ([..., K] each):
      dz[i,k]  = dy[i,k] if (not relu or y[i,k] > 0) else 0      (= dL/ds, what the convolution's
                                                                   gradient kernels take)
      dbias[k] = sum_i dz[i,k]
    (the derivative of max(., 0) at 0 is taken as 0, as y = 0 carries no sign)."""
    dy = np.asarray(dy, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    if dy.shape != y.shape:
        raise ValueError("shape mismatch")
    dz = np.where(y > 0.0, dy, 0.0) if relu else dy.copy()
    K = dy.shape[-1]
    dbias = np.zeros(K, dtype=np.float64)
    flat = dz.reshape(-1, K)
    for i in range(flat.shape[0]):          # pixel by pixel, in index order
        dbias += flat[i]
    return dz, dbias
