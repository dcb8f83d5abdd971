"""fp64 CPU oracle for the LARC weight update (layer-wise adaptive rate control).

TEST INFRASTRUCTURE ONLY, like the rest of this package.

The paper (Sec. "LARC") states the principle, not the formula: every layer gets
its own learning rate, and the magnitude of the update is defined relative to
the norm of the layer's weights.  The formula taken here is the published one
of layer-wise adaptive rate scaling with LARC's clipping, applied to SGD with
momentum and weight decay; per layer (tensor) with weights w, gradient g:

    local = trust * ||w|| / (||g|| + wd * ||w|| + eps)     (lr itself if ||w|| or ||g|| is 0)
    rate  = min(local, lr) if clip else local * lr          ("clip" and "scale" modes)
    u     = g + wd * w
    v    <- momentum * v + rate * u                         (v: momentum buffer; momentum 0: v = rate * u)
    w    <- w - v

With wd = 0, momentum = 0 and no clipping in effect, ||w_new - w|| = trust * ||w||
(scale mode: times lr): the update's size is a fixed fraction of the weights' norm.
"""
from __future__ import annotations

import numpy as np


def larc_sgd_step(ws, gs, vs, lr, trust, weight_decay=0.0, momentum=0.0, eps=0.0, clip=True):
    """ws, gs, vs: lists of arrays (one per layer; vs entries may be None when momentum == 0).
    Returns (new_ws, new_vs, rates)."""
    new_w, new_v, rates = [], [], []
    for w, g, v in zip(ws, gs, vs):
        w = np.asarray(w, dtype=np.float64)
        g = np.asarray(g, dtype=np.float64)
        wn = float(np.sqrt(np.sum(w * w)))
        gn = float(np.sqrt(np.sum(g * g)))
        if wn > 0.0 and gn > 0.0:
            local = trust * wn / (gn + weight_decay * wn + eps)
        else:
            local = lr if clip else 1.0
        rate = min(local, lr) if clip else local * lr
        u = g + weight_decay * w
        vv = rate * u if v is None else momentum * np.asarray(v, dtype=np.float64) + rate * u
        new_w.append(w - vv)
        new_v.append(vv)
        rates.append(rate)
    return new_w, new_v, rates
