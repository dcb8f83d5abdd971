"""fp64 CPU oracle for the logits layer fused with the loss.

TEST INFRASTRUCTURE ONLY, like the rest of this package: imported by
``tests/`` (and ``bench.py``'s cpu_baseline leg); shares no code with the HIP
library.

The paper's stated next optimisation (Sec. "Single GPU performance": fuse
point-wise work into neighbouring layers so that tensors travel to and from
DRAM fewer times) applied to the end of the network: the 1x1 convolution that
maps the decoder's C channels to the 3 classes, the weighted loss of Sec.
"Weighted loss" and both gradients of that convolution, as one operation on
the pixels' feature vectors:

    z_i   = W x_i                                  (W: [3, C], x_i: [C])
    loss  = scale * sum_i cw[label_i] * (logsumexp(z_i) - z_i[label_i])
    dz_i  = scale * cw[label_i] * (softmax(z_i) - onehot(label_i))
    dx_i  = W^T dz_i
    dW    = sum_i dz_i x_i^T

Written out as exactly those five lines: a matrix product, the loss oracle of
this package, two more matrix products.  Nothing is rounded in between.
"""
from __future__ import annotations

import numpy as np

from . import weighted_ce


def logits_ce_fused(x, w, labels, class_weights, scale):
    """x: [n, C], w: [3, C], labels: [n] uint8, class_weights: [3].
    Returns (logits [n,3], loss, dlogits [n,3], dx [n,C], dw [3,C]) in float64."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    if x.ndim != 2 or w.ndim != 2 or w.shape[1] != x.shape[1]:
        raise ValueError("shape mismatch")
    z = x @ w.T
    loss, dz = weighted_ce(z, labels, class_weights, scale)
    dx = dz @ w
    dw = dz.T @ x
    return z, loss, dz, dx, dw
