"""fp64 CPU oracle for the transposed ("deconvolutional") layers.

TEST INFRASTRUCTURE ONLY, like the rest of this package: imported by
``tests/`` (and nothing else); shares no code with the HIP library.

The paper's decoder up-samples with deconvolutional layers (caption of the
network schematic, Sec. "Segmentation Architecture").  A transposed
convolution is written here in its textbook "fractionally strided" form,
which shares nothing with the scatter loop of ``oracle_conv_bwd_data``:

  1. spread the input out: z[n, p*st_h, q*st_w, k] = x[n, p, q, k], zeros in
     between (st - 1 of them between neighbours),
  2. surround z with dil*(R-1) - pad zeros (crop instead if that is
     negative; extend at the far end up to the requested output size),
  3. correlate z, at unit stride and with the dilation kept, with the
     filter mirrored in both spatial axes, summing over the k channels:
       y[n,h,w,c] = sum_{r',s',k} z_pad[n, h + r'*dil_h, w + s'*dil_w, k]
                                  * w[k, R-1-r', S-1-s', c].

``ConvShape`` names the *underlying* convolution (the one whose adjoint this
is): x is [N,P,Q,K], w is [K,R,S,C], y is [N,H,W,C].  Because H and W are
given, the output size needs no separate "output padding" parameter: any
(H, W) whose forward output extent is (P, Q) is valid.

The sum over k of step 3 is a matrix product per tap (a library primitive);
taps are added in (r', s') order.
"""
from __future__ import annotations

import numpy as np

from . import ConvShape, conv_bwd_filter, conv_bwd_filter_at, conv_fwd, conv_fwd_at, out_shape


def _geometry(s: ConvShape):
    st_w = s.stride if s.stride_w is None else s.stride_w
    pad_w = s.pad if s.pad_w is None else s.pad_w
    dil_w = s.dil if s.dil_w is None else s.dil_w
    return (s.stride, st_w), (s.pad, pad_w), (s.dil, dil_w)


def _spread_and_pad(s: ConvShape, x: np.ndarray) -> np.ndarray:
    """Steps 1 and 2: z_pad of extent (H + dil_h*(R-1), W + dil_w*(S-1))."""
    (st_h, st_w), (pad_h, pad_w), (dil_h, dil_w) = _geometry(s)
    P, Q = out_shape(s)
    lead_h, lead_w = dil_h * (s.R - 1) - pad_h, dil_w * (s.S - 1) - pad_w
    ext_h, ext_w = s.H + dil_h * (s.R - 1), s.W + dil_w * (s.S - 1)
    zp = np.zeros((s.N, ext_h, ext_w, s.K), dtype=np.float64)
    for p in range(P):
        i = lead_h + p * st_h
        if not 0 <= i < ext_h:
            continue                       # cropped away (only when pad exceeds dil*(R-1))
        for q in range(Q):
            j = lead_w + q * st_w
            if 0 <= j < ext_w:
                zp[:, i, j, :] = x[:, p, q, :]
    return zp


def conv_transpose_fwd(s: ConvShape, x, w) -> np.ndarray:
    """y[N,H,W,C] from x[N,P,Q,K] and w[K,R,S,C] (see the module text)."""
    P, Q = out_shape(s)
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    if x.shape != (s.N, P, Q, s.K) or w.shape != (s.K, s.R, s.S, s.C):
        raise ValueError("shape mismatch")
    _, _, (dil_h, dil_w) = _geometry(s)
    zp = _spread_and_pad(s, x)
    y = np.zeros((s.N, s.H, s.W, s.C), dtype=np.float64)
    for r in range(s.R):                   # r, s_ count taps of the mirrored filter
        for s_ in range(s.S):
            window = zp[:, r * dil_h:r * dil_h + s.H, s_ * dil_w:s_ * dil_w + s.W, :]
            y += window @ w[:, s.R - 1 - r, s.S - 1 - s_, :]
    return y


def conv_transpose_fwd_at(s: ConvShape, x32, w32, flat_idx) -> np.ndarray:
    """y.ravel()[flat_idx] without forming y: the same three steps evaluated
    for single output elements (float32 storage, double arithmetic)."""
    (st_h, st_w), (pad_h, pad_w), (dil_h, dil_w) = _geometry(s)
    P, Q = out_shape(s)
    idx = np.asarray(flat_idx, dtype=np.int64)
    c = idx % s.C
    ww = (idx // s.C) % s.W
    h = (idx // (s.C * s.W)) % s.H
    n = idx // (s.C * s.W * s.H)
    lead_h, lead_w = dil_h * (s.R - 1) - pad_h, dil_w * (s.S - 1) - pad_w
    out = np.zeros(idx.shape, dtype=np.float64)
    for r in range(s.R):
        zi = h + r * dil_h - lead_h        # position in the spread-out image z
        ok_h = (zi >= 0) & (zi % st_h == 0) & (zi // st_h < P)
        for s_ in range(s.S):
            zj = ww + s_ * dil_w - lead_w
            ok = ok_h & (zj >= 0) & (zj % st_w == 0) & (zj // st_w < Q)
            if not ok.any():
                continue
            sel = np.nonzero(ok)[0]
            xs = x32[n[sel], zi[sel] // st_h, zj[sel] // st_w, :].astype(np.float64)
            ws = w32[:, s.R - 1 - r, s.S - 1 - s_, :].astype(np.float64)[:, c[sel]].T
            out[sel] += np.einsum("ik,ik->i", xs, ws)
    return out


def conv_transpose_bwd_data(s: ConvShape, dy, w) -> np.ndarray:
    """Gradient with respect to the transposed convolution's input.

    y is linear in x, and x[n,p,q,k] enters y[n, p*st-pad+r*dil, q*st-pad+s*dil, c]
    with coefficient w[k,r,s,c]; hence
      dx[n,p,q,k] = sum_{r,s,c} dy[n, p*st-pad+r*dil, q*st-pad+s*dil, c] * w[k,r,s,c],
    which is term by term the forward convolution of dy with w."""
    return conv_fwd(s, dy, w)


def conv_transpose_bwd_filter(s: ConvShape, x, dy) -> np.ndarray:
    """Gradient with respect to the filter: by the same linearity
      dw[k,r,s,c] = sum_{n,p,q} x[n,p,q,k] * dy[n, p*st-pad+r*dil, q*st-pad+s*dil, c],
    the filter-gradient sum of the underlying convolution with the roles of
    its input (here dy) and its output gradient (here x) as named there."""
    return conv_bwd_filter(s, dy, x)


def conv_transpose_bwd_data_at(s: ConvShape, dy32, w32, flat_idx) -> np.ndarray:
    """dx.ravel()[flat_idx] (float32 storage, double arithmetic); same sum as above."""
    return conv_fwd_at(s, dy32, w32, flat_idx)


def conv_transpose_bwd_filter_at(s: ConvShape, x32, dy32, flat_idx) -> np.ndarray:
    """dw.ravel()[flat_idx] (float32 storage, double arithmetic); same sum as above."""
    return conv_bwd_filter_at(s, dy32, x32, flat_idx)
