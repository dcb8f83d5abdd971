"""ctypes front end of the fp64 CPU oracle (``oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  Nothing in the product
package imports this module and this module imports nothing from it.

Every function takes and returns plain numpy arrays (NHWC activations, KRSC
filters).  The arithmetic lives entirely in ``oracle.c``; this file only
marshals arguments.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile ``oracle.c`` with gcc + OpenMP into ``liboracle.so``."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w",
                 "pad_h", "pad_w", "dil_h", "dil_w")]


@dataclass(frozen=True)
class ConvShape:
    """Convolution geometry in the paper's (N, H, W, C, K, R, S) naming."""
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
    stride_w: int | None = None
    pad_w: int | None = None
    dil_w: int | None = None

    def _c(self) -> _Desc:
        sw = self.stride if self.stride_w is None else self.stride_w
        pw = self.pad if self.pad_w is None else self.pad_w
        dw = self.dil if self.dil_w is None else self.dil_w
        return _Desc(self.N, self.H, self.W, self.C, self.K, self.R, self.S,
                     self.stride, sw, self.pad, pw, self.dil, dw)


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        fp = ctypes.POINTER(ctypes.c_float)
        ip = ctypes.POINTER(ctypes.c_int64)
        sp = ctypes.POINTER(_Desc)
        lib.oracle_conv_out_shape.argtypes = [sp, ctypes.POINTER(ctypes.c_int32),
                                              ctypes.POINTER(ctypes.c_int32)]
        lib.oracle_conv_out_shape.restype = ctypes.c_int
        for name in ("oracle_conv_fwd", "oracle_conv_bwd_data", "oracle_conv_bwd_filter"):
            f = getattr(lib, name)
            f.argtypes = [sp, dp, dp, dp]
            f.restype = None
        for name in ("oracle_conv_fwd_at", "oracle_conv_bwd_data_at", "oracle_conv_bwd_filter_at"):
            f = getattr(lib, name)
            f.argtypes = [sp, fp, fp, ip, ctypes.c_int64, dp]
            f.restype = None
        lib.oracle_weighted_ce.argtypes = [dp, ctypes.POINTER(ctypes.c_uint8), dp, ctypes.c_double,
                                           ctypes.c_int64, ctypes.c_int32, dp, dp]
        lib.oracle_weighted_ce.restype = None
        lib.oracle_weighted_ce_map.argtypes = [dp, ctypes.POINTER(ctypes.c_uint8), dp, ctypes.c_double,
                                               ctypes.c_int64, ctypes.c_int32, dp, dp]
        lib.oracle_weighted_ce_map.restype = None
        _lib = lib
    return _lib


def _d(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _f(a, shape):
    if a.dtype != np.float32 or not a.flags.c_contiguous:
        raise ValueError("float32 C-contiguous array required")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _fp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def out_shape(s: ConvShape):
    P, Q = ctypes.c_int32(), ctypes.c_int32()
    rc = _load().oracle_conv_out_shape(ctypes.byref(s._c()), ctypes.byref(P), ctypes.byref(Q))
    if rc != 0:
        raise ValueError(f"empty output for {s}")
    return P.value, Q.value


def conv_fwd(s: ConvShape, x, w):
    P, Q = out_shape(s)
    x = _d(x, (s.N, s.H, s.W, s.C))
    w = _d(w, (s.K, s.R, s.S, s.C))
    y = np.empty((s.N, P, Q, s.K), dtype=np.float64)
    _load().oracle_conv_fwd(ctypes.byref(s._c()), _dp(x), _dp(w), _dp(y))
    return y


def conv_bwd_data(s: ConvShape, dy, w):
    P, Q = out_shape(s)
    dy = _d(dy, (s.N, P, Q, s.K))
    w = _d(w, (s.K, s.R, s.S, s.C))
    dx = np.empty((s.N, s.H, s.W, s.C), dtype=np.float64)
    _load().oracle_conv_bwd_data(ctypes.byref(s._c()), _dp(dy), _dp(w), _dp(dx))
    return dx


def conv_bwd_filter(s: ConvShape, x, dy):
    P, Q = out_shape(s)
    x = _d(x, (s.N, s.H, s.W, s.C))
    dy = _d(dy, (s.N, P, Q, s.K))
    dw = np.empty((s.K, s.R, s.S, s.C), dtype=np.float64)
    _load().oracle_conv_bwd_filter(ctypes.byref(s._c()), _dp(x), _dp(dy), _dp(dw))
    return dw


def _at(fn_name, s, a, a_shape, b, b_shape, idx):
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.shape, dtype=np.float64)
    getattr(_load(), fn_name)(ctypes.byref(s._c()), _fp(_f(a, a_shape)), _fp(_f(b, b_shape)),
                              idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                              ctypes.c_int64(idx.size), _dp(out))
    return out


def conv_fwd_at(s: ConvShape, x32, w32, flat_idx):
    """y.ravel()[flat_idx] from float32-stored inputs, double arithmetic."""
    return _at("oracle_conv_fwd_at", s, x32, (s.N, s.H, s.W, s.C), w32, (s.K, s.R, s.S, s.C), flat_idx)


def conv_bwd_data_at(s: ConvShape, dy32, w32, flat_idx):
    P, Q = out_shape(s)
    return _at("oracle_conv_bwd_data_at", s, dy32, (s.N, P, Q, s.K), w32, (s.K, s.R, s.S, s.C), flat_idx)


def conv_bwd_filter_at(s: ConvShape, x32, dy32, flat_idx):
    P, Q = out_shape(s)
    return _at("oracle_conv_bwd_filter_at", s, x32, (s.N, s.H, s.W, s.C), dy32, (s.N, P, Q, s.K), flat_idx)


def weighted_ce(z, labels, class_weights, scale, want_grad=True):
    """Returns (loss, dz).  z: [..., n_classes]; labels: [...] uint8."""
    z = _d(z)
    n_classes = z.shape[-1]
    labels = np.ascontiguousarray(labels, dtype=np.uint8)
    n = labels.size
    if z.size != n * n_classes:
        raise ValueError("z and labels disagree on the pixel count")
    if n and int(labels.max()) >= n_classes:
        raise ValueError("label out of range")
    cw = _d(class_weights, (n_classes,))
    loss = ctypes.c_double(0.0)
    dz = np.empty_like(z) if want_grad else None
    _load().oracle_weighted_ce(_dp(z), labels.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), _dp(cw),
                               ctypes.c_double(scale), ctypes.c_int64(n), ctypes.c_int32(n_classes),
                               ctypes.byref(loss), _dp(dz) if want_grad else None)
    return loss.value, dz


def weighted_ce_map(z, labels, weight_map, scale, want_grad=True):
    """The loss with a per-pixel weight map (one weight per pixel, any values).
    Returns (loss, dz).  z: [..., n_classes]; labels, weight_map: [...]."""
    z = _d(z)
    n_classes = z.shape[-1]
    labels = np.ascontiguousarray(labels, dtype=np.uint8)
    n = labels.size
    if z.size != n * n_classes:
        raise ValueError("z and labels disagree on the pixel count")
    if n and int(labels.max()) >= n_classes:
        raise ValueError("label out of range")
    wm = _d(weight_map)
    if wm.size != n:
        raise ValueError("weight map and labels disagree on the pixel count")
    loss = ctypes.c_double(0.0)
    dz = np.empty_like(z) if want_grad else None
    _load().oracle_weighted_ce_map(_dp(z), labels.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), _dp(wm),
                                   ctypes.c_double(scale), ctypes.c_int64(n), ctypes.c_int32(n_classes),
                                   ctypes.byref(loss), _dp(dz) if want_grad else None)
    return loss.value, dz
