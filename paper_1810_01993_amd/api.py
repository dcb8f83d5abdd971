"""Thin Python binding of ``libdlconv.so`` (see ``include/dlconv.h``).

Argument marshalling only: every step of the computation runs in the HIP
kernels behind the C boundary.  torch is used to own device memory and to
name the current HIP stream.  There is no CPU fallback: if the library has
not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdlconv.so")

DL_F16, DL_BF16, DL_F32 = 0, 1, 2
PASS_FWD, PASS_BWD_DATA, PASS_BWD_FILTER = 0, 1, 2

EXPORTS = ("dl_conv_out_shape", "dl_conv_workspace_bytes", "dl_conv_describe", "conv2d_fwd", "conv2d_fwd_bias_relu", "conv2d_fwd_bias_add_relu", "conv2d_bwd_data",
           "conv2d_bwd_filter", "conv2d_transpose_fwd", "conv2d_transpose_bwd_data", "conv2d_transpose_bwd_filter",
           "dl_bias_relu_bwd_workspace_bytes", "bias_relu_bwd", "dl_larc_workspace_bytes", "larc_sgd_step", "dl_ce_workspace_bytes", "weighted_pixel_ce_fwd_bwd", "weighted_pixel_ce_fwd_bwd_static",
           "weighted_pixel_ce_map_fwd_bwd",
           "dl_logits_ce_workspace_bytes", "logits_ce_fused_fwd_bwd", "dl_status_string")


PROBE_EXPORTS = ("dl_probe_mfma", "dl_probe_stream")       # include/dlprobe.h: measurement aids
PROBE_SINK_FLOATS = 1024 * 256


class DlError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {_lib.dl_status_string(code).decode()} (status {code})")


class _Desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w",
                 "dil_h", "dil_w", "dtype", "dw_dtype")]


@dataclass(frozen=True)
class ConvDesc:
    """Mirror of ``dl_conv_desc``."""
    N: int
    H: int
    W: int
    C: int
    K: int
    R: int
    S: int
    stride_h: int = 1
    stride_w: int = 1
    pad_h: int = 0
    pad_w: int = 0
    dil_h: int = 1
    dil_w: int = 1
    dtype: int = DL_F16
    dw_dtype: int | None = None

    def c_struct(self) -> _Desc:
        dwt = self.dtype if self.dw_dtype is None else self.dw_dtype
        return _Desc(self.N, self.H, self.W, self.C, self.K, self.R, self.S, self.stride_h, self.stride_w,
                     self.pad_h, self.pad_w, self.dil_h, self.dil_w, self.dtype, dwt)


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1810_01993_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    dp = ctypes.POINTER(_Desc)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    lib.dl_conv_out_shape.argtypes = [dp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
    lib.dl_conv_workspace_bytes.argtypes = [dp, ctypes.c_int, ctypes.POINTER(sz)]
    lib.dl_conv_describe.argtypes = [dp, ctypes.c_int, ctypes.c_char_p, sz]
    for name in ("conv2d_fwd", "conv2d_bwd_data", "conv2d_bwd_filter", "conv2d_transpose_fwd",
                 "conv2d_transpose_bwd_data", "conv2d_transpose_bwd_filter"):
        getattr(lib, name).argtypes = [dp, vp, vp, vp, vp, sz, vp]
    lib.conv2d_fwd_bias_relu.argtypes = [dp, vp, vp, vp, ctypes.c_int32, vp, vp, sz, vp]
    lib.conv2d_fwd_bias_add_relu.argtypes = [dp, vp, vp, vp, vp, ctypes.c_int32, vp, vp, sz, vp]
    lib.dl_bias_relu_bwd_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.POINTER(sz)]
    lib.bias_relu_bwd.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, sz, vp]
    lib.dl_larc_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.POINTER(sz)]
    lib.larc_sgd_step.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                  ctypes.c_float, ctypes.c_float, ctypes.c_int32, vp, vp, sz, vp]
    lib.dl_ce_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.POINTER(sz)]
    for name in ("weighted_pixel_ce_fwd_bwd", "weighted_pixel_ce_map_fwd_bwd"):
        getattr(lib, name).argtypes = [vp, ctypes.c_int32, vp, vp, ctypes.c_float, ctypes.c_int64, vp, vp, vp, sz, vp]
    lib.weighted_pixel_ce_fwd_bwd_static.argtypes = [vp, ctypes.c_int32, vp, vp, ctypes.c_float, ctypes.c_int64, vp, vp, vp]
    lib.dl_logits_ce_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.POINTER(sz)]
    lib.logits_ce_fused_fwd_bwd.argtypes = [vp, vp, ctypes.c_int32, vp, vp, ctypes.c_float, ctypes.c_int64, ctypes.c_int32,
                                            vp, vp, vp, vp, vp, ctypes.c_int32, vp, sz, vp]
    lib.dl_probe_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.dl_probe_stream.argtypes = [ctypes.c_int32, vp, vp, vp, ctypes.c_int64, vp, vp]
    for name in EXPORTS + PROBE_EXPORTS:
        getattr(lib, name).restype = ctypes.c_int
    lib.dl_status_string.argtypes = [ctypes.c_int]
    lib.dl_status_string.restype = ctypes.c_char_p
    return lib


_lib = _load()


def _check(code: int, where: str):
    if code != 0:
        raise DlError(code, where)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return DL_F16
    if t.dtype == torch.bfloat16:
        return DL_BF16
    raise TypeError(f"fp16 or bf16 tensor required, got {t.dtype}")


def _dev_ptr(t: torch.Tensor | None) -> int | None:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("contiguous device tensor required")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def dl_conv_out_shape(desc: ConvDesc):
    P, Q = ctypes.c_int32(), ctypes.c_int32()
    _check(_lib.dl_conv_out_shape(ctypes.byref(desc.c_struct()), ctypes.byref(P), ctypes.byref(Q)), "dl_conv_out_shape")
    return P.value, Q.value


def dl_conv_workspace_bytes(desc: ConvDesc, which: int) -> int:
    n = ctypes.c_size_t()
    _check(_lib.dl_conv_workspace_bytes(ctypes.byref(desc.c_struct()), which, ctypes.byref(n)), "dl_conv_workspace_bytes")
    return n.value


def dl_conv_describe(desc: ConvDesc, which: int) -> str:
    """The kernels (with grids) that pass ``which`` of this convolution launches, in order."""
    buf = ctypes.create_string_buffer(2048)
    _check(_lib.dl_conv_describe(ctypes.byref(desc.c_struct()), which, buf, len(buf)), "dl_conv_describe")
    return buf.value.decode()


def dl_ce_workspace_bytes(n_pixels: int) -> int:
    n = ctypes.c_size_t()
    _check(_lib.dl_ce_workspace_bytes(n_pixels, ctypes.byref(n)), "dl_ce_workspace_bytes")
    return n.value


def _workspace(nbytes: int, device, workspace: torch.Tensor | None):
    if workspace is None:
        workspace = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)
    return workspace, workspace.numel() * workspace.element_size()


def _expect(t: torch.Tensor, shape, name: str):
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")


def conv2d_fwd(desc: ConvDesc, x: torch.Tensor, w: torch.Tensor, y: torch.Tensor | None = None,
               workspace: torch.Tensor | None = None) -> torch.Tensor:
    P, Q = dl_conv_out_shape(desc)
    _expect(x, (desc.N, desc.H, desc.W, desc.C), "x")
    _expect(w, (desc.K, desc.R, desc.S, desc.C), "w")
    if _dtype_code(x) != desc.dtype or w.dtype != x.dtype:
        raise TypeError("tensor dtype does not match the descriptor")
    if y is None:
        y = torch.empty((desc.N, P, Q, desc.K), dtype=x.dtype, device=x.device)
    _expect(y, (desc.N, P, Q, desc.K), "y")
    ws, nb = _workspace(dl_conv_workspace_bytes(desc, PASS_FWD), x.device, workspace)
    _check(_lib.conv2d_fwd(ctypes.byref(desc.c_struct()), _dev_ptr(x), _dev_ptr(w), _dev_ptr(y), _dev_ptr(ws), nb,
                           _stream()), "conv2d_fwd")
    return y


def conv2d_fwd_bias_relu(desc: ConvDesc, x: torch.Tensor, w: torch.Tensor, bias: torch.Tensor | None, relu: bool,
                         y: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """y = act(conv(x, w) + bias): bias float32[K] on the device or None; relu cuts negative results."""
    P, Q = dl_conv_out_shape(desc)
    _expect(x, (desc.N, desc.H, desc.W, desc.C), "x")
    _expect(w, (desc.K, desc.R, desc.S, desc.C), "w")
    if _dtype_code(x) != desc.dtype or w.dtype != x.dtype:
        raise TypeError("tensor dtype does not match the descriptor")
    if bias is not None and (bias.dtype != torch.float32 or tuple(bias.shape) != (desc.K,)):
        raise ValueError("bias must be float32[K]")
    if y is None:
        y = torch.empty((desc.N, P, Q, desc.K), dtype=x.dtype, device=x.device)
    _expect(y, (desc.N, P, Q, desc.K), "y")
    ws, nb = _workspace(dl_conv_workspace_bytes(desc, PASS_FWD), x.device, workspace)
    _check(_lib.conv2d_fwd_bias_relu(ctypes.byref(desc.c_struct()), _dev_ptr(x), _dev_ptr(w), _dev_ptr(bias),
                                     1 if relu else 0, _dev_ptr(y), _dev_ptr(ws), nb, _stream()),
           "conv2d_fwd_bias_relu")
    return y


def conv2d_fwd_bias_add_relu(desc: ConvDesc, x: torch.Tensor, w: torch.Tensor, bias: torch.Tensor | None,
                             residual: torch.Tensor | None, relu: bool, y: torch.Tensor | None = None,
                             workspace: torch.Tensor | None = None) -> torch.Tensor:
    """y = act(conv(x, w) + bias + residual): residual [N,P,Q,K] of x's dtype or None (a ResNet block's tail)."""
    P, Q = dl_conv_out_shape(desc)
    _expect(x, (desc.N, desc.H, desc.W, desc.C), "x")
    _expect(w, (desc.K, desc.R, desc.S, desc.C), "w")
    if _dtype_code(x) != desc.dtype or w.dtype != x.dtype:
        raise TypeError("tensor dtype does not match the descriptor")
    if bias is not None and (bias.dtype != torch.float32 or tuple(bias.shape) != (desc.K,)):
        raise ValueError("bias must be float32[K]")
    if residual is not None:
        _expect(residual, (desc.N, P, Q, desc.K), "residual")
        if residual.dtype != x.dtype:
            raise TypeError("the residual must have x's dtype")
    if y is None:
        y = torch.empty((desc.N, P, Q, desc.K), dtype=x.dtype, device=x.device)
    _expect(y, (desc.N, P, Q, desc.K), "y")
    ws, nb = _workspace(dl_conv_workspace_bytes(desc, PASS_FWD), x.device, workspace)
    _check(_lib.conv2d_fwd_bias_add_relu(ctypes.byref(desc.c_struct()), _dev_ptr(x), _dev_ptr(w), _dev_ptr(bias),
                                         _dev_ptr(residual), 1 if relu else 0, _dev_ptr(y), _dev_ptr(ws), nb, _stream()),
           "conv2d_fwd_bias_add_relu")
    return y


def conv2d_bwd_data(desc: ConvDesc, dy: torch.Tensor, w: torch.Tensor, dx: torch.Tensor | None = None,
                    workspace: torch.Tensor | None = None) -> torch.Tensor:
    P, Q = dl_conv_out_shape(desc)
    _expect(dy, (desc.N, P, Q, desc.K), "dy")
    _expect(w, (desc.K, desc.R, desc.S, desc.C), "w")
    if _dtype_code(dy) != desc.dtype or w.dtype != dy.dtype:
        raise TypeError("tensor dtype does not match the descriptor")
    if dx is None:
        dx = torch.empty((desc.N, desc.H, desc.W, desc.C), dtype=dy.dtype, device=dy.device)
    _expect(dx, (desc.N, desc.H, desc.W, desc.C), "dx")
    ws, nb = _workspace(dl_conv_workspace_bytes(desc, PASS_BWD_DATA), dy.device, workspace)
    _check(_lib.conv2d_bwd_data(ctypes.byref(desc.c_struct()), _dev_ptr(dy), _dev_ptr(w), _dev_ptr(dx), _dev_ptr(ws),
                                nb, _stream()), "conv2d_bwd_data")
    return dx


def conv2d_bwd_filter(desc: ConvDesc, x: torch.Tensor, dy: torch.Tensor, dw: torch.Tensor | None = None,
                      workspace: torch.Tensor | None = None) -> torch.Tensor:
    P, Q = dl_conv_out_shape(desc)
    _expect(x, (desc.N, desc.H, desc.W, desc.C), "x")
    _expect(dy, (desc.N, P, Q, desc.K), "dy")
    if _dtype_code(x) != desc.dtype or dy.dtype != x.dtype:
        raise TypeError("tensor dtype does not match the descriptor")
    dwt = desc.dtype if desc.dw_dtype is None else desc.dw_dtype
    if dw is None:
        dw = torch.empty((desc.K, desc.R, desc.S, desc.C), device=x.device,
                         dtype=torch.float32 if dwt == DL_F32 else x.dtype)
    _expect(dw, (desc.K, desc.R, desc.S, desc.C), "dw")
    ws, nb = _workspace(dl_conv_workspace_bytes(desc, PASS_BWD_FILTER), x.device, workspace)
    _check(_lib.conv2d_bwd_filter(ctypes.byref(desc.c_struct()), _dev_ptr(x), _dev_ptr(dy), _dev_ptr(dw),
                                  _dev_ptr(ws), nb, _stream()), "conv2d_bwd_filter")
    return dw


def conv2d_transpose_fwd(desc: ConvDesc, x: torch.Tensor, w: torch.Tensor, y: torch.Tensor | None = None,
                         workspace: torch.Tensor | None = None) -> torch.Tensor:
    """x: [N,P,Q,K] -> y: [N,H,W,C]; ``desc`` names the underlying convolution (see the header)."""
    P, Q = dl_conv_out_shape(desc)
    _expect(x, (desc.N, P, Q, desc.K), "x")
    _expect(w, (desc.K, desc.R, desc.S, desc.C), "w")
    if _dtype_code(x) != desc.dtype or w.dtype != x.dtype:
        raise TypeError("tensor dtype does not match the descriptor")
    if y is None:
        y = torch.empty((desc.N, desc.H, desc.W, desc.C), dtype=x.dtype, device=x.device)
    _expect(y, (desc.N, desc.H, desc.W, desc.C), "y")
    ws, nb = _workspace(dl_conv_workspace_bytes(desc, PASS_BWD_DATA), x.device, workspace)
    _check(_lib.conv2d_transpose_fwd(ctypes.byref(desc.c_struct()), _dev_ptr(x), _dev_ptr(w), _dev_ptr(y),
                                     _dev_ptr(ws), nb, _stream()), "conv2d_transpose_fwd")
    return y


def conv2d_transpose_bwd_data(desc: ConvDesc, dy: torch.Tensor, w: torch.Tensor, dx: torch.Tensor | None = None,
                              workspace: torch.Tensor | None = None) -> torch.Tensor:
    """dy: [N,H,W,C] -> dx: [N,P,Q,K]."""
    P, Q = dl_conv_out_shape(desc)
    _expect(dy, (desc.N, desc.H, desc.W, desc.C), "dy")
    _expect(w, (desc.K, desc.R, desc.S, desc.C), "w")
    if _dtype_code(dy) != desc.dtype or w.dtype != dy.dtype:
        raise TypeError("tensor dtype does not match the descriptor")
    if dx is None:
        dx = torch.empty((desc.N, P, Q, desc.K), dtype=dy.dtype, device=dy.device)
    _expect(dx, (desc.N, P, Q, desc.K), "dx")
    ws, nb = _workspace(dl_conv_workspace_bytes(desc, PASS_FWD), dy.device, workspace)
    _check(_lib.conv2d_transpose_bwd_data(ctypes.byref(desc.c_struct()), _dev_ptr(dy), _dev_ptr(w), _dev_ptr(dx),
                                          _dev_ptr(ws), nb, _stream()), "conv2d_transpose_bwd_data")
    return dx


def conv2d_transpose_bwd_filter(desc: ConvDesc, x: torch.Tensor, dy: torch.Tensor, dw: torch.Tensor | None = None,
                                workspace: torch.Tensor | None = None) -> torch.Tensor:
    """x: [N,P,Q,K], dy: [N,H,W,C] -> dw: [K,R,S,C]."""
    P, Q = dl_conv_out_shape(desc)
    _expect(x, (desc.N, P, Q, desc.K), "x")
    _expect(dy, (desc.N, desc.H, desc.W, desc.C), "dy")
    if _dtype_code(x) != desc.dtype or dy.dtype != x.dtype:
        raise TypeError("tensor dtype does not match the descriptor")
    dwt = desc.dtype if desc.dw_dtype is None else desc.dw_dtype
    if dw is None:
        dw = torch.empty((desc.K, desc.R, desc.S, desc.C), device=x.device,
                         dtype=torch.float32 if dwt == DL_F32 else x.dtype)
    _expect(dw, (desc.K, desc.R, desc.S, desc.C), "dw")
    ws, nb = _workspace(dl_conv_workspace_bytes(desc, PASS_BWD_FILTER), x.device, workspace)
    _check(_lib.conv2d_transpose_bwd_filter(ctypes.byref(desc.c_struct()), _dev_ptr(x), _dev_ptr(dy), _dev_ptr(dw),
                                            _dev_ptr(ws), nb, _stream()), "conv2d_transpose_bwd_filter")
    return dw


def bias_relu_bwd(dy: torch.Tensor, y: torch.Tensor | None, relu: bool, dz: torch.Tensor | None = None,
                  dbias: torch.Tensor | None = None, workspace: torch.Tensor | None = None):
    """dy, y: [..., K] fp16/bf16.  Returns (dz, dbias float32[K]); with relu False dz is dy itself."""
    K = dy.shape[-1]
    n = dy.numel() // K
    if relu:
        if y is None or y.shape != dy.shape or y.dtype != dy.dtype:
            raise ValueError("y must match dy")
        if dz is None:
            dz = torch.empty_like(dy)
    if dbias is None:
        dbias = torch.empty(K, dtype=torch.float32, device=dy.device)
    need = ctypes.c_size_t(0)
    _check(_lib.dl_bias_relu_bwd_workspace_bytes(n, K, ctypes.byref(need)), "dl_bias_relu_bwd_workspace_bytes")
    ws, nb = _workspace(int(need.value), dy.device, workspace)
    _check(_lib.bias_relu_bwd(_dev_ptr(dy), _dev_ptr(y) if relu else None, _dtype_code(dy), n, K, 1 if relu else 0,
                              _dev_ptr(dz) if relu else None, _dev_ptr(dbias), _dev_ptr(ws), nb, _stream()),
           "bias_relu_bwd")
    return (dz if relu else dy), dbias


class _LarcTensor(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("g", ctypes.c_void_p), ("v", ctypes.c_void_p), ("count", ctypes.c_int64)]


def larc_sgd_step(weights, grads, momenta, lr: float, trust: float, weight_decay: float = 0.0, momentum: float = 0.0,
                  eps: float = 0.0, clip: bool = True, rates: torch.Tensor | None = None,
                  workspace: torch.Tensor | None = None):
    """In-place LARC update of the fp32 tensors in ``weights`` (and ``momenta`` if momentum != 0) from
    ``grads`` (all fp16, all bf16 or all fp32).  Returns the per-tensor rates (float32[n], device)."""
    n = len(weights)
    if len(grads) != n or (momentum != 0.0 and (momenta is None or len(momenta) != n)):
        raise ValueError("one gradient (and momentum buffer) per weight tensor")
    gd = {torch.float16: DL_F16, torch.bfloat16: DL_BF16, torch.float32: DL_F32}[grads[0].dtype] if n else DL_F32
    table = (_LarcTensor * max(n, 1))()
    for i in range(n):
        w, g = weights[i], grads[i]
        if w.dtype != torch.float32 or g.dtype != grads[0].dtype or g.numel() != w.numel():
            raise ValueError("fp32 weights and gradients of one dtype and matching sizes required")
        v = momenta[i] if momentum != 0.0 else None
        if v is not None and (v.dtype != torch.float32 or v.numel() != w.numel()):
            raise ValueError("fp32 momentum buffer of the weight's size required")
        table[i] = _LarcTensor(_dev_ptr(w), _dev_ptr(g), _dev_ptr(v), w.numel())
    dev = weights[0].device if n else torch.device("cuda")
    if rates is None:
        rates = torch.empty(max(n, 1), dtype=torch.float32, device=dev)
    need = ctypes.c_size_t(0)
    _check(_lib.dl_larc_workspace_bytes(n, ctypes.byref(need)), "dl_larc_workspace_bytes")
    ws, nb = _workspace(int(need.value), dev, workspace)
    _check(_lib.larc_sgd_step(ctypes.cast(table, ctypes.c_void_p), n, gd, ctypes.c_float(lr), ctypes.c_float(trust),
                              ctypes.c_float(weight_decay), ctypes.c_float(momentum), ctypes.c_float(eps),
                              1 if clip else 0, _dev_ptr(rates), _dev_ptr(ws), nb, _stream()), "larc_sgd_step")
    return rates[:n]


def weighted_pixel_ce_fwd_bwd(logits: torch.Tensor, labels: torch.Tensor, class_weights: torch.Tensor,
                              scale: float, loss: torch.Tensor | None = None,
                              dlogits: torch.Tensor | None = None, workspace: torch.Tensor | None = None):
    """logits [..., 3] fp16/bf16, labels [...] uint8, class_weights float32[3]
    (device).  Returns (loss: float32[1] device tensor, dlogits)."""
    if logits.shape[-1] != 3:
        raise ValueError("3 classes expected in the last dimension")
    n = labels.numel()
    if logits.numel() != 3 * n or labels.dtype != torch.uint8:
        raise ValueError("labels must be uint8 with one entry per pixel")
    if class_weights.dtype != torch.float32 or class_weights.numel() != 3:
        raise ValueError("class_weights must be float32[3]")
    if loss is None:
        loss = torch.empty(1, dtype=torch.float32, device=logits.device)
    if dlogits is None:
        dlogits = torch.empty_like(logits)
    ws, nb = _workspace(dl_ce_workspace_bytes(n), logits.device, workspace)
    _check(_lib.weighted_pixel_ce_fwd_bwd(_dev_ptr(logits), _dtype_code(logits), _dev_ptr(labels),
                                          _dev_ptr(class_weights), ctypes.c_float(scale), n, _dev_ptr(loss),
                                          _dev_ptr(dlogits), _dev_ptr(ws), nb, _stream()),
           "weighted_pixel_ce_fwd_bwd")
    return loss, dlogits


CE_STATIC_MAX_PIXELS = 1 << 30


def weighted_pixel_ce_fwd_bwd_static(logits: torch.Tensor, labels: torch.Tensor, class_weights: torch.Tensor,
                                     scale: float, loss: torch.Tensor, dlogits: torch.Tensor):
    """``weighted_pixel_ce_fwd_bwd`` without a workspace and without any allocation, here or in the
    library: the caller brings every buffer (loss float32[1], dlogits like logits)."""
    n = labels.numel()
    if logits.shape[-1] != 3 or logits.numel() != 3 * n or labels.dtype != torch.uint8:
        raise ValueError("logits [..., 3] and uint8 labels with one entry per pixel expected")
    if class_weights.dtype != torch.float32 or class_weights.numel() != 3 or loss.dtype != torch.float32:
        raise ValueError("class_weights must be float32[3], loss float32[1]")
    if dlogits.dtype != logits.dtype or dlogits.numel() != logits.numel():
        raise ValueError("dlogits must match logits")
    _check(_lib.weighted_pixel_ce_fwd_bwd_static(_dev_ptr(logits), _dtype_code(logits), _dev_ptr(labels),
                                                 _dev_ptr(class_weights), ctypes.c_float(scale), n, _dev_ptr(loss),
                                                 _dev_ptr(dlogits), _stream()), "weighted_pixel_ce_fwd_bwd_static")
    return loss, dlogits


def weighted_pixel_ce_map_fwd_bwd(logits: torch.Tensor, labels: torch.Tensor, weight_map: torch.Tensor,
                                  scale: float, loss: torch.Tensor | None = None,
                                  dlogits: torch.Tensor | None = None, workspace: torch.Tensor | None = None):
    """The loss with a per-pixel weight map: weight_map float32 [...] (device), one
    weight per pixel.  Returns (loss: float32[1] device tensor, dlogits)."""
    if logits.shape[-1] != 3:
        raise ValueError("3 classes expected in the last dimension")
    n = labels.numel()
    if logits.numel() != 3 * n or labels.dtype != torch.uint8:
        raise ValueError("labels must be uint8 with one entry per pixel")
    if weight_map.dtype != torch.float32 or weight_map.numel() != n:
        raise ValueError("weight_map must be float32 with one entry per pixel")
    if loss is None:
        loss = torch.empty(1, dtype=torch.float32, device=logits.device)
    if dlogits is None:
        dlogits = torch.empty_like(logits)
    ws, nb = _workspace(dl_ce_workspace_bytes(n), logits.device, workspace)
    _check(_lib.weighted_pixel_ce_map_fwd_bwd(_dev_ptr(logits), _dtype_code(logits), _dev_ptr(labels),
                                              _dev_ptr(weight_map), ctypes.c_float(scale), n, _dev_ptr(loss),
                                              _dev_ptr(dlogits), _dev_ptr(ws), nb, _stream()),
           "weighted_pixel_ce_map_fwd_bwd")
    return loss, dlogits


def logits_ce_fused_fwd_bwd(x: torch.Tensor, w: torch.Tensor, labels: torch.Tensor, class_weights: torch.Tensor,
                            scale: float, want_logits: bool = True, want_dlogits: bool = True, dw_f32: bool = False,
                            dx: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                            logits: torch.Tensor | None = None, dlogits: torch.Tensor | None = None,
                            loss: torch.Tensor | None = None, dw: torch.Tensor | None = None):
    """The logits layer (1x1 convolution to the 3 classes) fused with the weighted loss: x [..., C]
    fp16/bf16, w [3, C] (or [3,1,1,C]) of the same type, labels [...] uint8, class_weights float32[3].
    Returns (logits or None, loss: float32[1] device tensor, dlogits or None, dx, dw)."""
    C = x.shape[-1]
    n = labels.numel()
    if x.numel() != n * C or w.numel() != 3 * C or w.dtype != x.dtype or labels.dtype != torch.uint8:
        raise ValueError("x [..., C], w [3, C] of one dtype and uint8 labels with one entry per pixel expected")
    if class_weights.dtype != torch.float32 or class_weights.numel() != 3:
        raise ValueError("class_weights must be float32[3]")
    dev = x.device
    if want_logits and logits is None:
        logits = torch.empty((n, 3), dtype=x.dtype, device=dev)
    if want_dlogits and dlogits is None:
        dlogits = torch.empty((n, 3), dtype=x.dtype, device=dev)
    for t in (logits if want_logits else None, dlogits if want_dlogits else None):
        if t is not None and (t.dtype != x.dtype or t.numel() != 3 * n):
            raise ValueError("logits / dlogits must be [n, 3] of x's dtype")
    if loss is None:
        loss = torch.empty(1, dtype=torch.float32, device=dev)
    if dx is None:
        dx = torch.empty_like(x)
    if dw is None:
        dw = torch.empty(w.shape, dtype=torch.float32 if dw_f32 else w.dtype, device=dev)
    if dx.dtype != x.dtype or dx.numel() != x.numel() or dw.numel() != w.numel() or \
            dw.dtype != (torch.float32 if dw_f32 else w.dtype) or loss.dtype != torch.float32:
        raise ValueError("dx must match x, dw must match w (or float32 with dw_f32), loss must be float32[1]")
    need = ctypes.c_size_t(0)
    _check(_lib.dl_logits_ce_workspace_bytes(n, C, ctypes.byref(need)), "dl_logits_ce_workspace_bytes")
    ws, nb = _workspace(int(need.value), dev, workspace)
    _check(_lib.logits_ce_fused_fwd_bwd(_dev_ptr(x), _dev_ptr(w), _dtype_code(x), _dev_ptr(labels), _dev_ptr(class_weights),
                                        ctypes.c_float(scale), n, C, _dev_ptr(logits) if want_logits else None,
                                        _dev_ptr(loss), _dev_ptr(dlogits) if want_dlogits else None, _dev_ptr(dx),
                                        _dev_ptr(dw), DL_F32 if dw_f32 else _dtype_code(x), _dev_ptr(ws), nb, _stream()),
           "logits_ce_fused_fwd_bwd")
    return (logits if want_logits else None), loss, (dlogits if want_dlogits else None), dx, dw


def logits_ce_workspace_bytes(n_pixels: int, C: int) -> int:
    need = ctypes.c_size_t(0)
    _check(_lib.dl_logits_ce_workspace_bytes(n_pixels, C, ctypes.byref(need)), "dl_logits_ce_workspace_bytes")
    return int(need.value)


def probe_mfma(shape: int, operands: int, iters: int, sink: torch.Tensor, clocks: torch.Tensor) -> float:
    """Enqueue the register-resident MFMA loop (include/dlprobe.h); returns the FLOPs it issues.
    sink: float32[PROBE_SINK_FLOATS], clocks: int64[2] (wall-clock ticks at 100 MHz, shader cycles)."""
    if sink.dtype != torch.float32 or sink.numel() < PROBE_SINK_FLOATS or clocks.dtype != torch.int64 or clocks.numel() < 2:
        raise ValueError("sink float32[PROBE_SINK_FLOATS] and clocks int64[2] required")
    flop = ctypes.c_double(0.0)
    _check(_lib.dl_probe_mfma(shape, operands, iters, _dev_ptr(sink), _dev_ptr(clocks), ctypes.byref(flop), _stream()),
           "dl_probe_mfma")
    return flop.value


def probe_stream(mode: int, src, aux, dst, nbytes: int, sink: torch.Tensor) -> None:
    """Enqueue one plain streaming kernel (include/dlprobe.h): 0 read, 1 copy, 2 write, 3 the loss's traffic mix."""
    _check(_lib.dl_probe_stream(mode, _dev_ptr(src), _dev_ptr(aux), _dev_ptr(dst), nbytes, _dev_ptr(sink), _stream()),
           "dl_probe_stream")


def desc_from_layer(layer, dtype: str, dw_f32: bool = False) -> ConvDesc:
    """ConvDesc for a ``layers.ConvLayer`` ('f16' | 'bf16')."""
    code = {"f16": DL_F16, "bf16": DL_BF16}[dtype]
    return ConvDesc(layer.N, layer.H, layer.W, layer.C, layer.K, layer.R, layer.S, layer.stride, layer.stride,
                    layer.pad, layer.pad, layer.dil, layer.dil, code, DL_F32 if dw_f32 else code)
