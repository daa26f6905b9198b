"""Thin ctypes binding over libpipe_hip.so: argument marshalling only.

Function names and argument order follow include/pipe.h.  Tensors are torch CUDA
(ROCm) tensors used as device memory; every step of the method runs inside the
library's HIP kernels.  There is no CPU fallback: importing this module without
the built library raises, and so does any call that returns an error code.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpipe_hip.so")

PIPE_ACT_NONE = 0
PIPE_ACT_GELU = 1
PIPE_ACT_SILU_GATED = 2
PIPE_ACT_RELU = 3


_ROUNDING_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p)


class PipeError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = _lib.pipe_strerror(code).decode()
        dev = _lib.pipe_last_device_error().decode()
        super().__init__("%s failed: %s (%d)%s" % (where, msg, code, (" [" + dev + "]") if dev and code == -4 else ""))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libpipe_hip.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(or python paper_2311_15806_amd/build.py); there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp, ci, cf = C.c_void_p, C.c_int, C.c_float
    pi = C.POINTER(C.c_int)
    lib.pipe_expand.argtypes = [vp, ci, ci, ci, ci, cf, ci, vp, C.POINTER(vp)]
    lib.pipe_expand_unstructured.argtypes = [vp, ci, ci, ci, ci, cf, ci, vp, C.POINTER(vp)]
    lib.pipe_expand_conv2d.argtypes = [vp, ci, ci, ci, ci, ci, ci, cf, ci, vp, C.POINTER(vp)]
    lib.pipe_expand_with_operator.argtypes = [vp, ci, ci, ci, ci, cf, ci, _ROUNDING_FN, vp, vp, vp, vp, vp, C.POINTER(vp)]
    lib.pipe_expansion_free.argtypes = [vp]
    lib.pipe_expansion_info.argtypes = [vp, pi, pi, pi, pi, pi, C.POINTER(cf), C.POINTER(C.c_int64)]
    lib.pipe_expansion_order.argtypes = [vp, ci, pi, vp, vp, vp]
    lib.pipe_forward.argtypes = [vp, vp, ci, cf, pi, ci, vp, ci, vp, vp]
    lib.pipe_forward_noalloc.argtypes = [vp, vp, ci, cf, pi, ci, vp, ci, vp, vp]
    lib.pipe_forward_acc.argtypes = [vp, vp, ci, cf, vp, vp, vp, vp]
    lib.pipe_forward_asymmetric.argtypes = [vp, vp, ci, pi, ci, vp, vp, vp]
    lib.pipe_forward_acc_asymmetric.argtypes = [vp, vp, ci, vp, vp, vp, vp, vp]
    lib.pipe_forward_conv2d_asymmetric.argtypes = [vp, vp] + [ci] * 9 + [pi, ci, vp, vp, vp]
    lib.pipe_forward_conv2d.argtypes = [vp, vp] + [ci] * 9 + [cf, pi, ci, vp, ci, vp, vp]
    lib.pipe_forward_conv2d_acc.argtypes = [vp, vp] + [ci] * 9 + [cf, vp, vp, vp, vp]
    lib.pipe_forward_depthwise2d.argtypes = [vp, vp] + [ci] * 9 + [cf, pi, ci, vp, ci, vp, vp]
    lib.pipe_mlp_forward.argtypes = [vp, vp, ci, vp, ci, cf, pi, ci, vp, vp, vp, vp, vp]
    lib.pipe_mlp_forward_asymmetric.argtypes = [vp, vp, ci, vp, ci, pi, ci, vp, vp, vp, vp, vp]
    lib.pipe_mlp_forward_given_scales.argtypes = [vp, vp, ci, vp, ci, cf, C.POINTER(C.c_float), pi, ci, vp, vp, vp, vp, vp]
    lib.pipe_chain_forward.argtypes = [vp, ci, vp, ci, cf, pi, ci, vp, vp, vp]
    lib.pipe_chain_forward_conv.argtypes = [vp, ci, vp, ci, ci, ci, cf, pi, ci, vp, vp, vp]
    lib.pipe_chain_forward_asymmetric.argtypes = [vp, ci, vp, ci, pi, ci, vp, vp, vp]
    lib.pipe_chain_forward_conv_asymmetric.argtypes = [vp, ci, vp, ci, ci, ci, pi, ci, vp, vp, vp]
    lib.pipe_prepare.argtypes = [vp, pi, ci, ci, vp]
    lib.pipe_prepare_mlp.argtypes = [vp, vp, ci, pi, ci, ci, vp]
    lib.pipe_prepare_chain.argtypes = [vp, ci, ci, ci, ci, pi, ci, vp]
    lib.pipe_set_kernel.argtypes = [ci]
    lib.pipe_fold_batchnorm.argtypes = [vp] * 6 + [cf, ci, ci, vp, vp, vp]
    lib.pipe_spectral_norm.argtypes = [vp, ci, ci, ci, C.POINTER(cf), vp]
    lib.pipe_expansion_reconstruct.argtypes = [vp, ci, vp, vp]
    lib.pipe_expansion_error_bound.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.pipe_error_bound_U.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_double), ci, C.POINTER(C.c_double)]
    pd = C.POINTER(C.c_double)
    lib.pipe_expansion_order_norms.argtypes = [vp, ci, pd, vp]
    lib.pipe_error_bound_U_ens.argtypes = [pd, pd, ci, ci, pi, ci, pd]
    lib.pipe_first_predictor_size.argtypes = [pd, pd, ci, ci, C.c_double, C.c_double, C.POINTER(ci)]
    lib.pipe_set_activation_bits.argtypes = [ci]
    lib.pipe_set_stream_split.argtypes = [ci]
    lib.pipe_set_decode_fusion.argtypes = [ci]
    lib.pipe_set_decode_resident.argtypes = [ci]
    lib.pipe_set_resident_spin_limit.argtypes = [ci]
    lib.pipe_resident_status.argtypes = [vp, pi]
    lib.pipe_resident_trace.argtypes = [vp]
    lib.pipe_set_token_tile.argtypes = [ci]
    lib.pipe_mfma_probe.argtypes = [ci, ci, C.POINTER(C.c_double), vp]
    lib.pipe_hbm_probe.argtypes = [C.c_int64, C.POINTER(C.c_double), vp]
    lib.pipe_timing_enable.argtypes = [ci]
    lib.pipe_timing_read.argtypes = [C.POINTER(C.c_double), pi]
    lib.pipe_strerror.argtypes = [ci]
    lib.pipe_strerror.restype = C.c_char_p
    lib.pipe_last_device_error.restype = C.c_char_p
    for f in ("pipe_expand", "pipe_expand_unstructured", "pipe_expansion_free", "pipe_expansion_info", "pipe_expansion_order",
              "pipe_forward", "pipe_forward_acc", "pipe_forward_asymmetric", "pipe_forward_acc_asymmetric", "pipe_forward_conv2d_asymmetric", "pipe_forward_conv2d", "pipe_mlp_forward",
              "pipe_set_kernel", "pipe_set_stream_split", "pipe_set_decode_fusion", "pipe_set_token_tile", "pipe_timing_enable", "pipe_timing_read", "pipe_mfma_probe", "pipe_hbm_probe"):
        getattr(lib, f).restype = ci
    return lib


_lib = _load()


def _check(code: int, where: str):
    if code != 0:
        raise PipeError(code, where)


def _ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected dtype %s, got %s" % (dtype, t.dtype))
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _split(split: Optional[Sequence[int]]):
    if split is None:
        return None, 0
    arr = (C.c_int * len(split))(*[int(s) for s in split])
    return arr, len(split)


class Expansion:
    """Owner of a pipe_expansion handle."""

    def __init__(self, handle: int):
        self._h = C.c_void_p(handle)
        o, i, b, k, g = (C.c_int() for _ in range(5))
        gm, pb = C.c_float(), C.c_int64()
        _check(_lib.pipe_expansion_info(self._h, o, i, b, k, g, gm, pb), "pipe_expansion_info")
        self.out_features, self.in_features, self.bits, self.K, self.group = o.value, i.value, b.value, k.value, g.value
        self.gamma, self.packed_bytes = gm.value, pb.value

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("expansion already freed")
        return self._h

    def free(self):
        if self._h is not None:
            _check(_lib.pipe_expansion_free(self._h), "pipe_expansion_free")
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    def order(self, k: int, codes: bool = True):
        """(group_ids int32 [n], scales fp32 [n*group], codes int8 [n*group, in]) as numpy."""
        return pipe_expansion_order(self, k, codes)

    def macs_per_token(self) -> int:
        """Integer multiply-accumulates per token: in * (stored rows over all orders)."""
        rows = 0
        for k in range(1, self.K + 1):
            n = C.c_int()
            _check(_lib.pipe_expansion_order(self.handle, k, n, None, None, None), "pipe_expansion_order")
            rows += n.value * self.group
        return rows * self.in_features


def pipe_expand(W: torch.Tensor, bits: int, K: int, gamma: float, group: int) -> Expansion:
    if W.dim() != 2:
        raise ValueError("W must be [out, in]")
    h = C.c_void_p()
    _check(_lib.pipe_expand(_ptr(W, torch.float32), W.shape[0], W.shape[1], int(bits), int(K),
                            float(gamma), int(group), _stream(), C.byref(h)), "pipe_expand")
    return Expansion(h.value)


def pipe_expand_conv2d(W: torch.Tensor, Cin: int, kh: int, kw: int, bits: int, K: int, gamma: float, group: int) -> Expansion:
    """W [out, Cin*kh*kw] (rows flattened [Cin, kh, kw]) expanded for the implicit-GEMM convolution."""
    if W.dim() != 2 or W.shape[1] != Cin * kh * kw:
        raise ValueError("W must be [out, Cin*kh*kw]")
    h = C.c_void_p()
    _check(_lib.pipe_expand_conv2d(_ptr(W, torch.float32), W.shape[0], int(Cin), int(kh), int(kw), int(bits), int(K),
                                   float(gamma), int(group), _stream(), C.byref(h)), "pipe_expand_conv2d")
    return Expansion(h.value)


def pipe_expand_unstructured(W: torch.Tensor, bits: int, K: int, gamma: float, group: int) -> Expansion:
    if W.dim() != 2:
        raise ValueError("W must be [out, in]")
    h = C.c_void_p()
    _check(_lib.pipe_expand_unstructured(_ptr(W, torch.float32), W.shape[0], W.shape[1], int(bits), int(K),
                                         float(gamma), int(group), _stream(), C.byref(h)), "pipe_expand_unstructured")
    return Expansion(h.value)


def pipe_expand_with_operator(W: torch.Tensor, bits: int, K: int, gamma: float, group: int, operator) -> Expansion:
    """operator(k, rows [R, in] fp32, scales [R] fp32, q_max) -> codes [R, in] (any integer-valued
    tensor on W's device), called once per order with views of the builder's scratch."""
    if W.dim() != 2:
        raise ValueError("W must be [out, in]")
    out, inn = W.shape
    rows_t = torch.empty((out, inn), dtype=torch.float32, device=W.device)
    scales_t = torch.empty((out,), dtype=torch.float32, device=W.device)
    codes_t = torch.empty((out, inn), dtype=torch.int8, device=W.device)
    failure = []

    def hook(_user, k, rows, in_, q_max, _stream_ptr):
        try:
            q = operator(k, rows_t[:rows], scales_t[:rows], q_max)
            if tuple(q.shape) != (rows, in_):
                raise ValueError("the operator returns one code per element")
            codes_t[:rows].copy_(q.clamp(-127, 127).to(torch.int8))
            return 0
        except BaseException as exc:   # never unwind through the C frames
            failure.append(exc)
            return 1

    cb = _ROUNDING_FN(hook)
    h = C.c_void_p()
    rc = _lib.pipe_expand_with_operator(_ptr(W, torch.float32), out, inn, int(bits), int(K), float(gamma), int(group), cb,
                                        None, _ptr(rows_t), _ptr(scales_t), _ptr(codes_t), _stream(), C.byref(h))
    if failure:
        raise failure[0]
    _check(rc, "pipe_expand_with_operator")
    return Expansion(h.value)


def pipe_expansion_order(e: Expansion, k: int, codes: bool = True):
    n = C.c_int()
    _check(_lib.pipe_expansion_order(e.handle, k, n, None, None, None), "pipe_expansion_order")
    rows = n.value * e.group
    gids = np.empty(n.value, dtype=np.int32)
    scales = np.empty(rows, dtype=np.float32)
    cds = np.empty((rows, e.in_features), dtype=np.int8) if codes else None
    _check(_lib.pipe_expansion_order(e.handle, k, n, gids.ctypes.data, scales.ctypes.data,
                                     cds.ctypes.data if codes else None), "pipe_expansion_order")
    return gids, scales, cds


def pipe_forward(e: Expansion, x: torch.Tensor, s_x: float = 0.0, split=None, bias=None,
                 reduce_members: bool = True, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    T = x.shape[0]
    if x.dim() != 2 or x.shape[1] != e.in_features:
        raise ValueError("x must be [T, in]")
    M = 1 if split is None else len(split)
    shape = (T, e.out_features) if reduce_members else (M, T, e.out_features)
    y = out if out is not None else torch.empty(shape, dtype=torch.float32, device=x.device)
    if tuple(y.shape) != shape:
        raise ValueError("output has the wrong shape")
    arr, m = _split(split)
    _check(_lib.pipe_forward(e.handle, _ptr(x, torch.float32), T, float(s_x), arr, m,
                             _ptr(bias, torch.float32), 1 if reduce_members else 0,
                             _ptr(y, torch.float32), _stream()), "pipe_forward")
    return y


def pipe_forward_noalloc(e: Expansion, x: torch.Tensor, out: torch.Tensor, s_x: float = 0.0, split=None, bias=None,
                         reduce_members: bool = True) -> torch.Tensor:
    """pipe_forward through the entry point that allocates nothing; the caller brings the output."""
    T = x.shape[0]
    if x.dim() != 2 or x.shape[1] != e.in_features:
        raise ValueError("x must be [T, in]")
    M = 1 if split is None else len(split)
    shape = (T, e.out_features) if reduce_members else (M, T, e.out_features)
    if tuple(out.shape) != shape:
        raise ValueError("output has the wrong shape")
    arr, m = _split(split)
    _check(_lib.pipe_forward_noalloc(e.handle, _ptr(x, torch.float32), T, float(s_x), arr, m,
                                     _ptr(bias, torch.float32), 1 if reduce_members else 0,
                                     _ptr(out, torch.float32), _stream()), "pipe_forward_noalloc")
    return out


def pipe_forward_acc(e: Expansion, x: torch.Tensor, s_x: float = 0.0):
    """Returns (acc int32 [K,T,out], Qx int8 [T,in], s_x fp32 [1]) device tensors."""
    T = x.shape[0]
    acc = torch.empty((e.K, T, e.out_features), dtype=torch.int32, device=x.device)
    qx = torch.empty((T, e.in_features), dtype=torch.int8, device=x.device)
    sx = torch.zeros(1, dtype=torch.float32, device=x.device)
    _check(_lib.pipe_forward_acc(e.handle, _ptr(x, torch.float32), T, float(s_x), _ptr(acc), _ptr(qx),
                                 _ptr(sx), _stream()), "pipe_forward_acc")
    return acc, qx, sx


def pipe_forward_asymmetric(e: Expansion, x: torch.Tensor, split=None, bias=None,
                            out: Optional[torch.Tensor] = None) -> torch.Tensor:
    T = x.shape[0]
    if x.dim() != 2 or x.shape[1] != e.in_features:
        raise ValueError("x must be [T, in]")
    y = out if out is not None else torch.empty((T, e.out_features), dtype=torch.float32, device=x.device)
    arr, m = _split(split)
    _check(_lib.pipe_forward_asymmetric(e.handle, _ptr(x, torch.float32), T, arr, m, _ptr(bias, torch.float32),
                                        _ptr(y, torch.float32), _stream()), "pipe_forward_asymmetric")
    return y


def pipe_forward_conv2d_asymmetric(e: Expansion, x: torch.Tensor, kh: int, kw: int, stride: int, pad: int,
                                   split=None, bias=None, nhwc: bool = False) -> torch.Tensor:
    if x.dim() != 4:
        raise ValueError("x must be [N,C,H,W] (or [N,H,W,C] with nhwc=True)")
    if nhwc:
        N, H, W, Cc = x.shape
    else:
        N, Cc, H, W = x.shape
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    y = torch.empty((N * Ho * Wo, e.out_features), dtype=torch.float32, device=x.device)
    arr, m = _split(split)
    _check(_lib.pipe_forward_conv2d_asymmetric(e.handle, _ptr(x, torch.float32), N, Cc, H, W, kh, kw, stride, pad,
                                               1 if nhwc else 0, arr, m, _ptr(bias, torch.float32), _ptr(y),
                                               _stream()), "pipe_forward_conv2d_asymmetric")
    return y


def pipe_forward_acc_asymmetric(e: Expansion, x: torch.Tensor):
    """(acc int32 [K,T,out], Q(x) uint8 [T,in], scale, zero point) of the asymmetric layer."""
    T = x.shape[0]
    acc = torch.empty((e.K, T, e.out_features), dtype=torch.int32, device=x.device)
    qx = torch.empty((T, e.in_features), dtype=torch.uint8, device=x.device)
    sx = torch.zeros(1, dtype=torch.float32, device=x.device)
    z = torch.zeros(1, dtype=torch.int32, device=x.device)
    _check(_lib.pipe_forward_acc_asymmetric(e.handle, _ptr(x, torch.float32), T, _ptr(acc), _ptr(qx), _ptr(sx), _ptr(z),
                                            _stream()), "pipe_forward_acc_asymmetric")
    return acc, qx, float(sx.item()), int(z.item())


def pipe_forward_conv2d(e: Expansion, x: torch.Tensor, kh: int, kw: int, stride: int, pad: int,
                        nhwc: bool = False, s_x: float = 0.0, split=None, bias=None,
                        reduce_members: bool = True, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if x.dim() != 4:
        raise ValueError("x must be 4-D")
    if nhwc:
        N, H, W, Cc = x.shape
    else:
        N, Cc, H, W = x.shape
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    T = N * Ho * Wo
    M = 1 if split is None else len(split)
    shape = (T, e.out_features) if reduce_members else (M, T, e.out_features)
    y = out if out is not None else torch.empty(shape, dtype=torch.float32, device=x.device)
    if tuple(y.shape) != shape:
        raise ValueError("output has the wrong shape")
    arr, m = _split(split)
    _check(_lib.pipe_forward_conv2d(e.handle, _ptr(x, torch.float32), N, Cc, H, W, kh, kw, stride, pad,
                                    1 if nhwc else 0, float(s_x), arr, m, _ptr(bias, torch.float32),
                                    1 if reduce_members else 0, _ptr(y, torch.float32), _stream()), "pipe_forward_conv2d")
    return y


def pipe_forward_conv2d_acc(e: Expansion, x: torch.Tensor, kh: int, kw: int, stride: int, pad: int,
                            nhwc: bool = False, s_x: float = 0.0):
    """(acc int32 [K, N*Ho*Wo, out], Q(x) int8 shaped like x, s_x fp32 [1]) of the convolution layer."""
    if x.dim() != 4:
        raise ValueError("x must be 4-D")
    if nhwc:
        N, H, W, Cc = x.shape
    else:
        N, Cc, H, W = x.shape
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    acc = torch.empty((e.K, N * Ho * Wo, e.out_features), dtype=torch.int32, device=x.device)
    qx = torch.empty(tuple(x.shape), dtype=torch.int8, device=x.device)
    sx = torch.zeros(1, dtype=torch.float32, device=x.device)
    _check(_lib.pipe_forward_conv2d_acc(e.handle, _ptr(x, torch.float32), N, Cc, H, W, kh, kw, stride, pad,
                                        1 if nhwc else 0, float(s_x), _ptr(acc), _ptr(qx), _ptr(sx), _stream()),
           "pipe_forward_conv2d_acc")
    return acc, qx, sx


def pipe_forward_depthwise2d(e: Expansion, x: torch.Tensor, kh: int, kw: int, stride: int, pad: int,
                             nhwc: bool = False, s_x: float = 0.0, split=None, bias=None,
                             reduce_members: bool = True) -> torch.Tensor:
    if x.dim() != 4:
        raise ValueError("x must be [N,C,H,W] or [N,H,W,C]")
    if nhwc:
        N, H, W, Cc = x.shape
    else:
        N, Cc, H, W = x.shape
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    M = 1 if split is None else len(split)
    T = N * Ho * Wo
    y = torch.empty((T, Cc) if reduce_members else (M, T, Cc), dtype=torch.float32, device=x.device)
    arr, m = _split(split)
    _check(_lib.pipe_forward_depthwise2d(e.handle, _ptr(x, torch.float32), N, Cc, H, W, kh, kw, stride, pad,
                                         1 if nhwc else 0, float(s_x), arr, m, _ptr(bias, torch.float32),
                                         1 if reduce_members else 0, _ptr(y), _stream()), "pipe_forward_depthwise2d")
    return y


def pipe_mlp_forward(l1: Expansion, l2: Expansion, act: int, x: torch.Tensor, s_x: float = 0.0,
                     split=None, bias1=None, bias2=None, return_hidden: bool = False,
                     out: Optional[torch.Tensor] = None):
    T = x.shape[0]
    M = 1 if split is None else len(split)
    y = out if out is not None else torch.empty((T, l2.out_features), dtype=torch.float32, device=x.device)
    h = torch.empty((M, T, l2.in_features), dtype=torch.float32, device=x.device) if return_hidden else None
    arr, m = _split(split)
    _check(_lib.pipe_mlp_forward(l1.handle, l2.handle, int(act), _ptr(x, torch.float32), T, float(s_x),
                                 arr, m, _ptr(bias1, torch.float32), _ptr(bias2, torch.float32),
                                 _ptr(h), _ptr(y), _stream()), "pipe_mlp_forward")
    return (y, h) if return_hidden else y


def pipe_mlp_forward_given_scales(l1: Expansion, l2: Expansion, act: int, x: torch.Tensor, s_x: float, s_h, split=None,
                                  bias1=None, bias2=None, return_hidden: bool = False, out: Optional[torch.Tensor] = None):
    """pipe_mlp_forward with given (static) scales: s_x for the input, s_h[m] for member m's hidden activation."""
    T = x.shape[0]
    M = 1 if split is None else len(split)
    y = out if out is not None else torch.empty((T, l2.out_features), dtype=torch.float32, device=x.device)
    h = torch.empty((M, T, l2.in_features), dtype=torch.float32, device=x.device) if return_hidden else None
    arr, m = _split(split)
    sh = (C.c_float * len(s_h))(*[float(v) for v in s_h])
    _check(_lib.pipe_mlp_forward_given_scales(l1.handle, l2.handle, int(act), _ptr(x, torch.float32), T, float(s_x), sh, arr, m,
                                              _ptr(bias1, torch.float32), _ptr(bias2, torch.float32), _ptr(h), _ptr(y),
                                              _stream()), "pipe_mlp_forward_given_scales")
    return (y, h) if return_hidden else y


def pipe_mlp_forward_asymmetric(l1: Expansion, l2: Expansion, act: int, x: torch.Tensor, split=None, bias1=None,
                                bias2=None, return_hidden: bool = False, out: Optional[torch.Tensor] = None):
    """pipe_mlp_forward with asymmetric activation codes in front of both layers."""
    T = x.shape[0]
    M = 1 if split is None else len(split)
    y = out if out is not None else torch.empty((T, l2.out_features), dtype=torch.float32, device=x.device)
    h = torch.empty((M, T, l2.in_features), dtype=torch.float32, device=x.device) if return_hidden else None
    arr, m = _split(split)
    _check(_lib.pipe_mlp_forward_asymmetric(l1.handle, l2.handle, int(act), _ptr(x, torch.float32), T, arr, m,
                                            _ptr(bias1, torch.float32), _ptr(bias2, torch.float32), _ptr(h), _ptr(y),
                                            _stream()), "pipe_mlp_forward_asymmetric")
    return (y, h) if return_hidden else y


class _ChainLayer(C.Structure):
    _fields_ = [("e", C.c_void_p), ("bias_dev", C.c_void_p), ("act", C.c_int), ("skip_from", C.c_int),
                ("skip_pre_act", C.c_int), ("kh", C.c_int), ("kw", C.c_int), ("stride", C.c_int), ("pad", C.c_int),
                ("s_in", C.c_void_p)]


def _chain_layers(layers):
    """(Expansion, bias or None, act, skip_from, skip_pre_act[, kh, kw, stride, pad[, s_in]]) -> C array;
    s_in: None or the given scales (one per member) of the tensors entering the layer."""
    arr = (_ChainLayer * len(layers))()
    keep = []
    for l, ly in enumerate(layers):
        e, bias, act, skip_from, pre = ly[:5]
        kh, kw, stride, pad = ly[5:9] if len(ly) >= 9 else (0, 0, 1, 0)
        s_in = ly[9] if len(ly) >= 10 else None
        s_ptr = None
        if s_in is not None:
            buf = (C.c_float * len(s_in))(*[float(v) for v in s_in])
            keep.append(buf)
            s_ptr = C.cast(buf, C.c_void_p)
        arr[l] = _ChainLayer(e.handle, _ptr(bias, torch.float32), int(act), int(skip_from), 1 if pre else 0,
                             int(kh), int(kw), int(stride), int(pad), s_ptr)
    arr._keep = keep   # the host arrays live as long as the layer array
    return arr


def pipe_chain_forward(layers, x: torch.Tensor, s_x: float = 0.0, split=None, return_acts: bool = False,
                       out: Optional[torch.Tensor] = None):
    """layers: sequence of (Expansion, bias or None, act, skip_from, skip_pre_act)."""
    T = x.shape[0]
    L = len(layers)
    M = 1 if split is None else len(split)
    arr_l = _chain_layers(layers)
    y = out if out is not None else torch.empty((T, layers[-1][0].out_features), dtype=torch.float32, device=x.device)
    acts, acts_arr = None, None
    if return_acts and L > 1:
        acts = [torch.empty((M, T, layers[l][0].out_features), dtype=torch.float32, device=x.device)
                for l in range(L - 1)]
        acts_arr = (C.c_void_p * (L - 1))(*[_ptr(a) for a in acts])
    arr, m = _split(split)
    _check(_lib.pipe_chain_forward(arr_l, L, _ptr(x, torch.float32), T, float(s_x), arr, m, acts_arr, _ptr(y),
                                   _stream()), "pipe_chain_forward")
    return (y, acts) if return_acts else y


def pipe_chain_forward_asymmetric(layers, x: torch.Tensor, split=None, return_acts: bool = False,
                                  out: Optional[torch.Tensor] = None):
    """pipe_chain_forward with asymmetric activation codes in front of every layer (fully-connected layers)."""
    T = x.shape[0]
    L = len(layers)
    M = 1 if split is None else len(split)
    arr_l = _chain_layers(layers)
    y = out if out is not None else torch.empty((T, layers[-1][0].out_features), dtype=torch.float32, device=x.device)
    acts, acts_arr = None, None
    if return_acts and L > 1:
        acts = [torch.empty((M, T, layers[l][0].out_features), dtype=torch.float32, device=x.device)
                for l in range(L - 1)]
        acts_arr = (C.c_void_p * (L - 1))(*[_ptr(a) for a in acts])
    arr, m = _split(split)
    _check(_lib.pipe_chain_forward_asymmetric(arr_l, L, _ptr(x, torch.float32), T, arr, m, acts_arr, _ptr(y),
                                              _stream()), "pipe_chain_forward_asymmetric")
    return (y, acts) if return_acts else y


def pipe_chain_forward_conv(layers, x: torch.Tensor, s_x: float = 0.0, split=None, return_acts: bool = False,
                            out: Optional[torch.Tensor] = None):
    """x [N, H, W, C] channels-last; layers: (Expansion, bias or None, act, skip_from, skip_pre_act, kh, kw,
    stride, pad), kh = kw = 0 for a layer applied per grid position.  Returns y [N, H_L, W_L, out] (and the
    tensors leaving layers 0..L-2 as [M, N, H_l, W_l, out_l])."""
    N, H, W, _ = x.shape
    L = len(layers)
    M = 1 if split is None else len(split)
    arr_l = _chain_layers(layers)
    grids = []
    h, w = H, W
    for l in range(L):
        if arr_l[l].kh > 0 and arr_l[l].kw > 0 and arr_l[l].stride > 0:
            h = (h + 2 * arr_l[l].pad - arr_l[l].kh) // arr_l[l].stride + 1
            w = (w + 2 * arr_l[l].pad - arr_l[l].kw) // arr_l[l].stride + 1
        grids.append((max(h, 0), max(w, 0)))
    shape_y = (N,) + grids[-1] + (layers[-1][0].out_features,)
    y = out if out is not None else torch.empty(shape_y, dtype=torch.float32, device=x.device)
    acts, acts_arr = None, None
    if return_acts and L > 1:
        acts = [torch.empty((M, N) + grids[l] + (layers[l][0].out_features,), dtype=torch.float32, device=x.device)
                for l in range(L - 1)]
        acts_arr = (C.c_void_p * (L - 1))(*[_ptr(a) for a in acts])
    arr, m = _split(split)
    _check(_lib.pipe_chain_forward_conv(arr_l, L, _ptr(x, torch.float32), N, H, W, float(s_x), arr, m, acts_arr,
                                        _ptr(y), _stream()), "pipe_chain_forward_conv")
    return (y, acts) if return_acts else y


def pipe_chain_forward_conv_asymmetric(layers, x: torch.Tensor, split=None, return_acts: bool = False,
                                       out: Optional[torch.Tensor] = None):
    """pipe_chain_forward_conv with asymmetric activation codes in front of every layer; x [N, H, W, C] channels-last."""
    N, H, W, _ = x.shape
    L = len(layers)
    M = 1 if split is None else len(split)
    arr_l = _chain_layers(layers)
    grids = []
    h, w = H, W
    for l in range(L):
        if arr_l[l].kh > 0 and arr_l[l].kw > 0 and arr_l[l].stride > 0:
            h = (h + 2 * arr_l[l].pad - arr_l[l].kh) // arr_l[l].stride + 1
            w = (w + 2 * arr_l[l].pad - arr_l[l].kw) // arr_l[l].stride + 1
        grids.append((max(h, 0), max(w, 0)))
    y = out if out is not None else torch.empty((N,) + grids[-1] + (layers[-1][0].out_features,), dtype=torch.float32,
                                               device=x.device)
    acts, acts_arr = None, None
    if return_acts and L > 1:
        acts = [torch.empty((M, N) + grids[l] + (layers[l][0].out_features,), dtype=torch.float32, device=x.device)
                for l in range(L - 1)]
        acts_arr = (C.c_void_p * (L - 1))(*[_ptr(a) for a in acts])
    arr, m = _split(split)
    _check(_lib.pipe_chain_forward_conv_asymmetric(arr_l, L, _ptr(x, torch.float32), N, H, W, arr, m, acts_arr, _ptr(y),
                                                   _stream()), "pipe_chain_forward_conv_asymmetric")
    return (y, acts) if return_acts else y


def pipe_prepare(e: Expansion, T_max: int, split=None) -> None:
    """Everything pipe_forward(e, x[T <= T_max], split=split) on the current stream would do on first use."""
    arr, m = _split(split)
    _check(_lib.pipe_prepare(e.handle, arr, m, int(T_max), _stream()), "pipe_prepare")


def pipe_prepare_mlp(l1: Expansion, l2: Expansion, act: int, T_max: int, split=None) -> None:
    arr, m = _split(split)
    _check(_lib.pipe_prepare_mlp(l1.handle, l2.handle, int(act), arr, m, int(T_max), _stream()), "pipe_prepare_mlp")


def pipe_prepare_chain(layers, N: int, H: int = 1, W: int = 1, split=None) -> None:
    """layers as for pipe_chain_forward / pipe_chain_forward_conv; a chain over T tokens is the grid T x 1 x 1."""
    arr_l = _chain_layers(layers)
    arr, m = _split(split)
    _check(_lib.pipe_prepare_chain(arr_l, len(layers), int(N), int(H), int(W), arr, m, _stream()), "pipe_prepare_chain")


def pipe_spectral_norm(W: torch.Tensor, iters: int = 50) -> float:
    s = C.c_float()
    _check(_lib.pipe_spectral_norm(_ptr(W, torch.float32), W.shape[0], W.shape[1], int(iters), C.byref(s), _stream()),
           "pipe_spectral_norm")
    return s.value


def pipe_expansion_reconstruct(e: Expansion, upto: Optional[int] = None) -> torch.Tensor:
    W = torch.empty((e.out_features, e.in_features), dtype=torch.float32, device="cuda")
    _check(_lib.pipe_expansion_reconstruct(e.handle, int(e.K if upto is None else upto), _ptr(W), _stream()),
           "pipe_expansion_reconstruct")
    return W


def pipe_expansion_error_bound(e: Expansion):
    """(u_lemma, u_stored): element-wise bounds on |W - sum_k R^k| from the stored scales."""
    a, b = C.c_double(), C.c_double()
    _check(_lib.pipe_expansion_error_bound(e.handle, C.byref(a), C.byref(b)), "pipe_expansion_error_bound")
    return a.value, b.value


def pipe_error_bound_U(s, u) -> float:
    L = len(s)
    sa, ua, U = (C.c_double * L)(*[float(v) for v in s]), (C.c_double * L)(*[float(v) for v in u]), C.c_double()
    _check(_lib.pipe_error_bound_U(sa, ua, L, C.byref(U)), "pipe_error_bound_U")
    return U.value


def pipe_expansion_order_norms(e: Expansion, iters: int = 50):
    out = (C.c_double * e.K)()
    _check(_lib.pipe_expansion_order_norms(e.handle, int(iters), out, _stream()), "pipe_expansion_order_norms")
    return list(out)


def _norm_table(norms, lam):
    L, K = len(norms), len(norms[0])
    flat = (C.c_double * (L * K))(*[float(v) for row in norms for v in row])
    lam_flat = None
    if lam is not None:
        lam_flat = (C.c_double * ((L - 1) * K))(*[float(v) for row in lam for v in row])
    return L, K, flat, lam_flat


def pipe_error_bound_U_ens(norms, split=None, lam=None) -> float:
    L, K, flat, lam_flat = _norm_table(norms, lam)
    arr, m = _split(split)
    U = C.c_double()
    _check(_lib.pipe_error_bound_U_ens(flat, lam_flat, L, K, arr, m, C.byref(U)), "pipe_error_bound_U_ens")
    return U.value


def pipe_first_predictor_size(norms, logit_norm: float, ratio: float, lam=None) -> int:
    L, K, flat, lam_flat = _norm_table(norms, lam)
    K1 = C.c_int()
    _check(_lib.pipe_first_predictor_size(flat, lam_flat, L, K, float(logit_norm), float(ratio), C.byref(K1)),
           "pipe_first_predictor_size")
    return K1.value


def pipe_fold_batchnorm(W: torch.Tensor, bias, gamma, beta, mean, var, eps: float):
    """(W', b') of the layer followed by a batch normalization, as one affine layer."""
    Wf = torch.empty_like(W)
    bf = torch.empty(W.shape[0], dtype=torch.float32, device=W.device)
    _check(_lib.pipe_fold_batchnorm(_ptr(W, torch.float32), _ptr(bias, torch.float32), _ptr(gamma, torch.float32),
                                    _ptr(beta, torch.float32), _ptr(mean, torch.float32), _ptr(var, torch.float32),
                                    float(eps), W.shape[0], W.shape[1], _ptr(Wf), _ptr(bf), _stream()),
           "pipe_fold_batchnorm")
    return Wf, bf


def pipe_set_kernel(which: int) -> None:
    _check(_lib.pipe_set_kernel(int(which)), "pipe_set_kernel")


def pipe_set_activation_bits(bits: int) -> None:
    _check(_lib.pipe_set_activation_bits(int(bits)), "pipe_set_activation_bits")


def pipe_set_token_tile(tokens: int) -> None:
    _check(_lib.pipe_set_token_tile(int(tokens)), "pipe_set_token_tile")


def pipe_set_stream_split(workgroups_per_bin: int) -> None:
    _check(_lib.pipe_set_stream_split(int(workgroups_per_bin)), "pipe_set_stream_split")


def pipe_set_decode_fusion(on: bool) -> None:
    _check(_lib.pipe_set_decode_fusion(1 if on else 0), "pipe_set_decode_fusion")


def pipe_set_decode_resident(on) -> None:
    """0 / False: per-layer launches; 1: automatic (default); 2 / True: the resident launch whenever it applies."""
    _check(_lib.pipe_set_decode_resident(2 if on is True else int(on)), "pipe_set_decode_resident")


def pipe_set_resident_spin_limit(polls: int) -> None:
    _check(_lib.pipe_set_resident_spin_limit(int(polls)), "pipe_set_resident_spin_limit")


def pipe_resident_status() -> int:
    """0, or non-zero if a resident launch on the current stream ran into its wait limit (synchronizes)."""
    v = C.c_int()
    _check(_lib.pipe_resident_status(_stream(), C.byref(v)), "pipe_resident_status")
    return v.value


def pipe_resident_trace(buf: Optional[torch.Tensor]) -> None:
    """buf: int64 device tensor [compute units, layers, 8] that later resident launches fill with phase timestamps; None = off."""
    _check(_lib.pipe_resident_trace(None if buf is None else _ptr(buf, torch.int64)), "pipe_resident_trace")


def pipe_timing_enable(on: bool) -> None:
    _check(_lib.pipe_timing_enable(1 if on else 0), "pipe_timing_enable")


def pipe_timing_read():
    """(total milliseconds, launches) of the contraction kernels bracketed since the last read."""
    ms, n = C.c_double(), C.c_int()
    _check(_lib.pipe_timing_read(C.byref(ms), C.byref(n)), "pipe_timing_read")
    return ms.value, n.value


def pipe_mfma_probe(iters: int = 20000, operands: int = 0) -> float:
    """int8 TOP/s an MFMA-only kernel sustains on this chip (diagnostic for reports);
    operands: 0 constant, 1 ternary codes x random int8, 2 random int8 x random int8."""
    t = C.c_double()
    _check(_lib.pipe_mfma_probe(int(iters), int(operands), C.byref(t), _stream()), "pipe_mfma_probe")
    return t.value


def pipe_hbm_probe(nbytes: int = 1 << 31) -> float:
    """GB/s of a plain streaming read with the weight-streaming kernel's access pattern."""
    t = C.c_double()
    _check(_lib.pipe_hbm_probe(int(nbytes), C.byref(t), _stream()), "pipe_hbm_probe")
    return t.value
