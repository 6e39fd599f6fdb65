"""ctypes binding of libnsk (argument marshalling only; every computation runs in the HIP kernels).

The raw entry points carry the names of ``include/nsk.h`` (``nsk_conv2d_fwd`` ...).  The
tensor-level helpers below take torch CUDA tensors that are ALREADY in the physical layout the
descriptor names (NHWC tensors have shape [N,H,W,C], filters [K,R,S,C]; NCHW tensors [N,C,H,W],
filters [K,C,R,S]) and only build descriptors, fetch pointers and the current stream, and size
the caller-owned workspace.  PyTorch is used for device memory and streams, nothing else.

There is no CPU fallback: if libnsk.so has not been built, importing works but the first call
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnsk.so")

NSK_OK = 0
NSK_ERR_NULL, NSK_ERR_BAD_DESC, NSK_ERR_UNSUPPORTED, NSK_ERR_WORKSPACE, NSK_ERR_ALIGNMENT, NSK_ERR_HIP = 1, 2, 3, 4, 5, 6
NSK_F32, NSK_BF16 = 0, 1
NSK_NCHW, NSK_NHWC = 0, 1
NSK_PASS_FWD, NSK_PASS_DGRAD, NSK_PASS_WGRAD = 0, 1, 2
NSK_BN_FWD, NSK_BN_BWD = 0, 1


class nsk_conv_desc_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "dil_h", "dil_w",
                 "dtype", "layout")]


class nsk_bn_desc_t(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int), ("C", ctypes.c_int), ("H", ctypes.c_int), ("W", ctypes.c_int),
                ("dtype", ctypes.c_int), ("layout", ctypes.c_int), ("eps", ctypes.c_float),
                ("momentum", ctypes.c_float), ("relu", ctypes.c_int)]


class nsk_pool_desc_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in
                ("N", "C", "H", "W", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "dtype", "layout")]


class nsk_linear_desc_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("N", "C", "K", "dtype")]


class nsk_param_t(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("grad", ctypes.c_void_p), ("state1", ctypes.c_void_p), ("state2", ctypes.c_void_p),
                ("w_lp", ctypes.c_void_p), ("n", ctypes.c_size_t), ("weight_decay", ctypes.c_float)]


class NskError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().nsk_status_string(status).decode()
        if status == NSK_ERR_HIP:
            msg += f" (hipError_t {lib().nsk_last_hip_error()})"
        super().__init__(f"{where}: {msg}")


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libnsk.so (built by paper_2409_11600_amd.build).  Raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2409_11600_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        cd, bd, pd = ctypes.POINTER(nsk_conv_desc_t), ctypes.POINTER(nsk_bn_desc_t), ctypes.POINTER(nsk_pool_desc_t)
        ip = ctypes.POINTER(ctypes.c_int)
        L.nsk_version.restype = ci
        L.nsk_version.argtypes = []
        L.nsk_test_hooks_reload.restype = None
        L.nsk_test_hooks_reload.argtypes = []
        L.nsk_status_string.restype = ctypes.c_char_p
        L.nsk_status_string.argtypes = [ci]
        L.nsk_last_hip_error.restype = ci
        L.nsk_last_hip_error.argtypes = []
        L.nsk_conv2d_out_dims.restype = ci
        L.nsk_conv2d_out_dims.argtypes = [cd, ip, ip]
        L.nsk_conv2d_workspace_bytes.restype = sz
        L.nsk_conv2d_workspace_bytes.argtypes = [cd, ci]
        L.nsk_conv2d_fwd.restype = ci
        L.nsk_conv2d_fwd.argtypes = [cd, vp, vp, vp, vp, sz, vp]
        L.nsk_conv2d_dgrad.restype = ci
        L.nsk_conv2d_dgrad.argtypes = [cd, vp, vp, vp, ci, vp, sz, vp]
        L.nsk_conv2d_wgrad.restype = ci
        L.nsk_conv2d_wgrad.argtypes = [cd, vp, vp, vp, ci, vp, sz, vp]
        L.nsk_conv2d_grouped_workspace_bytes.restype = sz
        L.nsk_conv2d_grouped_workspace_bytes.argtypes = [cd, ci, ci]
        L.nsk_conv2d_grouped_fwd.restype = ci
        L.nsk_conv2d_grouped_fwd.argtypes = [cd, ci, vp, vp, vp, vp, sz, vp]
        L.nsk_conv2d_grouped_dgrad.restype = ci
        L.nsk_conv2d_grouped_dgrad.argtypes = [cd, ci, vp, vp, vp, ci, vp, sz, vp]
        L.nsk_conv2d_grouped_wgrad.restype = ci
        L.nsk_conv2d_grouped_wgrad.argtypes = [cd, ci, vp, vp, vp, ci, vp, sz, vp]
        L.nsk_bn_workspace_bytes.restype = sz
        L.nsk_bn_workspace_bytes.argtypes = [bd, ci]
        L.nsk_bn_relu_add_fwd.restype = ci
        L.nsk_bn_relu_add_fwd.argtypes = [bd] + [vp] * 10 + [sz, vp]
        L.nsk_bn_fwd_coeffs.restype = ci
        L.nsk_bn_fwd_coeffs.argtypes = [bd, vp, vp, vp, ci, vp, vp, vp, vp, vp, vp, sz, vp]
        L.nsk_conv2d_act_supported.restype = ci
        L.nsk_conv2d_act_supported.argtypes = [cd]
        L.nsk_conv2d_act_workspace_bytes.restype = sz
        L.nsk_conv2d_act_workspace_bytes.argtypes = [cd, ci]
        L.nsk_conv2d_fwd_act.restype = ci
        L.nsk_conv2d_fwd_act.argtypes = [cd, vp, vp, vp, vp, vp, vp, sz, vp]
        L.nsk_conv2d_wgrad_act.restype = ci
        L.nsk_conv2d_wgrad_act.argtypes = [cd, vp, vp, vp, vp, ci, vp, sz, vp]
        L.nsk_bn_relu_bwd_act.restype = ci
        L.nsk_bn_relu_bwd_act.argtypes = [bd] + [vp] * 10 + [sz, vp]
        L.nsk_static_scratch_bytes.restype = sz
        L.nsk_static_scratch_bytes.argtypes = []
        L.nsk_bn_relu_add_fwd_static.restype = ci
        L.nsk_bn_relu_add_fwd_static.argtypes = [bd] + [vp] * 10
        L.nsk_bn_relu_add_bwd.restype = ci
        L.nsk_bn_relu_add_bwd.argtypes = [bd] + [vp] * 11 + [sz, vp]
        L.nsk_conv2d_stats_rows.restype = ci
        L.nsk_conv2d_stats_rows.argtypes = [cd]
        L.nsk_conv2d_fwd_stats.restype = ci
        L.nsk_conv2d_fwd_stats.argtypes = [cd, vp, vp, vp, vp, vp, sz, vp]
        L.nsk_bn_relu_add_fwd_stats.restype = ci
        L.nsk_bn_relu_add_fwd_stats.argtypes = [bd] + [vp] * 11 + [ci, vp, sz, vp]
        L.nsk_bn_mask_bytes.restype = sz
        L.nsk_bn_mask_bytes.argtypes = [bd]
        L.nsk_bn_relu_add_fwd_mask.restype = ci
        L.nsk_bn_relu_add_fwd_mask.argtypes = [bd] + [vp] * 11 + [sz, vp]
        L.nsk_bn_relu_add_bwd_mask.restype = ci
        L.nsk_bn_relu_add_bwd_mask.argtypes = [bd] + [vp] * 11 + [sz, vp]
        L.nsk_maxpool2d_out_dims.restype = ci
        L.nsk_maxpool2d_out_dims.argtypes = [pd, ip, ip]
        L.nsk_maxpool2d_fwd.restype = ci
        L.nsk_maxpool2d_fwd.argtypes = [pd, vp, vp, vp, vp]
        L.nsk_maxpool2d_bwd.restype = ci
        L.nsk_maxpool2d_bwd.argtypes = [pd, vp, vp, vp, vp]
        ld, cf = ctypes.POINTER(nsk_linear_desc_t), ctypes.c_float
        L.nsk_global_avgpool_fwd.restype = ci
        L.nsk_global_avgpool_fwd.argtypes = [ci] * 6 + [vp, vp, vp]
        L.nsk_global_avgpool_bwd.restype = ci
        L.nsk_global_avgpool_bwd.argtypes = [ci] * 6 + [vp, vp, ci, vp]
        L.nsk_linear_workspace_bytes.restype = sz
        L.nsk_linear_workspace_bytes.argtypes = [ld, ci]
        L.nsk_linear_fwd.restype = ci
        L.nsk_linear_fwd.argtypes = [ld, vp, vp, vp, vp, vp, sz, vp]
        L.nsk_linear_dgrad.restype = ci
        L.nsk_linear_dgrad.argtypes = [ld, vp, vp, vp, ci, vp, sz, vp]
        L.nsk_linear_wgrad.restype = ci
        L.nsk_linear_wgrad.argtypes = [ld, vp, vp, vp, vp, ci, vp, sz, vp]
        L.nsk_transpose2d.restype = ci
        L.nsk_transpose2d.argtypes = [ci, ci, ci, vp, vp, vp]
        L.nsk_softmax_xent_fwd.restype = ci
        L.nsk_softmax_xent_fwd.argtypes = [ci, ci, ci, vp, vp, vp, vp, vp]
        L.nsk_softmax_xent_bwd.restype = ci
        L.nsk_softmax_xent_bwd.argtypes = [ci, ci, ci, vp, vp, cf, vp, vp]
        L.nsk_sgd_momentum_step.restype = ci
        L.nsk_sgd_momentum_step.argtypes = [sz, vp, vp, vp, vp, cf, cf, cf, vp, vp]
        L.nsk_adamw_step.restype = ci
        L.nsk_adamw_step.argtypes = [sz, vp, vp, vp, vp, vp, ci, cf, cf, cf, cf, cf, vp, vp]
        pp = ctypes.POINTER(nsk_param_t)
        L.nsk_sgd_momentum_step_multi.restype = ci
        L.nsk_sgd_momentum_step_multi.argtypes = [ci, pp, cf, cf, vp, vp]
        L.nsk_adamw_step_multi.restype = ci
        L.nsk_adamw_step_multi.argtypes = [ci, pp, ci, cf, cf, cf, cf, vp, vp]
        L.nsk_sumsq_accumulate.restype = ci
        L.nsk_sumsq_accumulate.argtypes = [sz, vp, vp, vp, vp]
        L.nsk_clip_scale.restype = ci
        L.nsk_clip_scale.argtypes = [vp, cf, vp, vp]
        L.nsk_embedding_fwd.restype = ci
        L.nsk_embedding_fwd.argtypes = [ci, ci, ci, ci, vp, vp, vp, vp]
        L.nsk_embedding_bwd.restype = ci
        L.nsk_embedding_bwd.argtypes = [ci, ci, ci, ci, vp, vp, vp, ci, vp]
        L.nsk_gru_gates_fwd.restype = ci
        L.nsk_gru_gates_fwd.argtypes = [ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp]
        L.nsk_gru_gates_bwd.restype = ci
        L.nsk_gru_gates_bwd.argtypes = [ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.nsk_gru_step_supported.restype = ci
        L.nsk_gru_step_supported.argtypes = [ci, ci]
        L.nsk_gru_step_fwd.restype = ci
        L.nsk_gru_step_fwd.argtypes = [ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp]
        L.nsk_gru_step_bwd.restype = ci
        L.nsk_gru_step_bwd.argtypes = [ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        vpp, szp = ctypes.POINTER(vp), ctypes.POINTER(sz)
        L.nsk_pool_create.restype = ci
        L.nsk_pool_create.argtypes = [ci, vpp]
        L.nsk_pool_get.restype = ci
        L.nsk_pool_get.argtypes = [vp, sz, vpp]
        L.nsk_pool_put.restype = ci
        L.nsk_pool_put.argtypes = [vp, vp]
        L.nsk_pool_cached.restype = ci
        L.nsk_pool_cached.argtypes = [vp, ctypes.c_char_p, sz, vpp, ip]
        L.nsk_pool_stats.restype = ci
        L.nsk_pool_stats.argtypes = [vp, szp, szp, szp, szp]
        L.nsk_pool_destroy.restype = ci
        L.nsk_pool_destroy.argtypes = [vp]
        _lib = L
    return _lib


EXPORTS = ("nsk_version", "nsk_test_hooks_reload", "nsk_status_string", "nsk_last_hip_error", "nsk_conv2d_out_dims",
           "nsk_conv2d_workspace_bytes", "nsk_conv2d_fwd", "nsk_conv2d_dgrad", "nsk_conv2d_wgrad",
           "nsk_conv2d_grouped_workspace_bytes", "nsk_conv2d_grouped_fwd", "nsk_conv2d_grouped_dgrad",
           "nsk_conv2d_grouped_wgrad",
           "nsk_bn_workspace_bytes", "nsk_bn_relu_add_fwd", "nsk_bn_fwd_coeffs", "nsk_conv2d_act_supported", "nsk_conv2d_act_workspace_bytes",
           "nsk_conv2d_fwd_act", "nsk_conv2d_wgrad_act", "nsk_bn_relu_bwd_act", "nsk_static_scratch_bytes", "nsk_bn_relu_add_fwd_static",
           "nsk_bn_relu_add_bwd", "nsk_bn_mask_bytes",
           "nsk_bn_relu_add_fwd_mask", "nsk_bn_relu_add_bwd_mask", "nsk_conv2d_stats_rows", "nsk_conv2d_fwd_stats",
           "nsk_bn_relu_add_fwd_stats", "nsk_maxpool2d_out_dims",
           "nsk_maxpool2d_fwd", "nsk_maxpool2d_bwd",
           "nsk_global_avgpool_fwd", "nsk_global_avgpool_bwd", "nsk_linear_workspace_bytes", "nsk_linear_fwd",
           "nsk_linear_dgrad", "nsk_linear_wgrad", "nsk_transpose2d", "nsk_softmax_xent_fwd", "nsk_softmax_xent_bwd",
           "nsk_sgd_momentum_step", "nsk_adamw_step", "nsk_sgd_momentum_step_multi", "nsk_adamw_step_multi", "nsk_sumsq_accumulate", "nsk_clip_scale",
           "nsk_embedding_fwd", "nsk_embedding_bwd", "nsk_gru_gates_fwd", "nsk_gru_gates_bwd",
           "nsk_gru_step_supported", "nsk_gru_step_fwd", "nsk_gru_step_bwd",
           "nsk_pool_create", "nsk_pool_get", "nsk_pool_put", "nsk_pool_cached", "nsk_pool_stats", "nsk_pool_destroy")
NSK_POOL_DEVICE, NSK_POOL_HOST = 0, 1
NSK_SUMSQ_PARTIALS = 256


def __getattr__(name):  # raw entry points under their C names: binding.nsk_conv2d_fwd(...)
    if name in EXPORTS:
        return getattr(lib(), name)
    raise AttributeError(name)


# ------------------------------------------------------------------------------------ helpers

def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return NSK_F32
    if t.dtype == torch.bfloat16:
        return NSK_BF16
    raise TypeError(f"unsupported element type {t.dtype}")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors handed to libnsk must be contiguous CUDA tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _pair(v) -> Tuple[int, int]:
    return (int(v[0]), int(v[1])) if isinstance(v, (tuple, list)) else (int(v), int(v))


class Workspace:
    """Caller-owned scratch buffer, grown on demand and then reused (the paper's pooling idea:
    nothing is allocated in steady state)."""

    def __init__(self, device="cuda:0"):
        self.device = torch.device(device)
        self.buf: Optional[torch.Tensor] = None

    def get(self, nbytes: int):
        if nbytes == 0:
            return None, 0
        if self.buf is None or self.buf.numel() < nbytes:
            self.buf = torch.empty(int(nbytes), dtype=torch.uint8, device=self.device)
        return ctypes.c_void_p(self.buf.data_ptr()), self.buf.numel()


def conv_desc(act_dims, filt_dims, stride, pad, dilation, dtype_code, layout) -> nsk_conv_desc_t:
    """act_dims = (N,C,H,W), filt_dims = (K,R,S): logical sizes, whatever the physical layout."""
    N, C, H, W = act_dims
    K, R, S = filt_dims
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dilation)
    return nsk_conv_desc_t(N, C, H, W, K, R, S, sh, sw, ph, pw, dh, dw, dtype_code, layout)


def _logical(t: torch.Tensor, layout: int):
    """(N, C, H, W) of an activation tensor stored in `layout`."""
    if layout == NSK_NHWC:
        N, H, W, C = t.shape
    else:
        N, C, H, W = t.shape
    return int(N), int(C), int(H), int(W)


def _filter_logical(w: torch.Tensor, layout: int):
    if layout == NSK_NHWC:
        K, R, S, C = w.shape
    else:
        K, C, R, S = w.shape
    return int(K), int(C), int(R), int(S)


def _act_shape(N, C, H, W, layout):
    return (N, H, W, C) if layout == NSK_NHWC else (N, C, H, W)


def _check(status: int, where: str):
    if status != NSK_OK:
        raise NskError(status, where)


def conv2d_out_dims(desc: nsk_conv_desc_t) -> Tuple[int, int]:
    P, Q = ctypes.c_int(), ctypes.c_int()
    _check(lib().nsk_conv2d_out_dims(ctypes.byref(desc), ctypes.byref(P), ctypes.byref(Q)), "nsk_conv2d_out_dims")
    return P.value, Q.value


def conv2d_fwd(x, w, stride=1, pad=0, dilation=1, layout=NSK_NHWC, out=None, ws: Optional[Workspace] = None):
    N, C, H, W = _logical(x, layout)
    K, Cw, R, S = _filter_logical(w, layout)
    assert Cw == C and w.dtype == x.dtype
    d = conv_desc((N, C, H, W), (K, R, S), stride, pad, dilation, _dtype_code(x), layout)
    P, Q = conv2d_out_dims(d)
    if out is None:
        out = torch.empty(_act_shape(N, K, P, Q, layout), dtype=x.dtype, device=x.device)
    ws = ws or Workspace(x.device)
    wp, wb = ws.get(lib().nsk_conv2d_workspace_bytes(ctypes.byref(d), NSK_PASS_FWD))
    _check(lib().nsk_conv2d_fwd(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(out), wp, wb, _stream()), "nsk_conv2d_fwd")
    return out


def conv2d_fwd_stats(x, w, stride=1, pad=0, dilation=1, layout=NSK_NHWC, out=None, stats=None,
                     ws: Optional[Workspace] = None):
    """Forward convolution that also returns the per-channel partial sums of its output: (y, stats) with stats a
    float32 tensor [2, rows, K] (sums, sums of squares) for bn_relu_add_fwd(..., stats=stats)."""
    N, C, H, W = _logical(x, layout)
    K, Cw, R, S = _filter_logical(w, layout)
    assert Cw == C and w.dtype == x.dtype
    d = conv_desc((N, C, H, W), (K, R, S), stride, pad, dilation, _dtype_code(x), layout)
    P, Q = conv2d_out_dims(d)
    if out is None:
        out = torch.empty(_act_shape(N, K, P, Q, layout), dtype=x.dtype, device=x.device)
    rows = int(lib().nsk_conv2d_stats_rows(ctypes.byref(d)))
    assert rows > 0
    if stats is None:
        stats = torch.empty((2, rows, K), dtype=torch.float32, device=x.device)
    assert stats.numel() == 2 * rows * K and stats.dtype == torch.float32
    ws = ws or Workspace(x.device)
    wp, wb = ws.get(lib().nsk_conv2d_workspace_bytes(ctypes.byref(d), NSK_PASS_FWD))
    _check(lib().nsk_conv2d_fwd_stats(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(out), _ptr(stats), wp, wb, _stream()),
           "nsk_conv2d_fwd_stats")
    return out, stats


def conv2d_dgrad(dy, w, x_logical, stride=1, pad=0, dilation=1, layout=NSK_NHWC, out=None, accumulate=False,
                 ws: Optional[Workspace] = None):
    """x_logical = (N,C,H,W) of the forward input."""
    N, C, H, W = x_logical
    K, Cw, R, S = _filter_logical(w, layout)
    assert Cw == C and w.dtype == dy.dtype
    d = conv_desc((N, C, H, W), (K, R, S), stride, pad, dilation, _dtype_code(dy), layout)
    if out is None:
        assert not accumulate
        out = torch.empty(_act_shape(N, C, H, W, layout), dtype=dy.dtype, device=dy.device)
    ws = ws or Workspace(dy.device)
    wp, wb = ws.get(lib().nsk_conv2d_workspace_bytes(ctypes.byref(d), NSK_PASS_DGRAD))
    _check(lib().nsk_conv2d_dgrad(ctypes.byref(d), _ptr(dy), _ptr(w), _ptr(out), int(bool(accumulate)), wp, wb,
                                  _stream()), "nsk_conv2d_dgrad")
    return out


def conv2d_wgrad(x, dy, filt_logical, stride=1, pad=0, dilation=1, layout=NSK_NHWC, out=None, accumulate=False,
                 ws: Optional[Workspace] = None):
    """filt_logical = (K,C,R,S).  Returns float32 dw shaped like the filter in `layout`."""
    N, C, H, W = _logical(x, layout)
    K, Cw, R, S = filt_logical
    assert Cw == C and x.dtype == dy.dtype
    d = conv_desc((N, C, H, W), (K, R, S), stride, pad, dilation, _dtype_code(x), layout)
    if out is None:
        assert not accumulate
        shape = (K, R, S, C) if layout == NSK_NHWC else (K, C, R, S)
        out = torch.empty(shape, dtype=torch.float32, device=x.device)
    assert out.dtype == torch.float32
    ws = ws or Workspace(x.device)
    wp, wb = ws.get(lib().nsk_conv2d_workspace_bytes(ctypes.byref(d), NSK_PASS_WGRAD))
    _check(lib().nsk_conv2d_wgrad(ctypes.byref(d), _ptr(x), _ptr(dy), _ptr(out), int(bool(accumulate)), wp, wb,
                                  _stream()), "nsk_conv2d_wgrad")
    return out


def conv2d_grouped_fwd(x, w, groups, stride=1, pad=0, dilation=1, layout=NSK_NHWC, out=None,
                       ws: Optional[Workspace] = None):
    """Grouped convolution: w holds C/groups input channels per output channel."""
    N, C, H, W = _logical(x, layout)
    K, Cw, R, S = _filter_logical(w, layout)
    assert Cw * groups == C and w.dtype == x.dtype
    d = conv_desc((N, C, H, W), (K, R, S), stride, pad, dilation, _dtype_code(x), layout)
    P, Q = conv2d_out_dims(d)
    if out is None:
        out = torch.empty(_act_shape(N, K, P, Q, layout), dtype=x.dtype, device=x.device)
    ws = ws or Workspace(x.device)
    wp, wb = ws.get(lib().nsk_conv2d_grouped_workspace_bytes(ctypes.byref(d), int(groups), NSK_PASS_FWD))
    _check(lib().nsk_conv2d_grouped_fwd(ctypes.byref(d), int(groups), _ptr(x), _ptr(w), _ptr(out), wp, wb, _stream()),
           "nsk_conv2d_grouped_fwd")
    return out


def conv2d_grouped_dgrad(dy, w, x_logical, groups, stride=1, pad=0, dilation=1, layout=NSK_NHWC, out=None,
                         accumulate=False, ws: Optional[Workspace] = None):
    """x_logical = (N,C,H,W) of the forward input."""
    N, C, H, W = x_logical
    K, Cw, R, S = _filter_logical(w, layout)
    assert Cw * groups == C and w.dtype == dy.dtype
    d = conv_desc((N, C, H, W), (K, R, S), stride, pad, dilation, _dtype_code(dy), layout)
    if out is None:
        assert not accumulate
        out = torch.empty(_act_shape(N, C, H, W, layout), dtype=dy.dtype, device=dy.device)
    ws = ws or Workspace(dy.device)
    wp, wb = ws.get(lib().nsk_conv2d_grouped_workspace_bytes(ctypes.byref(d), int(groups), NSK_PASS_DGRAD))
    _check(lib().nsk_conv2d_grouped_dgrad(ctypes.byref(d), int(groups), _ptr(dy), _ptr(w), _ptr(out),
                                          int(bool(accumulate)), wp, wb, _stream()), "nsk_conv2d_grouped_dgrad")
    return out


def conv2d_grouped_wgrad(x, dy, filt_logical, groups, stride=1, pad=0, dilation=1, layout=NSK_NHWC, out=None,
                         accumulate=False, ws: Optional[Workspace] = None):
    """filt_logical = (K, C/groups, R, S).  Returns float32 dw shaped like the filter in `layout`."""
    N, C, H, W = _logical(x, layout)
    K, Cw, R, S = filt_logical
    assert Cw * groups == C and x.dtype == dy.dtype
    d = conv_desc((N, C, H, W), (K, R, S), stride, pad, dilation, _dtype_code(x), layout)
    if out is None:
        assert not accumulate
        shape = (K, R, S, Cw) if layout == NSK_NHWC else (K, Cw, R, S)
        out = torch.empty(shape, dtype=torch.float32, device=x.device)
    assert out.dtype == torch.float32
    ws = ws or Workspace(x.device)
    wp, wb = ws.get(lib().nsk_conv2d_grouped_workspace_bytes(ctypes.byref(d), int(groups), NSK_PASS_WGRAD))
    _check(lib().nsk_conv2d_grouped_wgrad(ctypes.byref(d), int(groups), _ptr(x), _ptr(dy), _ptr(out),
                                          int(bool(accumulate)), wp, wb, _stream()), "nsk_conv2d_grouped_wgrad")
    return out


def bn_desc(x: torch.Tensor, layout, eps, momentum, relu) -> nsk_bn_desc_t:
    N, C, H, W = _logical(x, layout)
    return nsk_bn_desc_t(N, C, H, W, _dtype_code(x), layout, float(eps), float(momentum), int(bool(relu)))


def bn_mask_bytes(x, layout=NSK_NHWC, relu=True) -> int:
    """Bytes of the ReLU mask the *_mask calls exchange for a tensor like x; 0 if they do not apply."""
    d = bn_desc(x, layout, 1e-5, 0.1, relu)
    return int(lib().nsk_bn_mask_bytes(ctypes.byref(d)))


def bn_relu_add_fwd(x, gamma, beta, residual=None, eps=1e-5, relu=True, layout=NSK_NHWC, momentum=0.1,
                    running_mean=None, running_var=None, out=None, save_mean=None, save_invstd=None,
                    ws: Optional[Workspace] = None, relu_mask=None, stats=None):
    """Returns (out, save_mean, save_invstd).  With relu_mask (uint8 tensor of bn_mask_bytes(x) bytes) the ReLU
    mask is written there for bn_relu_add_bwd(..., relu_mask=...).  With stats ([2, rows, C] float32 partial sums of
    x and x*x, as returned by conv2d_fwd_stats) the statistics pass over x is skipped."""
    d = bn_desc(x, layout, eps, momentum, relu)
    C = d.C
    if out is None:
        out = torch.empty_like(x)
    if save_mean is None:
        save_mean = torch.empty(C, dtype=torch.float32, device=x.device)
    if save_invstd is None:
        save_invstd = torch.empty(C, dtype=torch.float32, device=x.device)
    ws = ws or Workspace(x.device)
    wp, wb = ws.get(lib().nsk_bn_workspace_bytes(ctypes.byref(d), NSK_BN_FWD))
    if stats is not None:
        _check(lib().nsk_bn_relu_add_fwd_stats(ctypes.byref(d), _ptr(x), _ptr(residual), _ptr(gamma), _ptr(beta), _ptr(out),
                                               _ptr(relu_mask), _ptr(save_mean), _ptr(save_invstd), _ptr(running_mean),
                                               _ptr(running_var), _ptr(stats), int(stats.shape[1]), wp, wb, _stream()),
               "nsk_bn_relu_add_fwd_stats")
        return out, save_mean, save_invstd
    if relu_mask is not None:
        _check(lib().nsk_bn_relu_add_fwd_mask(ctypes.byref(d), _ptr(x), _ptr(residual), _ptr(gamma), _ptr(beta), _ptr(out),
                                              _ptr(relu_mask), _ptr(save_mean), _ptr(save_invstd), _ptr(running_mean),
                                              _ptr(running_var), wp, wb, _stream()), "nsk_bn_relu_add_fwd_mask")
        return out, save_mean, save_invstd
    _check(lib().nsk_bn_relu_add_fwd(ctypes.byref(d), _ptr(x), _ptr(residual), _ptr(gamma), _ptr(beta), _ptr(out),
                                     _ptr(save_mean), _ptr(save_invstd), _ptr(running_mean), _ptr(running_var),
                                     wp, wb, _stream()), "nsk_bn_relu_add_fwd")
    return out, save_mean, save_invstd


def bn_fwd_coeffs(y, gamma, beta, stats, eps=1e-5, layout=NSK_NHWC, momentum=0.1, running_mean=None, running_var=None,
                  ws: Optional[Workspace] = None):
    """Batch statistics of y from its partial sums and the coefficients of the activation relu(scale*y + shift) that
    the consumers of y apply on load: returns (save_mean, save_invstd, coeffs) with coeffs float32 [2, C]."""
    d = bn_desc(y, layout, eps, momentum, True)
    mean = torch.empty(d.C, dtype=torch.float32, device=y.device)
    invstd = torch.empty(d.C, dtype=torch.float32, device=y.device)
    coeffs = torch.empty((2, d.C), dtype=torch.float32, device=y.device)
    ws = ws or Workspace(y.device)
    wp, wb = ws.get(lib().nsk_bn_workspace_bytes(ctypes.byref(d), NSK_BN_FWD))
    _check(lib().nsk_bn_fwd_coeffs(ctypes.byref(d), _ptr(gamma), _ptr(beta), _ptr(stats), int(stats.shape[1]), _ptr(mean),
                                   _ptr(invstd), _ptr(running_mean), _ptr(running_var), _ptr(coeffs), wp, wb, _stream()),
           "nsk_bn_fwd_coeffs")
    return mean, invstd, coeffs


def conv2d_fwd_act(x, coeffs, w, stride=1, pad=0, dilation=1, out=None, want_stats=False, ws: Optional[Workspace] = None):
    """Forward convolution of relu(coeffs[0]*x + coeffs[1]) (NHWC).  Returns y, or (y, stats) with want_stats."""
    N, C, H, W = _logical(x, NSK_NHWC)
    K, Cw, R, S = _filter_logical(w, NSK_NHWC)
    assert Cw == C and w.dtype == x.dtype and coeffs.numel() == 2 * C
    d = conv_desc((N, C, H, W), (K, R, S), stride, pad, dilation, _dtype_code(x), NSK_NHWC)
    P, Q = conv2d_out_dims(d)
    if out is None:
        out = torch.empty(_act_shape(N, K, P, Q, NSK_NHWC), dtype=x.dtype, device=x.device)
    stats = None
    if want_stats:
        rows = int(lib().nsk_conv2d_stats_rows(ctypes.byref(d)))
        stats = torch.empty((2, rows, K), dtype=torch.float32, device=x.device)
    ws = ws or Workspace(x.device)
    wp, wb = ws.get(lib().nsk_conv2d_act_workspace_bytes(ctypes.byref(d), NSK_PASS_FWD))
    _check(lib().nsk_conv2d_fwd_act(ctypes.byref(d), _ptr(x), _ptr(coeffs), _ptr(w), _ptr(out), _ptr(stats), wp, wb, _stream()),
           "nsk_conv2d_fwd_act")
    return (out, stats) if want_stats else out


def conv2d_wgrad_act(x, coeffs, dy, filt_logical, stride=1, pad=0, dilation=1, out=None, accumulate=False,
                     ws: Optional[Workspace] = None):
    """Backward-weight with x replaced by relu(coeffs[0]*x + coeffs[1]) (NHWC)."""
    N, C, H, W = _logical(x, NSK_NHWC)
    K, Cw, R, S = filt_logical
    assert Cw == C and x.dtype == dy.dtype
    d = conv_desc((N, C, H, W), (K, R, S), stride, pad, dilation, _dtype_code(x), NSK_NHWC)
    if out is None:
        assert not accumulate
        out = torch.empty((K, R, S, C), dtype=torch.float32, device=x.device)
    ws = ws or Workspace(x.device)
    wp, wb = ws.get(lib().nsk_conv2d_act_workspace_bytes(ctypes.byref(d), NSK_PASS_WGRAD))
    _check(lib().nsk_conv2d_wgrad_act(ctypes.byref(d), _ptr(x), _ptr(coeffs), _ptr(dy), _ptr(out), int(bool(accumulate)), wp, wb,
                                      _stream()), "nsk_conv2d_wgrad_act")
    return out


def bn_relu_bwd_act(x, coeffs, dout, gamma, save_mean, save_invstd, eps=1e-5, ws: Optional[Workspace] = None):
    """Backward of a batch-norm + ReLU whose output was never stored: returns (dx, dgamma, dbeta)."""
    d = bn_desc(x, NSK_NHWC, eps, 0.1, True)
    dx = torch.empty_like(x)
    dgamma = torch.empty(d.C, dtype=torch.float32, device=x.device)
    dbeta = torch.empty(d.C, dtype=torch.float32, device=x.device)
    ws = ws or Workspace(x.device)
    wp, wb = ws.get(lib().nsk_bn_workspace_bytes(ctypes.byref(d), NSK_BN_BWD))
    _check(lib().nsk_bn_relu_bwd_act(ctypes.byref(d), _ptr(x), _ptr(coeffs), _ptr(dout), _ptr(gamma), _ptr(save_mean),
                                     _ptr(save_invstd), _ptr(dx), _ptr(dgamma), _ptr(dbeta), wp, wb, _stream()),
           "nsk_bn_relu_bwd_act")
    return dx, dgamma, dbeta


def bn_relu_add_fwd_static(x, gamma, beta, residual=None, eps=1e-5, relu=True, layout=NSK_NHWC, momentum=0.1,
                           running_mean=None, running_var=None, out=None, save_mean=None, save_invstd=None):
    """nsk_bn_relu_add_fwd_static: the call that takes no workspace and allocates nothing (its partial sums live in a
    device array of the library).  The caller passes every output; this wrapper only creates the ones left out."""
    d = bn_desc(x, layout, eps, momentum, relu)
    if out is None:
        out = torch.empty_like(x)
    if save_mean is None:
        save_mean = torch.empty(d.C, dtype=torch.float32, device=x.device)
    if save_invstd is None:
        save_invstd = torch.empty(d.C, dtype=torch.float32, device=x.device)
    _check(lib().nsk_bn_relu_add_fwd_static(ctypes.byref(d), _ptr(x), _ptr(residual), _ptr(gamma), _ptr(beta), _ptr(out),
                                            _ptr(save_mean), _ptr(save_invstd), _ptr(running_mean), _ptr(running_var),
                                            _stream()), "nsk_bn_relu_add_fwd_static")
    return out, save_mean, save_invstd


def bn_relu_add_bwd(x, out, dout, gamma, save_mean, save_invstd, relu=True, layout=NSK_NHWC, eps=1e-5,
                    dx=None, dresidual=None, want_dresidual=False, dgamma=None, dbeta=None,
                    ws: Optional[Workspace] = None, relu_mask=None):
    """Returns (dx, dresidual or None, dgamma, dbeta).  With relu_mask (as written by bn_relu_add_fwd) `out` is
    not read and may be None."""
    d = bn_desc(x, layout, eps, 0.1, relu)
    C = d.C
    if dx is None:
        dx = torch.empty_like(x)
    if dresidual is None and want_dresidual:
        dresidual = torch.empty_like(x)
    if dgamma is None:
        dgamma = torch.empty(C, dtype=torch.float32, device=x.device)
    if dbeta is None:
        dbeta = torch.empty(C, dtype=torch.float32, device=x.device)
    ws = ws or Workspace(x.device)
    wp, wb = ws.get(lib().nsk_bn_workspace_bytes(ctypes.byref(d), NSK_BN_BWD))
    if relu_mask is not None:
        _check(lib().nsk_bn_relu_add_bwd_mask(ctypes.byref(d), _ptr(x), _ptr(relu_mask), _ptr(dout), _ptr(gamma),
                                              _ptr(save_mean), _ptr(save_invstd), _ptr(dx), _ptr(dresidual), _ptr(dgamma),
                                              _ptr(dbeta), wp, wb, _stream()), "nsk_bn_relu_add_bwd_mask")
        return dx, dresidual, dgamma, dbeta
    _check(lib().nsk_bn_relu_add_bwd(ctypes.byref(d), _ptr(x), _ptr(out), _ptr(dout), _ptr(gamma), _ptr(save_mean),
                                     _ptr(save_invstd), _ptr(dx), _ptr(dresidual), _ptr(dgamma), _ptr(dbeta),
                                     wp, wb, _stream()), "nsk_bn_relu_add_bwd")
    return dx, dresidual, dgamma, dbeta


def pool_desc(x: torch.Tensor, window, stride, pad, layout) -> nsk_pool_desc_t:
    N, C, H, W = _logical(x, layout)
    R, S = _pair(window)
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    return nsk_pool_desc_t(N, C, H, W, R, S, sh, sw, ph, pw, _dtype_code(x), layout)


def maxpool2d_fwd(x, window=3, stride=2, pad=1, layout=NSK_NHWC, out=None, idx=None):
    """Returns (y, idx int8)."""
    d = pool_desc(x, window, stride, pad, layout)
    P, Q = ctypes.c_int(), ctypes.c_int()
    _check(lib().nsk_maxpool2d_out_dims(ctypes.byref(d), ctypes.byref(P), ctypes.byref(Q)), "nsk_maxpool2d_out_dims")
    shape = _act_shape(d.N, d.C, P.value, Q.value, layout)
    if out is None:
        out = torch.empty(shape, dtype=x.dtype, device=x.device)
    if idx is None:
        idx = torch.empty(shape, dtype=torch.int8, device=x.device)
    _check(lib().nsk_maxpool2d_fwd(ctypes.byref(d), _ptr(x), _ptr(out), _ptr(idx), _stream()), "nsk_maxpool2d_fwd")
    return out, idx


def maxpool2d_bwd(dy, idx, x_logical, window=3, stride=2, pad=1, layout=NSK_NHWC, out=None):
    N, C, H, W = x_logical
    R, S = _pair(window)
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    d = nsk_pool_desc_t(N, C, H, W, R, S, sh, sw, ph, pw, _dtype_code(dy), layout)
    if out is None:
        out = torch.empty(_act_shape(N, C, H, W, layout), dtype=dy.dtype, device=dy.device)
    _check(lib().nsk_maxpool2d_bwd(ctypes.byref(d), _ptr(dy), _ptr(idx), _ptr(out), _stream()), "nsk_maxpool2d_bwd")
    return out


# ------------------------------------------------------------------------------------ training-step tail

def global_avgpool_fwd(x, layout=NSK_NHWC, out=None):
    N, C, H, W = _logical(x, layout)
    if out is None:
        out = torch.empty((N, C), dtype=x.dtype, device=x.device)
    _check(lib().nsk_global_avgpool_fwd(_dtype_code(x), layout, N, C, H, W, _ptr(x), _ptr(out), _stream()),
           "nsk_global_avgpool_fwd")
    return out


def global_avgpool_bwd(dy, x_logical, layout=NSK_NHWC, out=None, accumulate=False):
    N, C, H, W = x_logical
    if out is None:
        assert not accumulate
        out = torch.empty(_act_shape(N, C, H, W, layout), dtype=dy.dtype, device=dy.device)
    _check(lib().nsk_global_avgpool_bwd(_dtype_code(dy), layout, N, C, H, W, _ptr(dy), _ptr(out), int(accumulate),
                                        _stream()), "nsk_global_avgpool_bwd")
    return out


def _linear_desc(N, C, K, t):
    return nsk_linear_desc_t(int(N), int(C), int(K), _dtype_code(t))


def linear_fwd(x, w, bias=None, out=None, ws: Optional[Workspace] = None):
    """y = x @ w^T (+ bias): x [N,C], w [K,C], bias float [K]."""
    (N, C), (K, Cw) = x.shape, w.shape
    assert C == Cw and w.dtype == x.dtype
    d = _linear_desc(N, C, K, x)
    if out is None:
        out = torch.empty((N, K), dtype=x.dtype, device=x.device)
    ws = ws or Workspace(x.device)
    wp, wb = ws.get(lib().nsk_linear_workspace_bytes(ctypes.byref(d), NSK_PASS_FWD))
    _check(lib().nsk_linear_fwd(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(bias), _ptr(out), wp, wb, _stream()),
           "nsk_linear_fwd")
    return out


def linear_dgrad(dy, w, out=None, accumulate=False, ws: Optional[Workspace] = None):
    (N, K), (Kw, C) = dy.shape, w.shape
    assert K == Kw and w.dtype == dy.dtype
    d = _linear_desc(N, C, K, dy)
    if out is None:
        assert not accumulate
        out = torch.empty((N, C), dtype=dy.dtype, device=dy.device)
    ws = ws or Workspace(dy.device)
    wp, wb = ws.get(lib().nsk_linear_workspace_bytes(ctypes.byref(d), NSK_PASS_DGRAD))
    _check(lib().nsk_linear_dgrad(ctypes.byref(d), _ptr(dy), _ptr(w), _ptr(out), int(accumulate), wp, wb, _stream()),
           "nsk_linear_dgrad")
    return out


def linear_wgrad(x, dy, dw=None, db=None, accumulate=False, want_db=True, ws: Optional[Workspace] = None):
    (N, C), (Nd, K) = x.shape, dy.shape
    assert N == Nd and x.dtype == dy.dtype
    d = _linear_desc(N, C, K, x)
    if dw is None:
        assert not accumulate
        dw = torch.empty((K, C), dtype=torch.float32, device=x.device)
    if db is None and want_db:
        assert not accumulate
        db = torch.empty((K,), dtype=torch.float32, device=x.device)
    ws = ws or Workspace(x.device)
    wp, wb = ws.get(lib().nsk_linear_workspace_bytes(ctypes.byref(d), NSK_PASS_WGRAD))
    _check(lib().nsk_linear_wgrad(ctypes.byref(d), _ptr(x), _ptr(dy), _ptr(dw), _ptr(db), int(accumulate), wp, wb,
                                  _stream()), "nsk_linear_wgrad")
    return dw, db


def transpose2d(src, out=None):
    """out[c][r] = src[r][c]."""
    rows, cols = src.shape
    if out is None:
        out = torch.empty((cols, rows), dtype=src.dtype, device=src.device)
    _check(lib().nsk_transpose2d(_dtype_code(src), int(rows), int(cols), _ptr(src), _ptr(out), _stream()), "nsk_transpose2d")
    return out


def softmax_xent_fwd(logits, labels, per_sample=None, loss=None):
    """labels: int32 [N].  Returns (loss [1] float32, per_sample [N] float32), both on the device."""
    N, K = logits.shape
    assert labels.dtype == torch.int32 and labels.numel() == N
    if per_sample is None:
        per_sample = torch.empty((N,), dtype=torch.float32, device=logits.device)
    if loss is None:
        loss = torch.empty((1,), dtype=torch.float32, device=logits.device)
    _check(lib().nsk_softmax_xent_fwd(_dtype_code(logits), int(N), int(K), _ptr(logits), _ptr(labels), _ptr(per_sample),
                                      _ptr(loss), _stream()), "nsk_softmax_xent_fwd")
    return loss, per_sample


def softmax_xent_bwd(logits, labels, dloss=1.0, out=None):
    N, K = logits.shape
    assert labels.dtype == torch.int32 and labels.numel() == N
    if out is None:
        out = torch.empty_like(logits)
    _check(lib().nsk_softmax_xent_bwd(_dtype_code(logits), int(N), int(K), _ptr(logits), _ptr(labels), float(dloss),
                                      _ptr(out), _stream()), "nsk_softmax_xent_bwd")
    return out


def sgd_momentum_step(w, grad, velocity, lr, momentum=0.9, weight_decay=0.0, w_lp=None, grad_scale=None):
    """In place on the float32 tensors w, grad (zeroed), velocity; w_lp: optional bfloat16 copy of w."""
    n = w.numel()
    assert grad.numel() == n and velocity.numel() == n and all(t.dtype == torch.float32 for t in (w, grad, velocity))
    assert w_lp is None or (w_lp.dtype == torch.bfloat16 and w_lp.numel() == n)
    _check(lib().nsk_sgd_momentum_step(n, _ptr(w), _ptr(grad), _ptr(velocity), _ptr(w_lp), float(lr), float(momentum),
                                       float(weight_decay), _ptr(grad_scale), _stream()), "nsk_sgd_momentum_step")


def adamw_step(w, grad, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, w_lp=None,
               grad_scale=None):
    n = w.numel()
    assert all(t.numel() == n and t.dtype == torch.float32 for t in (w, grad, m, v))
    assert w_lp is None or (w_lp.dtype == torch.bfloat16 and w_lp.numel() == n)
    _check(lib().nsk_adamw_step(n, _ptr(w), _ptr(grad), _ptr(m), _ptr(v), _ptr(w_lp), int(step), float(lr), float(beta1),
                                float(beta2), float(eps), float(weight_decay), _ptr(grad_scale), _stream()),
           "nsk_adamw_step")


def param_table(records):
    """records: iterable of (w, grad, state1, state2 or None, w_lp or None, weight_decay) tensors -> ctypes array of
    nsk_param_t (keep the tensors alive while it is in use)."""
    records = list(records)
    tab = (nsk_param_t * len(records))()
    for i, (w, g, s1, s2, lp, wd) in enumerate(records):
        n = w.numel()
        assert all(t.dtype == torch.float32 and t.numel() == n and t.is_contiguous() for t in (w, g, s1))
        assert s2 is None or (s2.dtype == torch.float32 and s2.numel() == n)
        assert lp is None or (lp.dtype == torch.bfloat16 and lp.numel() == n)
        tab[i] = nsk_param_t(w.data_ptr(), g.data_ptr(), s1.data_ptr(), s2.data_ptr() if s2 is not None else None,
                             lp.data_ptr() if lp is not None else None, n, float(wd))
    return tab


def sgd_momentum_step_multi(tab, lr, momentum=0.9, grad_scale=None):
    _check(lib().nsk_sgd_momentum_step_multi(len(tab), tab, float(lr), float(momentum), _ptr(grad_scale), _stream()),
           "nsk_sgd_momentum_step_multi")


def adamw_step_multi(tab, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, grad_scale=None):
    _check(lib().nsk_adamw_step_multi(len(tab), tab, int(step), float(lr), float(beta1), float(beta2), float(eps),
                                      _ptr(grad_scale), _stream()), "nsk_adamw_step_multi")


def clip_scale(grads, max_norm, partials=None, sumsq=None, scale=None):
    """Device float [1] = min(1, max_norm / (global L2 norm of `grads` + 1e-6)); no host synchronisation."""
    dev = grads[0].device
    if partials is None:
        partials = torch.empty((NSK_SUMSQ_PARTIALS,), dtype=torch.float32, device=dev)
    if sumsq is None:
        sumsq = torch.empty((1,), dtype=torch.float32, device=dev)
    if scale is None:
        scale = torch.empty((1,), dtype=torch.float32, device=dev)
    sumsq.zero_()
    for g in grads:
        assert g.dtype == torch.float32
        _check(lib().nsk_sumsq_accumulate(g.numel(), _ptr(g), _ptr(partials), _ptr(sumsq), _stream()),
               "nsk_sumsq_accumulate")
    _check(lib().nsk_clip_scale(_ptr(sumsq), float(max_norm), _ptr(scale), _stream()), "nsk_clip_scale")
    return scale


# ------------------------------------------------------------------------------------ recurrent workload

def embedding_fwd(tokens, table, out=None):
    """tokens: int32 [n]; table [V, E] -> out [n, E]."""
    n, (V, E) = tokens.numel(), table.shape
    assert tokens.dtype == torch.int32
    if out is None:
        out = torch.empty((n, E), dtype=table.dtype, device=table.device)
    _check(lib().nsk_embedding_fwd(_dtype_code(table), n, int(E), int(V), _ptr(tokens), _ptr(table), _ptr(out), _stream()),
           "nsk_embedding_fwd")
    return out


def embedding_bwd(tokens, dout, V, dtable=None, accumulate=False):
    n, E = tokens.numel(), dout.shape[-1]
    assert tokens.dtype == torch.int32 and dout.numel() == n * E
    if dtable is None:
        assert not accumulate
        dtable = torch.empty((V, E), dtype=torch.float32, device=dout.device)
    _check(lib().nsk_embedding_bwd(_dtype_code(dout), n, int(E), int(V), _ptr(tokens), _ptr(dout), _ptr(dtable),
                                   int(accumulate), _stream()), "nsk_embedding_bwd")
    return dtable


def gru_gates_fwd(gi, gh, b_ih, b_hh, h_prev, h_new=None, saved=None):
    N, H = h_prev.shape
    if h_new is None:
        h_new = torch.empty_like(h_prev)
    if saved is None:
        saved = torch.empty((N, 4 * H), dtype=h_prev.dtype, device=h_prev.device)
    _check(lib().nsk_gru_gates_fwd(_dtype_code(h_prev), int(N), int(H), _ptr(gi), _ptr(gh), _ptr(b_ih), _ptr(b_hh),
                                   _ptr(h_prev), _ptr(h_new), _ptr(saved), _stream()), "nsk_gru_gates_fwd")
    return h_new, saved


def gru_gates_bwd(saved, h_prev, dh_a, dh_b=None, dh_c=None, dgi=None, dgh=None, dh_direct=None):
    N, H = h_prev.shape
    mk = lambda w: torch.empty((N, w), dtype=h_prev.dtype, device=h_prev.device)
    dgi = mk(3 * H) if dgi is None else dgi
    dgh = mk(3 * H) if dgh is None else dgh
    dh_direct = mk(H) if dh_direct is None else dh_direct
    _check(lib().nsk_gru_gates_bwd(_dtype_code(h_prev), int(N), int(H), _ptr(saved), _ptr(h_prev), _ptr(dh_a), _ptr(dh_b),
                                   _ptr(dh_c), _ptr(dgi), _ptr(dgh), _ptr(dh_direct), _stream()), "nsk_gru_gates_bwd")
    return dgi, dgh, dh_direct


def gru_step_supported(N: int, H: int) -> bool:
    return bool(lib().nsk_gru_step_supported(int(N), int(H)))


def gru_step_fwd(gi, w_hh, b_ih, b_hh, h_prev, h_new=None, saved=None):
    N, H = h_prev.shape
    h_new = torch.empty_like(h_prev) if h_new is None else h_new
    saved = torch.empty((N, 4 * H), dtype=h_prev.dtype, device=h_prev.device) if saved is None else saved
    _check(lib().nsk_gru_step_fwd(_dtype_code(h_prev), int(N), int(H), _ptr(gi), _ptr(w_hh), _ptr(b_ih), _ptr(b_hh),
                                  _ptr(h_prev), _ptr(h_new), _ptr(saved), _stream()), "nsk_gru_step_fwd")
    return h_new, saved


def gru_step_bwd(saved, h_prev, w_hh_t, dh_a=None, dh_direct_next=None, dgh_next=None, dgi=None, dgh=None, dh_direct=None):
    N, H = h_prev.shape
    mk = lambda w: torch.empty((N, w), dtype=h_prev.dtype, device=h_prev.device)
    dgi = mk(3 * H) if dgi is None else dgi
    dgh = mk(3 * H) if dgh is None else dgh
    dh_direct = mk(H) if dh_direct is None else dh_direct
    _check(lib().nsk_gru_step_bwd(_dtype_code(h_prev), int(N), int(H), _ptr(saved), _ptr(h_prev), _ptr(dh_a),
                                  _ptr(dh_direct_next), _ptr(dgh_next), _ptr(w_hh_t), _ptr(dgi), _ptr(dgh), _ptr(dh_direct),
                                  _stream()), "nsk_gru_step_bwd")
    return dgi, dgh, dh_direct


# ------------------------------------------------------------------------------------ memory pool

class Pool:
    """Size-keyed pool of raw buffers plus a name-keyed cache (nsk_pool_*).  Pointers are plain integers."""

    def __init__(self, kind=NSK_POOL_DEVICE):
        self._h = ctypes.c_void_p()
        _check(lib().nsk_pool_create(kind, ctypes.byref(self._h)), "nsk_pool_create")

    def get(self, nbytes: int) -> int:
        p = ctypes.c_void_p()
        _check(lib().nsk_pool_get(self._h, int(nbytes), ctypes.byref(p)), "nsk_pool_get")
        return p.value

    def put(self, ptr: int):
        _check(lib().nsk_pool_put(self._h, ctypes.c_void_p(ptr)), "nsk_pool_put")

    def cached(self, name: str, nbytes: int):
        """(pointer, created)"""
        p, c = ctypes.c_void_p(), ctypes.c_int()
        _check(lib().nsk_pool_cached(self._h, name.encode(), int(nbytes), ctypes.byref(p), ctypes.byref(c)), "nsk_pool_cached")
        return p.value, bool(c.value)

    def stats(self) -> dict:
        v = [ctypes.c_size_t() for _ in range(4)]
        _check(lib().nsk_pool_stats(self._h, *[ctypes.byref(x) for x in v]), "nsk_pool_stats")
        return dict(zip(("bytes_allocated", "allocations", "requests", "hits"), (x.value for x in v)))

    def destroy(self):
        if self._h:
            _check(lib().nsk_pool_destroy(self._h), "nsk_pool_destroy")
            self._h = ctypes.c_void_p()
