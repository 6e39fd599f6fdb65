"""CPU oracle for the residual-CNN training hot path (ctypes front end).

TEST INFRASTRUCTURE ONLY.  The arithmetic lives in ``nsk_oracle.c`` next to this
file: plain fp64 nested loops that follow the definitions of convolution,
batch-norm + ReLU + residual-add and max pooling implied by the ResNet recipe
the paper trains with (section "Experiments and Discussion"), with gradients
derived by hand under the accumulate-into-existing-buffer rule of section
"Automatic Differentiation".  Only tests, the smoke check and the bench's
``cpu_baseline`` leg may import this package; the GPU library never does and
shares no code with it.

All tensors here are numpy float64, activations NCHW, filters KCRS.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nsk_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile nsk_oracle.c with gcc into liboracle.so (next to the source)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-fno-fast-math", "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        bp = ctypes.POINTER(ctypes.c_int8)
        i, i64, d = ctypes.c_int, ctypes.c_int64, ctypes.c_double
        lib.oracle_num_threads.restype = i
        lib.oracle_conv2d_out_dims.argtypes = [ip, ip, ip]
        lib.oracle_conv2d_fwd.argtypes = [dp, dp, dp, ip]
        lib.oracle_conv2d_dgrad.argtypes = [dp, dp, dp, ip, i]
        lib.oracle_conv2d_wgrad.argtypes = [dp, dp, dp, ip, i]
        lib.oracle_conv2d_fwd_at.argtypes = [dp, dp, ip, i64, ip, dp]
        lib.oracle_conv2d_dgrad_at.argtypes = [dp, dp, ip, i64, ip, dp]
        lib.oracle_conv2d_wgrad_at.argtypes = [dp, dp, ip, i64, ip, dp]
        lib.oracle_bn_relu_add_fwd.argtypes = [dp, dp, dp, dp, dp, dp, dp, dp, dp, i, i, i, i, d, d, i]
        lib.oracle_bn_relu_add_bwd.argtypes = [dp, dp, dp, dp, dp, dp, dp, dp, dp, dp, i, i, i, i, i]
        lib.oracle_maxpool2d_fwd.argtypes = [dp, dp, bp] + [i] * 10
        lib.oracle_maxpool2d_bwd.argtypes = [dp, bp, dp] + [i] * 10
        lib.oracle_round_bf16.argtypes = [dp, dp, i64]
        for name in ("oracle_conv2d_out_dims", "oracle_conv2d_fwd", "oracle_conv2d_dgrad",
                     "oracle_conv2d_wgrad", "oracle_conv2d_fwd_at", "oracle_conv2d_dgrad_at",
                     "oracle_conv2d_wgrad_at", "oracle_bn_relu_add_fwd", "oracle_bn_relu_add_bwd",
                     "oracle_maxpool2d_fwd", "oracle_maxpool2d_bwd", "oracle_round_bf16"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _dp(a: Optional[np.ndarray]):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _ip(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _pair(v) -> Tuple[int, int]:
    if isinstance(v, (tuple, list)):
        return int(v[0]), int(v[1])
    return int(v), int(v)


def _dims(xshape: Sequence[int], wshape: Sequence[int], stride, pad, dilation) -> np.ndarray:
    N, C, H, W = (int(v) for v in xshape)
    K, Cw, R, S = (int(v) for v in wshape)
    if Cw != C:
        raise ValueError(f"filter has {Cw} input channels, activation has {C}")
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dilation)
    if min(sh, sw, dh, dw) < 1 or min(ph, pw) < 0:
        raise ValueError("stride and dilation must be >= 1, padding >= 0")
    return np.array([N, C, H, W, K, R, S, sh, sw, ph, pw, dh, dw], dtype=np.int32)


def num_threads() -> int:
    """Threads the OpenMP loops will use."""
    return int(_load().oracle_num_threads())


def conv2d_out_dims(xshape, wshape, stride=1, pad=0, dilation=1) -> Tuple[int, int]:
    """P, Q = floor((H + 2*pad - dil*(R-1) - 1)/stride) + 1 per axis (0 if the filter does not fit)."""
    d = _dims(xshape, wshape, stride, pad, dilation)
    P, Q = ctypes.c_int32(), ctypes.c_int32()
    _load().oracle_conv2d_out_dims(_ip(d), ctypes.byref(P), ctypes.byref(Q))
    return P.value, Q.value


def conv2d_fwd(x, w, stride=1, pad=0, dilation=1) -> np.ndarray:
    """Cross-correlation y = x * w with zero padding; x NCHW, w KCRS -> y NKPQ."""
    x, w = _f64(x), _f64(w)
    d = _dims(x.shape, w.shape, stride, pad, dilation)
    P, Q = conv2d_out_dims(x.shape, w.shape, stride, pad, dilation)
    y = np.empty((x.shape[0], w.shape[0], P, Q), dtype=np.float64)
    _load().oracle_conv2d_fwd(_dp(x), _dp(w), _dp(y), _ip(d))
    return y


def conv2d_dgrad(dy, w, xshape, stride=1, pad=0, dilation=1, into: Optional[np.ndarray] = None) -> np.ndarray:
    """Gradient of <conv(x,w),dy> with respect to x.  `into` (float64, x-shaped) is added to."""
    dy, w = _f64(dy), _f64(w)
    d = _dims(xshape, w.shape, stride, pad, dilation)
    P, Q = conv2d_out_dims(xshape, w.shape, stride, pad, dilation)
    if dy.shape != (d[0], d[4], P, Q):
        raise ValueError(f"dy shape {dy.shape} != {(d[0], d[4], P, Q)}")
    if into is None:
        dx = np.empty(tuple(int(v) for v in xshape), dtype=np.float64)
        acc = 0
    else:
        dx = into
        assert dx.dtype == np.float64 and dx.flags.c_contiguous and dx.shape == tuple(xshape)
        acc = 1
    _load().oracle_conv2d_dgrad(_dp(dy), _dp(w), _dp(dx), _ip(d), acc)
    return dx


def conv2d_wgrad(x, dy, wshape, stride=1, pad=0, dilation=1, into: Optional[np.ndarray] = None) -> np.ndarray:
    """Gradient of <conv(x,w),dy> with respect to w.  `into` (float64, w-shaped) is added to."""
    x, dy = _f64(x), _f64(dy)
    d = _dims(x.shape, wshape, stride, pad, dilation)
    P, Q = conv2d_out_dims(x.shape, wshape, stride, pad, dilation)
    if dy.shape != (d[0], d[4], P, Q):
        raise ValueError(f"dy shape {dy.shape} != {(d[0], d[4], P, Q)}")
    if into is None:
        dw = np.empty(tuple(int(v) for v in wshape), dtype=np.float64)
        acc = 0
    else:
        dw = into
        assert dw.dtype == np.float64 and dw.flags.c_contiguous and dw.shape == tuple(wshape)
        acc = 1
    _load().oracle_conv2d_wgrad(_dp(x), _dp(dy), _dp(dw), _ip(d), acc)
    return dw


# Grouped convolution (not in the paper's workloads; the definition is the textbook one): the C input channels and the
# K output channels are split into `groups` equal runs, output run g sees input run g only, and w is [K][C/groups][R][S].
# Written as exactly that: a loop over the groups around the plain functions above.

def conv2d_grouped_fwd(x, w, groups, stride=1, pad=0, dilation=1) -> np.ndarray:
    x, w = _f64(x), _f64(w)
    C, K = x.shape[1], w.shape[0]
    if C % groups or K % groups or w.shape[1] != C // groups:
        raise ValueError("channel counts do not split into the groups")
    cg, kg = C // groups, K // groups
    return np.concatenate([conv2d_fwd(x[:, g * cg:(g + 1) * cg], w[g * kg:(g + 1) * kg], stride, pad, dilation)
                           for g in range(groups)], axis=1)


def conv2d_grouped_dgrad(dy, w, xshape, groups, stride=1, pad=0, dilation=1, into: Optional[np.ndarray] = None) -> np.ndarray:
    dy, w = _f64(dy), _f64(w)
    N, C, H, W = (int(v) for v in xshape)
    K = w.shape[0]
    cg, kg = C // groups, K // groups
    parts = [conv2d_dgrad(dy[:, g * kg:(g + 1) * kg], w[g * kg:(g + 1) * kg], (N, cg, H, W), stride, pad, dilation)
             for g in range(groups)]
    dx = np.concatenate(parts, axis=1)
    return dx if into is None else into + dx


def conv2d_grouped_wgrad(x, dy, wshape, groups, stride=1, pad=0, dilation=1, into: Optional[np.ndarray] = None) -> np.ndarray:
    x, dy = _f64(x), _f64(dy)
    K, cgw, R, S = (int(v) for v in wshape)
    C = x.shape[1]
    cg, kg = C // groups, K // groups
    assert cgw == cg
    parts = [conv2d_wgrad(x[:, g * cg:(g + 1) * cg], dy[:, g * kg:(g + 1) * kg], (kg, cg, R, S), stride, pad, dilation)
             for g in range(groups)]
    dw = np.concatenate(parts, axis=0)
    return dw if into is None else into + dw


def _coords(coords, ndim_hi) -> np.ndarray:
    c = np.ascontiguousarray(coords, dtype=np.int32)
    if c.ndim != 2 or c.shape[1] != 4:
        raise ValueError("coords must be [count, 4]")
    hi = np.asarray(ndim_hi)
    if c.size and (c.min() < 0 or (c >= hi[None, :]).any()):
        raise ValueError("coordinate out of range")
    return c


def conv2d_fwd_at(x, w, coords, stride=1, pad=0, dilation=1) -> np.ndarray:
    """y at the listed (n,k,p,q) coordinates only."""
    x, w = _f64(x), _f64(w)
    d = _dims(x.shape, w.shape, stride, pad, dilation)
    P, Q = conv2d_out_dims(x.shape, w.shape, stride, pad, dilation)
    c = _coords(coords, (d[0], d[4], P, Q))
    out = np.empty(c.shape[0], dtype=np.float64)
    _load().oracle_conv2d_fwd_at(_dp(x), _dp(w), _ip(d), c.shape[0], _ip(c), _dp(out))
    return out


def conv2d_dgrad_at(dy, w, xshape, coords, stride=1, pad=0, dilation=1) -> np.ndarray:
    """dx at the listed (n,c,h,w) coordinates only."""
    dy, w = _f64(dy), _f64(w)
    d = _dims(xshape, w.shape, stride, pad, dilation)
    P, Q = conv2d_out_dims(xshape, w.shape, stride, pad, dilation)
    if dy.shape != (d[0], d[4], P, Q):
        raise ValueError(f"dy shape {dy.shape} != {(d[0], d[4], P, Q)}")
    c = _coords(coords, tuple(xshape))
    out = np.empty(c.shape[0], dtype=np.float64)
    _load().oracle_conv2d_dgrad_at(_dp(dy), _dp(w), _ip(d), c.shape[0], _ip(c), _dp(out))
    return out


def conv2d_wgrad_at(x, dy, wshape, coords, stride=1, pad=0, dilation=1) -> np.ndarray:
    """dw at the listed (k,c,r,s) coordinates only."""
    x, dy = _f64(x), _f64(dy)
    d = _dims(x.shape, wshape, stride, pad, dilation)
    P, Q = conv2d_out_dims(x.shape, wshape, stride, pad, dilation)
    if dy.shape != (d[0], d[4], P, Q):
        raise ValueError(f"dy shape {dy.shape} != {(d[0], d[4], P, Q)}")
    c = _coords(coords, tuple(wshape))
    out = np.empty(c.shape[0], dtype=np.float64)
    _load().oracle_conv2d_wgrad_at(_dp(x), _dp(dy), _ip(d), c.shape[0], _ip(c), _dp(out))
    return out


def bn_relu_add_fwd(x, gamma, beta, residual=None, eps=1e-5, relu=True, momentum=0.1,
                    running_mean: Optional[np.ndarray] = None, running_var: Optional[np.ndarray] = None):
    """Returns (out, save_mean, save_invstd).  running_* (float64 [C]) are updated in place."""
    x = _f64(x)
    N, C, H, W = x.shape
    gamma, beta = _f64(gamma), _f64(beta)
    assert gamma.shape == (C,) and beta.shape == (C,)
    res = None if residual is None else _f64(residual)
    if res is not None and res.shape != x.shape:
        raise ValueError("residual shape differs from x")
    for r in (running_mean, running_var):
        if r is not None:
            assert r.dtype == np.float64 and r.shape == (C,) and r.flags.c_contiguous
    out = np.empty_like(x)
    mean = np.empty(C, dtype=np.float64)
    invstd = np.empty(C, dtype=np.float64)
    _load().oracle_bn_relu_add_fwd(_dp(x), _dp(res), _dp(gamma), _dp(beta), _dp(out), _dp(mean),
                                   _dp(invstd), _dp(running_mean), _dp(running_var),
                                   N, C, H, W, float(eps), float(momentum), int(bool(relu)))
    return out, mean, invstd


def bn_relu_add_bwd(x, out, dout, gamma, save_mean, save_invstd, relu=True, want_dresidual=False):
    """Returns (dx, dresidual or None, dgamma, dbeta)."""
    x, out, dout = _f64(x), _f64(out), _f64(dout)
    N, C, H, W = x.shape
    assert out.shape == x.shape and dout.shape == x.shape
    gamma, save_mean, save_invstd = _f64(gamma), _f64(save_mean), _f64(save_invstd)
    dx = np.empty_like(x)
    dres = np.empty_like(x) if want_dresidual else None
    dgamma = np.empty(C, dtype=np.float64)
    dbeta = np.empty(C, dtype=np.float64)
    _load().oracle_bn_relu_add_bwd(_dp(x), _dp(out), _dp(dout), _dp(gamma), _dp(save_mean),
                                   _dp(save_invstd), _dp(dx), _dp(dres), _dp(dgamma), _dp(dbeta),
                                   N, C, H, W, int(bool(relu)))
    return dx, dres, dgamma, dbeta


def maxpool2d_fwd(x, window=3, stride=2, pad=1):
    """Returns (y, idx) with idx int8 = r*S+s of the first maximum of each window."""
    x = _f64(x)
    N, C, H, W = x.shape
    R, S = _pair(window)
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    P, Q = conv2d_out_dims((N, C, H, W), (1, C, R, S), (sh, sw), (ph, pw), 1)
    y = np.empty((N, C, P, Q), dtype=np.float64)
    idx = np.empty((N, C, P, Q), dtype=np.int8)
    _load().oracle_maxpool2d_fwd(_dp(x), _dp(y), idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int8)),
                                 N, C, H, W, R, S, sh, sw, ph, pw)
    return y, idx


def maxpool2d_bwd(dy, idx, xshape, window=3, stride=2, pad=1):
    dy = _f64(dy)
    idx = np.ascontiguousarray(idx, dtype=np.int8)
    N, C, H, W = (int(v) for v in xshape)
    R, S = _pair(window)
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    assert dy.shape == idx.shape
    dx = np.empty((N, C, H, W), dtype=np.float64)
    _load().oracle_maxpool2d_bwd(_dp(dy), idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int8)), _dp(dx),
                                 N, C, H, W, R, S, sh, sw, ph, pw)
    return dx


def round_bf16(a) -> np.ndarray:
    """Nearest bfloat16 (ties to even) of every element, as float64."""
    a = _f64(a)
    out = np.empty_like(a)
    _load().oracle_round_bf16(_dp(a), _dp(out), a.size)
    return out
