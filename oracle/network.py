"""Oracle execution of a whole workload (forward, then backward) from the primitive oracle ops.

TEST INFRASTRUCTURE ONLY (see the package docstring).  A workload is a flat list of units,
each one assignment in the sense of the paper's section "Automatic Differentiation": the
forward pass runs them in order and records what backward needs; the backward pass walks
the list in reverse, and a tensor that feeds several units has its gradients ACCUMULATED
(first contribution overwrites, later ones add), which is the rule that section states for
the right operand of `y = x@w + x` and that section "Caching and Pooling" states for
weight gradients.

`grid` is applied to every activation-sized tensor at the point where the GPU library
would store it in its storage type: identity for fp32 workloads (the oracle stays fp64),
round-to-bf16 for bf16 workloads.  Reduction outputs (dw, dgamma, dbeta, mean, invstd)
are never rounded.
"""
from __future__ import annotations

from typing import Callable, Dict

import numpy as np

import oracle


def _identity(a):
    return a


def storage_grid(dtype: str) -> Callable[[np.ndarray], np.ndarray]:
    return oracle.round_bf16 if dtype == "bf16" else _identity


def forward(wl: dict, x: np.ndarray, params: Dict[str, dict], eps: float = 1e-5) -> dict:
    """Runs all units in order.  Returns dict(act=..., saved=...) with every named activation."""
    grid = storage_grid(wl["dtype"])
    act = {"x": np.asarray(x, dtype=np.float64)}
    saved = {}
    for u in wl["units"]:
        src = act[u["src"]]
        if u["kind"] == "pool":
            y, idx = oracle.maxpool2d_fwd(src, 3, 2, 1)
            act[u["dst"]] = y
            saved[u["name"]] = dict(idx=idx)
            continue
        p = params[u["name"]]
        y = grid(oracle.conv2d_fwd(src, p["w"], u["stride"], u["pad"], 1))
        if u["kind"] == "conv":
            act[u["dst"]] = y
            continue
        res = act[u["res"]] if u["res"] else None
        out, mean, invstd = oracle.bn_relu_add_fwd(y, p["gamma"], p["beta"], res, eps, relu=u["relu"])
        act[u["dst"]] = grid(out)
        saved[u["name"]] = dict(y=y, mean=mean, invstd=invstd)
    return dict(act=act, saved=saved)


def backward(wl: dict, fwd: dict, params: Dict[str, dict], dout: np.ndarray) -> dict:
    """Walks the units in reverse from the gradient of the workload's output.

    Returns dict(grad=<activation gradients by tensor name>, dw=, dgamma=, dbeta= by unit name,
    trace=<per unit: the tensors each backward step consumed and produced, for per-step parity>).
    """
    grid = storage_grid(wl["dtype"])
    act, saved = fwd["act"], fwd["saved"]
    grad: Dict[str, np.ndarray] = {wl["output"]: np.asarray(dout, dtype=np.float64)}
    dw, dgamma, dbeta, trace = {}, {}, {}, {}

    def send(name, g_unrounded):
        # the storage rounding happens after the add, as one store of the accumulated value
        grad[name] = grid(grad[name] + g_unrounded) if name in grad else grid(g_unrounded)
        return grad[name]

    for u in reversed(wl["units"]):
        g = grad[u["dst"]]
        src = act[u["src"]]
        tr = trace[u["name"]] = dict(g_in=g, src_grad_before=grad.get(u["src"]))
        if u["kind"] == "pool":
            tr["src_grad_after"] = send(u["src"], oracle.maxpool2d_bwd(g, saved[u["name"]]["idx"], src.shape, 3, 2, 1))
            continue
        p = params[u["name"]]
        if u["kind"] == "conv_bn":
            s = saved[u["name"]]
            dy, dres, dg, db = oracle.bn_relu_add_bwd(s["y"], act[u["dst"]], g, p["gamma"], s["mean"],
                                                      s["invstd"], relu=u["relu"],
                                                      want_dresidual=u["res"] is not None)
            dgamma[u["name"]], dbeta[u["name"]] = dg, db
            dy = grid(dy)
            if u["res"]:
                tr["dres"] = send(u["res"], dres)
                if u["res"] == u["src"]:
                    tr["src_grad_before"] = tr["dres"]
        else:
            dy = g
        tr["dy"] = dy
        dw[u["name"]] = oracle.conv2d_wgrad(src, dy, p["w"].shape, u["stride"], u["pad"], 1)
        tr["src_grad_after"] = send(u["src"], oracle.conv2d_dgrad(dy, p["w"], src.shape, u["stride"], u["pad"], 1))
    return dict(grad=grad, dw=dw, dgamma=dgamma, dbeta=dbeta, trace=trace)
