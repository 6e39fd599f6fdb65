"""Issues the libnsk call sequence of a whole workload (forward, then backward) on one GPU.

Sequencing and buffer management only: every arithmetic step is a libnsk entry point.  A workload
is the flat unit list of ``nsk_inputs.workload``; forward walks it in order, backward in reverse,
and a tensor that feeds several units gets its gradient contributions ACCUMULATED -- the first
writer overwrites, later ones pass accumulate=1 (the paper's rule for the right operand of
``y = x@w + x``, section "Automatic Differentiation").  All buffers, descriptors and the
workspace are created once in the constructor, so running a step allocates nothing (section
"Caching and Pooling") and the step can be captured into a HIP graph.

Operation overlapping (the paper's section of that name): a weight gradient depends only on tensors
that already exist when its backward-data twin starts, and nothing in the same step reads it.  With
a second stream given to ``backward``/``step`` the backward-weight calls are issued there (with
their own workspace), each after an event that marks its inputs ready, and the main stream joins
the side stream at the end of the step.  Results are bitwise identical either way.  Measured on
MI355X the step is not faster (+-3%): every convolution kernel already holds all CUs with one
LDS-filling block each, so the second stream's kernels mostly queue behind them.
"""
from __future__ import annotations

import ctypes
from typing import Dict, List

import numpy as np
import torch

import nsk_inputs
from . import binding as B


def _to_device(a: np.ndarray, dtype, layout, device, is_filter=False):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if layout == B.NSK_NHWC:
        t = t.permute(0, 2, 3, 1)          # NCHW -> NHWC, KCRS -> KRSC
    return t.contiguous().to(device=device, dtype=dtype)


class GpuNetwork:
    def __init__(self, wl: dict, tensors: dict, layout: int = B.NSK_NHWC, device: str = "cuda:0", eps: float = 1e-5,
                 use_relu_mask: bool = True, use_fused_stats: bool = True, use_fused_act: bool = False):
        self.wl, self.layout, self.device = wl, layout, torch.device(device)
        self.dtype = torch.bfloat16 if wl["dtype"] == "bf16" else torch.float32
        self.code = B.NSK_BF16 if wl["dtype"] == "bf16" else B.NSK_F32
        self.shapes = nsk_inputs.tensor_shapes(wl)
        L = B.lib()
        dev, dt = self.device, self.dtype

        def act_buf(name):
            N, C, H, W = self.shapes[name]
            return torch.empty(B._act_shape(N, C, H, W, layout), dtype=dt, device=dev)

        self.act: Dict[str, torch.Tensor] = {n: act_buf(n) for n in self.shapes}
        self.grad: Dict[str, torch.Tensor] = {n: act_buf(n) for n in self.shapes}
        self.act["x"].copy_(_to_device(tensors["x"], dt, layout, dev))
        self.grad[wl["output"]].copy_(_to_device(tensors["dout"], dt, layout, dev))
        self.w, self.gamma, self.beta = {}, {}, {}
        self.dw, self.dgamma, self.dbeta = {}, {}, {}
        self.y, self.dy, self.mean, self.invstd, self.idx, self.mask, self.stats = {}, {}, {}, {}, {}, {}, {}
        ws_bytes = 0
        self.fwd_calls: List[tuple] = []
        self.bwd_calls: List[tuple] = []
        self._keep = []          # descriptors must outlive the call lists
        ptr = lambda t: ctypes.c_void_p(t.data_ptr()) if t is not None else None

        fwd_plan, bwd_plan = [], []
        written = {wl["output"]}
        # use_fused_act: a conv + batch-norm + ReLU (no residual) whose result feeds exactly one convolution never
        # stores its normalised activation; the consumer applies it to the raw convolution output on load
        # (nsk_conv2d_fwd_act / nsk_conv2d_wgrad_act) and the batch-norm's backward pass takes its mask from there too.
        # fused_away[tensor name] = name of the unit that would have produced it.
        self.fused_away: Dict[str, str] = {}
        self.coeffs: Dict[str, torch.Tensor] = {}
        if use_fused_act and use_fused_stats and layout == B.NSK_NHWC:
            for u in wl["units"]:
                if u["kind"] != "conv_bn" or not u["relu"] or u["res"] or u["dst"] == wl["output"]:
                    continue
                readers = [v for v in wl["units"] if v["src"] == u["dst"]]
                as_res = [v for v in wl["units"] if v.get("res") == u["dst"]]
                if len(readers) != 1 or as_res or readers[0]["kind"] not in ("conv", "conv_bn"):
                    continue
                v = readers[0]
                vd = B.conv_desc(self.shapes[v["src"]], (v["K"], v["R"], v["S"]), v["stride"], v["pad"], 1, self.code, layout)
                if L.nsk_conv2d_act_supported(ctypes.byref(vd)):
                    self.fused_away[u["dst"]] = u["name"]
        for u in wl["units"]:
            name = u["name"]
            N, C, H, W = self.shapes[u["src"]]
            if u["kind"] == "pool":
                d = B.nsk_pool_desc_t(N, C, H, W, 3, 3, 2, 2, 1, 1, self.code, layout)
                self._keep.append(d)
                self.idx[name] = torch.empty(self.act[u["dst"]].shape, dtype=torch.int8, device=dev)
                fwd_plan.append((L.nsk_maxpool2d_fwd, (ctypes.byref(d), ptr(self.act[u["src"]]), ptr(self.act[u["dst"]]),
                                                       ptr(self.idx[name])), None))
                continue
            p = tensors["params"][name]
            K, R, S = u["K"], u["R"], u["S"]
            self.w[name] = _to_device(p["w"], dt, layout, dev, True)
            self.dw[name] = torch.zeros_like(self.w[name], dtype=torch.float32)
            cd = B.conv_desc((N, C, H, W), (K, R, S), u["stride"], u["pad"], 1, self.code, layout)
            self._keep.append(cd)
            for ps in (B.NSK_PASS_FWD, B.NSK_PASS_DGRAD, B.NSK_PASS_WGRAD):
                ws_bytes = max(ws_bytes, L.nsk_conv2d_workspace_bytes(ctypes.byref(cd), ps))
            producer = self.fused_away.get(u["src"])     # the unit whose activation this convolution applies on load
            if producer:
                for ps in (B.NSK_PASS_FWD, B.NSK_PASS_WGRAD):
                    ws_bytes = max(ws_bytes, L.nsk_conv2d_act_workspace_bytes(ctypes.byref(cd), ps))
            if u["kind"] == "conv":
                if producer:
                    fwd_plan.append((L.nsk_conv2d_fwd_act, (ctypes.byref(cd), ptr(self.y[producer]), ptr(self.coeffs[producer]),
                                                            ptr(self.w[name]), ptr(self.act[u["dst"]]), None), "ws"))
                else:
                    fwd_plan.append((L.nsk_conv2d_fwd, (ctypes.byref(cd), ptr(self.act[u["src"]]), ptr(self.w[name]),
                                                        ptr(self.act[u["dst"]])), "ws"))
                continue
            self.gamma[name] = torch.from_numpy(np.asarray(p["gamma"], np.float32)).to(dev)
            self.beta[name] = torch.from_numpy(np.asarray(p["beta"], np.float32)).to(dev)
            self.dgamma[name] = torch.zeros(K, dtype=torch.float32, device=dev)
            self.dbeta[name] = torch.zeros(K, dtype=torch.float32, device=dev)
            self.mean[name] = torch.zeros(K, dtype=torch.float32, device=dev)
            self.invstd[name] = torch.zeros(K, dtype=torch.float32, device=dev)
            self.y[name] = torch.empty_like(self.act[u["dst"]])
            self.dy[name] = torch.empty_like(self.act[u["dst"]])
            Nn, Kk, P, Q = self.shapes[u["dst"]]
            bd = B.nsk_bn_desc_t(Nn, Kk, P, Q, self.code, layout, eps, 0.1, int(u["relu"]))
            self._keep.append(bd)
            ws_bytes = max(ws_bytes, L.nsk_bn_workspace_bytes(ctypes.byref(bd), B.NSK_BN_FWD),
                           L.nsk_bn_workspace_bytes(ctypes.byref(bd), B.NSK_BN_BWD))
            res = self.act[u["res"]] if u["res"] else None
            # where the library offers it, the ReLU mask goes from forward to backward as one byte per vector and
            # the backward pass never reads the normalised activation
            mb = int(L.nsk_bn_mask_bytes(ctypes.byref(bd))) if use_relu_mask else 0
            if mb:
                self.mask[name] = torch.empty(mb, dtype=torch.uint8, device=dev)
            if use_fused_stats:
                # the convolution leaves per-channel partial sums of its output; the batch-norm takes its statistics
                # from them instead of reading the activation once more
                rows = int(L.nsk_conv2d_stats_rows(ctypes.byref(cd)))
                self.stats[name] = torch.empty((2, rows, K), dtype=torch.float32, device=dev)
                if producer:
                    fwd_plan.append((L.nsk_conv2d_fwd_act, (ctypes.byref(cd), ptr(self.y[producer]), ptr(self.coeffs[producer]),
                                                            ptr(self.w[name]), ptr(self.y[name]), ptr(self.stats[name])), "ws"))
                else:
                    fwd_plan.append((L.nsk_conv2d_fwd_stats, (ctypes.byref(cd), ptr(self.act[u["src"]]), ptr(self.w[name]),
                                                              ptr(self.y[name]), ptr(self.stats[name])), "ws"))
                if u["dst"] in self.fused_away:
                    # statistics and coefficients only: the consumer applies the activation
                    self.coeffs[name] = torch.empty((2, K), dtype=torch.float32, device=dev)
                    fwd_plan.append((L.nsk_bn_fwd_coeffs, (ctypes.byref(bd), ptr(self.gamma[name]), ptr(self.beta[name]),
                                                           ptr(self.stats[name]), rows, ptr(self.mean[name]),
                                                           ptr(self.invstd[name]), None, None, ptr(self.coeffs[name])), "ws"))
                    continue
                fwd_plan.append((L.nsk_bn_relu_add_fwd_stats, (ctypes.byref(bd), ptr(self.y[name]), ptr(res),
                                                               ptr(self.gamma[name]), ptr(self.beta[name]),
                                                               ptr(self.act[u["dst"]]), ptr(self.mask.get(name)),
                                                               ptr(self.mean[name]), ptr(self.invstd[name]), None, None,
                                                               ptr(self.stats[name]), rows), "ws"))
                continue
            fwd_plan.append((L.nsk_conv2d_fwd, (ctypes.byref(cd), ptr(self.act[u["src"]]), ptr(self.w[name]),
                                                ptr(self.y[name])), "ws"))
            if mb:
                fwd_plan.append((L.nsk_bn_relu_add_fwd_mask, (ctypes.byref(bd), ptr(self.y[name]), ptr(res),
                                                              ptr(self.gamma[name]), ptr(self.beta[name]),
                                                              ptr(self.act[u["dst"]]), ptr(self.mask[name]),
                                                              ptr(self.mean[name]), ptr(self.invstd[name]), None, None), "ws"))
            else:
                fwd_plan.append((L.nsk_bn_relu_add_fwd, (ctypes.byref(bd), ptr(self.y[name]), ptr(res), ptr(self.gamma[name]),
                                                         ptr(self.beta[name]), ptr(self.act[u["dst"]]), ptr(self.mean[name]),
                                                         ptr(self.invstd[name]), None, None), "ws"))

        # backward: reverse walk; first contribution to a gradient overwrites, later ones accumulate
        for u in reversed(wl["units"]):
            name = u["name"]
            N, C, H, W = self.shapes[u["src"]]
            g_dst = self.grad[u["dst"]]
            if u["kind"] == "pool":
                assert u["src"] not in written
                d = B.nsk_pool_desc_t(N, C, H, W, 3, 3, 2, 2, 1, 1, self.code, layout)
                self._keep.append(d)
                bwd_plan.append((L.nsk_maxpool2d_bwd, (ctypes.byref(d), ptr(g_dst), ptr(self.idx[name]),
                                                       ptr(self.grad[u["src"]])), None))
                written.add(u["src"])
                continue
            K, R, S = u["K"], u["R"], u["S"]
            cd = B.conv_desc((N, C, H, W), (K, R, S), u["stride"], u["pad"], 1, self.code, layout)
            self._keep.append(cd)
            if u["kind"] == "conv_bn":
                Nn, Kk, P, Q = self.shapes[u["dst"]]
                bd = B.nsk_bn_desc_t(Nn, Kk, P, Q, self.code, layout, eps, 0.1, int(u["relu"]))
                self._keep.append(bd)
                dres = None
                if u["res"]:
                    assert u["res"] not in written, "residual gradient must be the first contribution"
                    dres = self.grad[u["res"]]
                    written.add(u["res"])
                if u["dst"] in self.fused_away:
                    bwd_plan.append((L.nsk_bn_relu_bwd_act, (ctypes.byref(bd), ptr(self.y[name]), ptr(self.coeffs[name]),
                                                             ptr(g_dst), ptr(self.gamma[name]), ptr(self.mean[name]),
                                                             ptr(self.invstd[name]), ptr(self.dy[name]),
                                                             ptr(self.dgamma[name]), ptr(self.dbeta[name])), "ws"))
                elif name in self.mask:
                    bwd_plan.append((L.nsk_bn_relu_add_bwd_mask, (ctypes.byref(bd), ptr(self.y[name]), ptr(self.mask[name]),
                                                                  ptr(g_dst), ptr(self.gamma[name]), ptr(self.mean[name]),
                                                                  ptr(self.invstd[name]), ptr(self.dy[name]), ptr(dres),
                                                                  ptr(self.dgamma[name]), ptr(self.dbeta[name])), "ws"))
                else:
                    bwd_plan.append((L.nsk_bn_relu_add_bwd, (ctypes.byref(bd), ptr(self.y[name]), ptr(self.act[u["dst"]]),
                                                             ptr(g_dst), ptr(self.gamma[name]), ptr(self.mean[name]),
                                                             ptr(self.invstd[name]), ptr(self.dy[name]), ptr(dres),
                                                             ptr(self.dgamma[name]), ptr(self.dbeta[name])), "ws"))
                dy = self.dy[name]
            else:
                dy = g_dst
            producer = self.fused_away.get(u["src"])
            if producer:
                bwd_plan.append((L.nsk_conv2d_wgrad_act, (ctypes.byref(cd), ptr(self.y[producer]), ptr(self.coeffs[producer]),
                                                          ptr(dy), ptr(self.dw[name]), 0), "side"))
            else:
                bwd_plan.append((L.nsk_conv2d_wgrad, (ctypes.byref(cd), ptr(self.act[u["src"]]), ptr(dy), ptr(self.dw[name]), 0),
                                 "side"))
            acc = 1 if u["src"] in written else 0
            bwd_plan.append((L.nsk_conv2d_dgrad, (ctypes.byref(cd), ptr(dy), ptr(self.w[name]), ptr(self.grad[u["src"]]),
                                                  acc), "ws"))
            written.add(u["src"])

        # two workspaces: calls issued on the side stream must not share scratch with the main stream's
        self.ws = torch.empty(max(int(ws_bytes), 256), dtype=torch.uint8, device=dev)
        self.ws_side = torch.empty(max(int(ws_bytes), 256), dtype=torch.uint8, device=dev)
        wsp, wsb = ctypes.c_void_p(self.ws.data_ptr()), ctypes.c_size_t(self.ws.numel())
        wsp2 = ctypes.c_void_p(self.ws_side.data_ptr())
        fin = lambda plan: [(f, a + ((wsp2 if w == "side" else wsp, wsb) if w else ())) for f, a, w in plan]
        self.fwd_calls, self.bwd_calls = fin(fwd_plan), fin(bwd_plan)
        self.bwd_side = [w == "side" for _, _, w in bwd_plan]   # calls that may run on a side stream

    def _run(self, calls, side_flags=None, side_stream=None):
        main = torch.cuda.current_stream(self.device)
        st = ctypes.c_void_p(main.cuda_stream)
        st2 = ctypes.c_void_p(side_stream.cuda_stream) if side_stream is not None else None
        used_side = False
        for i, (f, args) in enumerate(calls):
            if st2 is not None and side_flags[i]:
                side_stream.wait_stream(main)      # inputs of this call are ready once the main stream gets here
                rc = f(*args, st2)
                used_side = True
            else:
                rc = f(*args, st)
            if rc != B.NSK_OK:
                raise B.NskError(rc, f.__name__)
        if used_side:
            main.wait_stream(side_stream)

    def forward(self):
        self._run(self.fwd_calls)

    def backward(self, side_stream=None):
        self._run(self.bwd_calls, self.bwd_side, side_stream)

    def step(self, side_stream=None):
        self._run(self.fwd_calls)
        self._run(self.bwd_calls, self.bwd_side, side_stream)

    # ---- results back on the host in the oracle's index order (NCHW / KCRS, float64)
    def host(self, t: torch.Tensor) -> np.ndarray:
        a = t.detach().to(torch.float32).cpu()
        if self.layout == B.NSK_NHWC and a.dim() == 4:
            a = a.permute(0, 3, 1, 2)
        return a.contiguous().numpy().astype(np.float64)
