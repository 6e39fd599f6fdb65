"""A whole training step on one GPU: the residual blocks of a workload (GpuNetwork), the head of the ResNet recipe
(global average pool, fully connected layer), the loss node and the optimizer update.

Sequencing and buffer management only: every arithmetic step is a libnsk entry point.  The step follows the order
the paper gives (section "Automatic Differentiation"): forward in program order up to a loss, then backward in
reverse with gradients accumulated where a tensor feeds several units, then the optimizer, which also clears the
parameter gradients (section "Caching and Pooling").  Parameters are kept as float master copies; for bf16 workloads
the kernels read a bf16 copy that the optimizer call rewrites.  With `group_streams` every parameter group (filters,
batch-norm scales and shifts, classifier) is updated on a stream of its own (section "Operation Overlapping").
All buffers are created in the constructor; a step allocates nothing.
"""
from __future__ import annotations

import contextlib
from typing import Dict, List, Optional

import numpy as np
import torch

from . import binding as B
from .network import GpuNetwork


class GpuTrainer:
    def __init__(self, net: GpuNetwork, fc_w: np.ndarray, fc_b: np.ndarray, labels: np.ndarray, lr: float = 0.1,
                 momentum: float = 0.9, weight_decay: float = 1e-4, optimizer: str = "sgd", clip: Optional[float] = None,
                 group_streams: bool = False):
        self.net, self.lr, self.momentum, self.wd, self.optimizer, self.clip = net, lr, momentum, weight_decay, optimizer, clip
        dev, dt = net.device, net.dtype
        out = net.wl["output"]
        self.N, self.C, self.H, self.W = net.shapes[out]
        self.K = int(fc_w.shape[0])
        f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)
        self.labels = torch.from_numpy(np.ascontiguousarray(labels, dtype=np.int32)).to(dev)
        self.pooled = torch.empty((self.N, self.C), dtype=dt, device=dev)
        self.dpooled = torch.empty_like(self.pooled)
        self.logits = torch.empty((self.N, self.K), dtype=dt, device=dev)
        self.dlogits = torch.empty_like(self.logits)
        self.per_sample = torch.empty((self.N,), dtype=torch.float32, device=dev)
        self.loss = torch.empty((1,), dtype=torch.float32, device=dev)
        self.fc_w_master, self.fc_b = f32(fc_w), f32(fc_b)
        self.fc_w = self.fc_w_master.to(dt)
        self.fc_dw = torch.zeros_like(self.fc_w_master)
        self.fc_db = torch.zeros_like(self.fc_b)
        self.ws = B.Workspace(dev)
        # parameter groups: (master, gradient, low-precision copy or None), each with its optimizer state
        lp = dt == torch.bfloat16
        self.groups: Dict[str, List[tuple]] = {"filters": [], "bn": [], "classifier": []}
        self.master: Dict[str, torch.Tensor] = {}
        for name, w in net.w.items():
            self.master[name] = w.to(torch.float32) if lp else w     # fp32 workloads: the kernels read the master itself
            self.groups["filters"].append((self.master[name], net.dw[name], w if lp else None, True))
        for name in net.gamma:
            self.groups["bn"].append((net.gamma[name], net.dgamma[name], None, False))
            self.groups["bn"].append((net.beta[name], net.dbeta[name], None, False))
        self.groups["classifier"].append((self.fc_w_master, self.fc_dw, self.fc_w if lp else None, True))
        self.groups["classifier"].append((self.fc_b, self.fc_db, None, False))
        self.state = {id(p[0]): [torch.zeros_like(p[0]) for _ in range(2 if optimizer == "adamw" else 1)]
                      for g in self.groups.values() for p in g}
        # one launch table per parameter group
        self.tables = {gname: B.param_table((m, g, self.state[id(m)][0], self.state[id(m)][1] if optimizer == "adamw" else None,
                                             lpc, self.wd if decay else 0.0)   # the recipe decays filters and classifier weights only
                                            for (m, g, lpc, decay) in params)
                       for gname, params in self.groups.items()}
        self.t = 0
        self.streams = {g: torch.cuda.Stream(device=dev) for g in self.groups} if group_streams else None
        self.partials = torch.empty((B.NSK_SUMSQ_PARTIALS,), dtype=torch.float32, device=dev)
        self.sumsq = torch.empty((1,), dtype=torch.float32, device=dev)
        self.scale = torch.empty((1,), dtype=torch.float32, device=dev)
        self._lp = lp

    def forward(self):
        net = self.net
        net.forward()
        B.global_avgpool_fwd(net.act[net.wl["output"]], net.layout, out=self.pooled)
        B.linear_fwd(self.pooled, self.fc_w if self._lp else self.fc_w_master, self.fc_b, out=self.logits, ws=self.ws)
        B.softmax_xent_fwd(self.logits, self.labels, per_sample=self.per_sample, loss=self.loss)

    def backward(self):
        net = self.net
        w = self.fc_w if self._lp else self.fc_w_master
        B.softmax_xent_bwd(self.logits, self.labels, 1.0, out=self.dlogits)
        B.linear_wgrad(self.pooled, self.dlogits, dw=self.fc_dw, db=self.fc_db, ws=self.ws)
        B.linear_dgrad(self.dlogits, w, out=self.dpooled, ws=self.ws)
        B.global_avgpool_bwd(self.dpooled, (self.N, self.C, self.H, self.W), net.layout, out=net.grad[net.wl["output"]])
        net.backward()

    def update(self):
        self.t += 1
        scale = None
        if self.clip is not None:
            scale = B.clip_scale([p[1] for g in self.groups.values() for p in g], self.clip, self.partials, self.sumsq,
                                 self.scale)
        main = torch.cuda.current_stream(self.net.device)
        for gname, params in self.groups.items():
            if not params:
                continue
            st = self.streams[gname] if self.streams else None
            if st is not None:
                st.wait_stream(main)
            with torch.cuda.stream(st) if st is not None else contextlib.nullcontext():
                if self.optimizer == "adamw":
                    B.adamw_step_multi(self.tables[gname], self.t, self.lr, grad_scale=scale)
                else:
                    B.sgd_momentum_step_multi(self.tables[gname], self.lr, self.momentum, grad_scale=scale)
            if st is not None:
                main.wait_stream(st)

    def step(self):
        self.forward()
        self.backward()
        self.update()

