"""The recurrent workload on one GPU: embedding -> one GRU layer -> output layer on the last state -> cross entropy,
backward through time, gradient clip and AdamW (the recipe of the paper's section "Experiments and Discussion").

Sequencing and buffer management only: every arithmetic step is a libnsk entry point.  The input products of all time
steps are one matrix product (x @ W_ih over T*N rows); each step then costs one product (h @ W_hh) and one fused gate
kernel, and in the backward pass one gate kernel and one product (dgh @ W_hh, by the backward-data form of the `@`
operator); the four weight and bias gradients and the gradient of the embedded input are again single products over
all T*N rows.  All buffers are created in the constructor; a step allocates nothing and can be captured into a HIP
graph.
"""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B


class GpuGruClassifier:
    def __init__(self, tokens: np.ndarray, labels: np.ndarray, table, w_ih, w_hh, b_ih, b_hh, w_out, b_out,
                 dtype: str = "f32", lr: float = 1e-3, weight_decay: float = 1e-4, clip: Optional[float] = 5.0,
                 device: str = "cuda:0"):
        dev = torch.device(device)
        self.dt = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.T, self.N = tokens.shape                       # time-major: tokens[t][n]
        self.V, self.E = table.shape
        self.H = w_hh.shape[1]
        self.K = w_out.shape[0]
        self.lr, self.wd, self.clip = lr, weight_decay, clip
        T, N, E, H, K, dt = self.T, self.N, self.E, self.H, self.K, self.dt
        f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)
        self.tokens = torch.from_numpy(np.ascontiguousarray(tokens.reshape(-1), dtype=np.int32)).to(dev)
        self.labels = torch.from_numpy(np.ascontiguousarray(labels, dtype=np.int32)).to(dev)
        # float masters; the kernels read copies in the storage type (the masters themselves for fp32)
        self.master = {"table": f32(table), "w_ih": f32(w_ih), "w_hh": f32(w_hh), "b_ih": f32(b_ih), "b_hh": f32(b_hh),
                       "w_out": f32(w_out), "b_out": f32(b_out)}
        lp = dt == torch.bfloat16
        self.w = {k: (v.to(dt) if lp and k in ("table", "w_ih", "w_hh", "w_out") else v) for k, v in self.master.items()}
        self.grad = {k: torch.zeros_like(v) for k, v in self.master.items()}
        # W_hh^T, refreshed after every update: the backward step kernel reads a hidden unit's column of W_hh as a row of
        # it (and so does the unfused path's recurrent product, through the backward-data form of the `@` operator)
        self.w_hh_t = torch.empty((self.H, 3 * self.H), dtype=dt, device=dev)
        B.transpose2d(self.w["w_hh"], out=self.w_hh_t)
        z = lambda *s: torch.zeros(s, dtype=dt, device=dev)
        self.x = z(T * N, E)
        self.gi = z(T * N, 3 * H)
        self.gh = z(N, 3 * H)
        self.h = z(T + 1, N, H)                             # h[0] is the zero initial state
        self.saved = z(T, N, 4 * H)
        self.logits, self.dlogits = z(N, K), z(N, K)
        self.per_sample = torch.zeros(N, dtype=torch.float32, device=dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        self.dh_top = z(N, H)
        self.dgi, self.dgh = z(T * N, 3 * H), z(T * N, 3 * H)
        self.dh_direct, self.dh_rec = [z(N, H), z(N, H)], [z(N, H), z(N, H)]
        self.dx = z(T * N, E)
        self.ws = B.Workspace(dev)
        order = ["table", "w_ih", "w_hh", "w_out", "b_ih", "b_hh", "b_out"]
        self.m = {k: torch.zeros_like(self.master[k]) for k in order}
        self.v = {k: torch.zeros_like(self.master[k]) for k in order}
        decay = {"table": weight_decay, "w_ih": weight_decay, "w_hh": weight_decay, "w_out": weight_decay}
        self.table_rec = B.param_table((self.master[k], self.grad[k], self.m[k], self.v[k],
                                        self.w[k] if lp and k in ("table", "w_ih", "w_hh", "w_out") else None,
                                        decay.get(k, 0.0)) for k in order)
        self.order = order
        self.partials = torch.empty(B.NSK_SUMSQ_PARTIALS, dtype=torch.float32, device=dev)
        self.sumsq = torch.empty(1, dtype=torch.float32, device=dev)
        self.scale = torch.empty(1, dtype=torch.float32, device=dev)
        self.t = 0
        self.fused_steps = B.gru_step_supported(N, H)

    def forward(self):
        T, N, H, w = self.T, self.N, self.H, self.w
        B.embedding_fwd(self.tokens, w["table"], out=self.x)
        B.linear_fwd(self.x, w["w_ih"], None, out=self.gi, ws=self.ws)
        gi = self.gi.view(T, N, 3 * H)
        for t in range(T):
            if self.fused_steps:
                B.gru_step_fwd(gi[t], w["w_hh"], w["b_ih"], w["b_hh"], self.h[t], h_new=self.h[t + 1], saved=self.saved[t])
                continue
            B.linear_dgrad(self.h[t], self.w_hh_t, out=self.gh, ws=self.ws)      # h @ W_hh (see w_hh_t)
            B.gru_gates_fwd(gi[t], self.gh, w["b_ih"], w["b_hh"], self.h[t], h_new=self.h[t + 1], saved=self.saved[t])
        B.linear_fwd(self.h[T], w["w_out"], w["b_out"], out=self.logits, ws=self.ws)
        B.softmax_xent_fwd(self.logits, self.labels, per_sample=self.per_sample, loss=self.loss)

    def backward(self):
        T, N, H, w, g = self.T, self.N, self.H, self.w, self.grad
        B.softmax_xent_bwd(self.logits, self.labels, 1.0, out=self.dlogits)
        B.linear_wgrad(self.h[T], self.dlogits, dw=g["w_out"], db=g["b_out"], ws=self.ws)
        B.linear_dgrad(self.dlogits, w["w_out"], out=self.dh_top, ws=self.ws)
        dgi, dgh = self.dgi.view(T, N, 3 * H), self.dgh.view(T, N, 3 * H)
        for t in reversed(range(T)):
            p = t & 1
            if self.fused_steps:
                last = t == T - 1
                B.gru_step_bwd(self.saved[t], self.h[t], self.w_hh_t, dh_a=self.dh_top if last else None,
                               dh_direct_next=None if last else self.dh_direct[p ^ 1], dgh_next=None if last else dgh[t + 1],
                               dgi=dgi[t], dgh=dgh[t], dh_direct=self.dh_direct[p])
                continue
            if t == T - 1:
                B.gru_gates_bwd(self.saved[t], self.h[t], self.dh_top, dgi=dgi[t], dgh=dgh[t], dh_direct=self.dh_direct[p])
            else:                                            # the two parts of the gradient the step after this one left
                B.gru_gates_bwd(self.saved[t], self.h[t], self.dh_direct[p ^ 1], self.dh_rec[p ^ 1], dgi=dgi[t], dgh=dgh[t],
                                dh_direct=self.dh_direct[p])
            if t > 0:
                B.linear_dgrad(dgh[t], w["w_hh"], out=self.dh_rec[p], ws=self.ws)
        hs = self.h[:T].view(T * N, H)
        B.linear_wgrad(self.x, self.dgi, dw=g["w_ih"], db=g["b_ih"], ws=self.ws)
        B.linear_wgrad(hs, self.dgh, dw=g["w_hh"], db=g["b_hh"], ws=self.ws)
        B.linear_dgrad(self.dgi, w["w_ih"], out=self.dx, ws=self.ws)
        B.embedding_bwd(self.tokens, self.dx, self.V, dtable=g["table"])

    def update(self):
        self.t += 1
        scale = None
        if self.clip is not None:
            scale = B.clip_scale([self.grad[k] for k in self.order], self.clip, self.partials, self.sumsq, self.scale)
        B.adamw_step_multi(self.table_rec, self.t, self.lr, grad_scale=scale)
        B.transpose2d(self.w["w_hh"], out=self.w_hh_t)

    def step(self):
        self.forward()
        self.backward()
        self.update()
