"""Whole training steps (residual blocks, average pool, fully connected layer, loss, backward, SGD update) through
libnsk against the same sequence built from the oracle's primitives, on the same seeded tensors."""
import numpy as np
import pytest
import torch

import nsk_inputs as gen
from oracle import network as onet
from oracle import train as T
from paper_2409_11600_amd import binding as B
from paper_2409_11600_amd.network import GpuNetwork
from paper_2409_11600_amd.trainer import GpuTrainer
from parity import max_rel_err

pytestmark = pytest.mark.gpu

LR, MU, WD, CLASSES = 0.05, 0.9, 1e-3, 10


class OracleTrainer:
    """The oracle's training step: forward to the loss, backward, SGD with momentum.  Masters are float64; what the
    kernels would read in a storage type goes through `grid` first."""

    def __init__(self, wl, tensors, fc_w, fc_b, labels):
        self.wl, self.x, self.labels = wl, tensors["x"], labels
        self.grid = onet.storage_grid(wl["dtype"])
        self.master = {n: {k: np.asarray(v, dtype=np.float64) for k, v in p.items()} for n, p in tensors["params"].items()}
        self.fc_w, self.fc_b = fc_w.astype(np.float64), fc_b.astype(np.float64)
        self.vel = {}
        self.losses = []

    def _sgd(self, key, w, g, wd):
        w2, v, _ = T.sgd_momentum_step(w, g, self.vel.get(key, np.zeros_like(w)), LR, MU, wd)
        self.vel[key] = v
        return w2

    def step(self):
        wl, grid = self.wl, self.grid
        params = {n: dict(p, w=grid(p["w"])) for n, p in self.master.items()}
        fwd = onet.forward(wl, self.x, params)
        out = fwd["act"][wl["output"]]
        w_used = grid(self.fc_w)
        pooled = grid(T.global_avgpool_fwd(out))
        logits = grid(T.linear_fwd(pooled, w_used, self.fc_b))
        loss, _ = T.softmax_xent_fwd(logits, self.labels)
        self.losses.append(loss)
        dlogits = grid(T.softmax_xent_bwd(logits, self.labels))
        dw, db = T.linear_wgrad(pooled, dlogits)
        dpooled = grid(T.linear_dgrad(dlogits, w_used))
        dout = grid(T.global_avgpool_bwd(dpooled, out.shape))
        bwd = onet.backward(wl, fwd, params, dout)
        for n, p in self.master.items():
            p["w"] = self._sgd(("w", n), p["w"], bwd["dw"][n], WD)
            if "gamma" in p and n in bwd["dgamma"]:
                p["gamma"] = self._sgd(("g", n), p["gamma"], bwd["dgamma"][n], 0.0)
                p["beta"] = self._sgd(("b", n), p["beta"], bwd["dbeta"][n], 0.0)
        self.fc_w = self._sgd("fcw", self.fc_w, dw, WD)
        self.fc_b = self._sgd("fcb", self.fc_b, db, 0.0)


def _setup(config, batch, stage="A"):
    wl = gen.workload(config, batch=batch, stage=stage)
    t = gen.workload_tensors(wl)
    shapes = gen.tensor_shapes(wl)
    N, C, _, _ = shapes[wl["output"]]
    fc_w = (gen.normal(wl["seed"], 2000, (CLASSES, C)) / np.sqrt(C)).astype(np.float32)
    fc_b = (0.1 * gen.normal(wl["seed"], 2001, (CLASSES,))).astype(np.float32)
    labels = (gen.uniform(wl["seed"], 2002, (N,)) * CLASSES).astype(np.int32) % CLASSES
    return wl, t, fc_w, fc_b, labels


@pytest.mark.parametrize("config,batch,streams", [(1, None, False), (2, 4, True)])
def test_two_fp32_training_steps_match_the_oracle(config, batch, streams):
    wl, t, fc_w, fc_b, labels = _setup(config, batch)
    assert wl["dtype"] == "f32"
    print(f"training steps on {wl['name']} input {wl['input']} group_streams={streams}", flush=True)
    ref = OracleTrainer(wl, t, fc_w, fc_b, labels)
    net = GpuNetwork(wl, t, B.NSK_NHWC)
    tr = GpuTrainer(net, fc_w, fc_b, labels, lr=LR, momentum=MU, weight_decay=WD, group_streams=streams)
    for step in range(2):
        before = {n: net.host(tr.master[n]) for n in net.w}
        before_fc = tr.fc_w_master.cpu().numpy().astype(np.float64)
        ref_before = {n: p["w"].copy() for n, p in ref.master.items()}
        ref_before_fc = ref.fc_w.copy()
        tr.step()
        ref.step()
        torch.cuda.synchronize()
        tol = 1e-4 if step == 0 else 2e-3      # the second step starts from weights that already differ by rounding
        assert abs(float(tr.loss.item()) - ref.losses[-1]) <= tol * abs(ref.losses[-1])
        for n in net.w:                        # compare the UPDATES: the weights themselves barely move in one step
            got = net.host(tr.master[n]) - before[n]
            want = ref.master[n]["w"] - ref_before[n]
            assert max_rel_err(got, want) <= 10 * tol, (n, step)
        got_fc = tr.fc_w_master.cpu().numpy().astype(np.float64) - before_fc
        assert max_rel_err(got_fc, ref.fc_w - ref_before_fc) <= 10 * tol
        assert max_rel_err(tr.fc_b.cpu().numpy(), ref.fc_b) <= 10 * tol
        for n in net.gamma:
            assert max_rel_err(net.gamma[n].cpu().numpy(), ref.master[n]["gamma"]) <= 10 * tol
            assert max_rel_err(net.beta[n].cpu().numpy(), ref.master[n]["beta"]) <= 10 * tol
        assert not tr.fc_dw.any() and all(not g.any() for g in net.dw.values())     # gradients cleared


def test_bf16_training_steps_track_the_oracle_and_reduce_the_loss():
    wl, t, fc_w, fc_b, labels = _setup(3, 8)
    assert wl["dtype"] == "bf16"
    print(f"training steps on {wl['name']} input {wl['input']} (bf16)", flush=True)
    ref = OracleTrainer(wl, t, fc_w, fc_b, labels)
    net = GpuNetwork(wl, t, B.NSK_NHWC)
    tr = GpuTrainer(net, fc_w, fc_b, labels, lr=LR, momentum=MU, weight_decay=WD)
    losses = []
    for step in range(4):
        tr.step()
        torch.cuda.synchronize()
        losses.append(float(tr.loss.item()))
        if step < 2:
            ref.step()
            assert abs(losses[-1] - ref.losses[-1]) <= 2e-2 * abs(ref.losses[-1])
        for n, w in net.w.items():             # the bf16 copy the kernels read is the rounded master
            assert torch.equal(w, tr.master[n].to(torch.bfloat16))
    assert np.all(np.isfinite(losses)) and losses[-1] < losses[0]


def test_adamw_with_gradient_clip_runs_the_recurrent_experiments_recipe():
    """AdamW, learning rate 0.001, weight decay 0.0001, gradient clip 5 (section "Experiments and Discussion") on the
    small fp32 block: first-step updates against the oracle's AdamW with the oracle's clip factor."""
    wl, t, fc_w, fc_b, labels = _setup(1, None)
    net = GpuNetwork(wl, t, B.NSK_NHWC)
    tr = GpuTrainer(net, fc_w, fc_b, labels, lr=1e-3, weight_decay=1e-4, optimizer="adamw", clip=5.0)
    tr.forward()
    tr.backward()
    torch.cuda.synchronize()
    grads = {n: net.host(g) for n, g in net.dw.items()}
    all_grads = [g.cpu().numpy().astype(np.float64) for grp in tr.groups.values() for (_, g, _, _) in grp]
    s = T.clip_scale(all_grads, 5.0)
    before = {n: net.host(tr.master[n]) for n in net.w}
    tr.update()
    torch.cuda.synchronize()
    assert abs(float(tr.scale.item()) - s) <= 1e-5 * s
    for n in net.w:
        want, _, _, _ = T.adamw_step(before[n], grads[n], np.zeros_like(before[n]), np.zeros_like(before[n]), 1, 1e-3,
                                     beta1=float(np.float32(0.9)), beta2=float(np.float32(0.999)), weight_decay=1e-4,
                                     grad_scale=s)
        assert max_rel_err(net.host(tr.master[n]) - before[n], want - before[n]) <= 1e-3


def test_a_captured_training_step_replays_to_the_same_bits_as_eager_steps():
    """The whole step (blocks, head, loss, backward, multi-tensor SGD) captured into a HIP graph: every replay leaves
    exactly the state the same number of eager steps leaves.  Replays are separated by host synchronisations and an
    eager read of the loss, as a training loop would do."""
    def make():
        wl, t, fc_w, fc_b, labels = _setup(3, 8)
        net = GpuNetwork(wl, t, B.NSK_NHWC)
        return GpuTrainer(net, fc_w, fc_b, labels, lr=LR, momentum=MU, weight_decay=WD)

    eager, graphed = make(), make()
    eager_losses, graph_losses = [], []
    for _ in range(5):
        eager.step()
        torch.cuda.synchronize()
        eager_losses.append(float(eager.loss.item()))
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        graphed.step()                       # first step eagerly (sizes the workspaces)
        stream.synchronize()
        graph_losses.append(float(graphed.loss.item()))
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            graphed.step()
        for _ in range(4):
            g.replay()
            stream.synchronize()
            graph_losses.append(float(graphed.loss.item()))
    torch.cuda.synchronize()
    assert graph_losses == eager_losses
    for n in eager.net.w:
        assert torch.equal(eager.master[n], graphed.master[n]) and torch.equal(eager.net.w[n], graphed.net.w[n])
    assert torch.equal(eager.fc_w_master, graphed.fc_w_master) and torch.equal(eager.fc_b, graphed.fc_b)
    for n in eager.net.gamma:
        assert torch.equal(eager.net.gamma[n], graphed.net.gamma[n]) and torch.equal(eager.net.beta[n], graphed.net.beta[n])
