"""Pins the oracle's workload executor (unit list forward + reverse walk with gradient
accumulation, section "Automatic Differentiation") against torch CPU float64 autograd and
central finite differences on tiny residual blocks."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import nsk_inputs as gen
import oracle
from oracle import network as onet


def _tiny(kind):
    units = []
    if kind == "basic":
        gen._basic_block(units, "b1", "x", "y", 4, 4, 1)
        shape = (2, 4, 6, 6)
    elif kind == "basic_down":
        gen._basic_block(units, "b1", "x", "m", 4, 6, 2)
        gen._basic_block(units, "b2", "m", "y", 6, 6, 1)
        shape = (2, 4, 8, 6)
    elif kind == "bottleneck":
        gen._bottleneck_block(units, "d", "x", "m", 4, 2, 8, 2)
        gen._bottleneck_block(units, "i", "m", "y", 8, 2, 8, 1)
        shape = (2, 4, 8, 8)
    elif kind == "stem_pool":
        units.append(gen._conv("stem", "x", "s0", 3, 4, 7, 2, 3))
        units.append(dict(kind="pool", name="pool", src="s0", dst="p0", C=4))
        gen._basic_block(units, "b1", "p0", "y", 4, 4, 1)
        shape = (2, 3, 18, 18)
    elif kind == "conv_only":
        units.append(gen._conv("conv", "x", "y", 3, 5, 3, 1, 1, bn=False))
        shape = (2, 3, 6, 7)
    wl = dict(name=kind, config=0, dtype="f32", seed=77, input=shape, input_dist="normal",
              units=units, output=units[-1]["dst"])
    t = gen.workload_tensors(wl)
    for i, (name, p) in enumerate(t["params"].items()):      # non-trivial affine parameters
        p["gamma"] = (1.0 + 0.3 * gen.normal(78, i, p["gamma"].shape)).astype(np.float64)
        p["beta"] = (0.2 * gen.normal(79, i, p["beta"].shape)).astype(np.float64)
        p["w"] = p["w"].astype(np.float64)
    return wl, t


def _torch_run(wl, t):
    leaves = {"x": torch.from_numpy(t["x"].astype(np.float64)).requires_grad_(True)}
    P = {n: {k: torch.from_numpy(np.asarray(v, dtype=np.float64)).requires_grad_(True) for k, v in p.items()}
         for n, p in t["params"].items()}
    act = dict(leaves)
    for u in wl["units"]:
        s = act[u["src"]]
        if u["kind"] == "pool":
            act[u["dst"]] = F.max_pool2d(s, 3, 2, 1)
            continue
        p = P[u["name"]]
        y = F.conv2d(s, p["w"], None, u["stride"], u["pad"])
        if u["kind"] == "conv_bn":
            y = F.batch_norm(y, None, None, p["gamma"], p["beta"], training=True, eps=1e-5)
            if u["res"]:
                y = y + act[u["res"]]
            if u["relu"]:
                y = torch.relu(y)
        act[u["dst"]] = y
    out = act[wl["output"]]
    out.backward(torch.from_numpy(t["dout"].astype(np.float64)))
    return out.detach().numpy(), leaves["x"].grad.numpy(), P


@pytest.mark.parametrize("kind", ["conv_only", "basic", "basic_down", "bottleneck", "stem_pool"])
def test_network_matches_torch_autograd(kind):
    wl, t = _tiny(kind)
    f = onet.forward(wl, t["x"], t["params"])
    b = onet.backward(wl, f, t["params"], t["dout"])
    out, dx, P = _torch_run(wl, t)
    np.testing.assert_allclose(f["act"][wl["output"]], out, rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(b["grad"]["x"], dx, rtol=1e-9, atol=1e-9)
    for u in wl["units"]:
        if u["kind"] == "pool":
            continue
        np.testing.assert_allclose(b["dw"][u["name"]], P[u["name"]]["w"].grad.numpy(), rtol=1e-9, atol=1e-9)
        if u["kind"] == "conv_bn":
            np.testing.assert_allclose(b["dgamma"][u["name"]], P[u["name"]]["gamma"].grad.numpy(), rtol=1e-9, atol=1e-9)
            np.testing.assert_allclose(b["dbeta"][u["name"]], P[u["name"]]["beta"].grad.numpy(), rtol=1e-9, atol=1e-9)


def test_block_central_differences():
    wl, t = _tiny("basic")
    x = t["x"].astype(np.float64)
    dout = t["dout"].astype(np.float64)

    def loss(xv, params):
        return np.vdot(onet.forward(wl, xv, params)["act"]["y"], dout)

    f = onet.forward(wl, x, t["params"])
    b = onet.backward(wl, f, t["params"], dout)
    h = 1e-6
    rng = np.random.default_rng(3)
    for _ in range(6):
        j = tuple(rng.integers(0, s) for s in x.shape)
        e = np.zeros_like(x)
        e[j] = h
        fd = (loss(x + e, t["params"]) - loss(x - e, t["params"])) / (2 * h)
        assert abs(fd - b["grad"]["x"][j]) < 2e-5 * max(1.0, abs(fd))
    w = t["params"]["b1.c1"]["w"]
    for _ in range(6):
        j = tuple(rng.integers(0, s) for s in w.shape)
        e = np.zeros_like(w)
        e[j] = h
        hi = {**t["params"], "b1.c1": {**t["params"]["b1.c1"], "w": w + e}}
        lo = {**t["params"], "b1.c1": {**t["params"]["b1.c1"], "w": w - e}}
        fd = (loss(x, hi) - loss(x, lo)) / (2 * h)
        assert abs(fd - b["dw"]["b1.c1"][j]) < 2e-5 * max(1.0, abs(fd))


def test_bf16_grid_is_applied_to_stored_activations():
    wl, t = _tiny("basic")
    wl = dict(wl, dtype="bf16")
    f = onet.forward(wl, gen.to_bf16_grid(t["x"]), t["params"])
    y = f["act"]["y"]
    assert np.array_equal(y, oracle.round_bf16(y))
    b = onet.backward(wl, f, t["params"], gen.to_bf16_grid(t["dout"]))
    assert np.array_equal(b["grad"]["x"], oracle.round_bf16(b["grad"]["x"]))


def test_recipes_have_the_configured_shapes():
    sh = gen.tensor_shapes(gen.workload(3))
    assert sh["s0"] == (256, 16, 32, 32) and sh["s2b1"] == (256, 32, 16, 16) and sh["s3b2"] == (256, 64, 8, 8)
    sh = gen.tensor_shapes(gen.workload(4))
    assert sh["s0"] == (64, 64, 112, 112) and sh["p0"] == (64, 64, 56, 56) and sh["b2"] == (64, 64, 56, 56)
    sh = gen.tensor_shapes(gen.workload(5, stage="A"))
    assert sh["down.a"] == (128, 64, 112, 112) and sh["y"] == (128, 256, 56, 56)
    sh = gen.tensor_shapes(gen.workload(5, stage="B"))
    assert sh["down.b"] == (128, 256, 14, 14) and sh["y"] == (128, 1024, 14, 14)
