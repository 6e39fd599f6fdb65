"""Seeded synthetic inputs shared by the oracle tests, the GPU parity tests and the bench.

Holds no arithmetic of the method: only counter-based random tensors (numpy's Philox
bit generator keyed by (seed, tensor_id)) with the shapes and value distributions of the
paper's small-image and large-image residual-network workloads (section "Experiments and
Discussion": CIFAR-10-sized 3x32x32 and ImageNet-sized 3x224x224 inputs, ResNet recipe).
All tensors are produced as float32 in NCHW / KCRS index order so the values do not
depend on which layout a consumer later permutes them into.
"""
from __future__ import annotations

from typing import Sequence

import numpy as np


def _gen(seed: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed) & (2**64 - 1), int(tensor_id)]))


def normal(seed: int, tensor_id: int, shape: Sequence[int], std: float = 1.0) -> np.ndarray:
    """N(0, std^2) float32 tensor."""
    a = _gen(seed, tensor_id).standard_normal(size=tuple(shape), dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def uniform(seed: int, tensor_id: int, shape: Sequence[int]) -> np.ndarray:
    """U[0,1) float32 tensor (pixel-like inputs)."""
    return _gen(seed, tensor_id).random(size=tuple(shape), dtype=np.float32)


def he_normal(seed: int, tensor_id: int, wshape: Sequence[int]) -> np.ndarray:
    """Filter [K,C,R,S] ~ N(0, 2/(C*R*S)) (He initialisation, fan-in mode)."""
    K, C, R, S = wshape
    return normal(seed, tensor_id, wshape, std=float(np.sqrt(2.0 / (C * R * S))))


def to_bf16_grid(a: np.ndarray) -> np.ndarray:
    """Round a float32 array to the nearest bfloat16 (ties to even), kept as float32.

    Bit manipulation only, so the inputs handed to the oracle and to the GPU are the
    same numbers.  Not finite values pass through unchanged.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    out = r.astype(np.uint32).view(np.float32).reshape(a.shape)
    bad = ~np.isfinite(a)
    if bad.any():
        out = out.copy()
        out[bad] = a[bad]
    return out


def sample_coords(seed: int, tensor_id: int, shape: Sequence[int], count: int,
                  with_corners: bool = True) -> np.ndarray:
    """`count` random 4-D coordinates inside `shape` (int32 [count,4]), plus all 16 corners."""
    g = _gen(seed, tensor_id)
    cols = [g.integers(0, int(s), size=count, dtype=np.int64) for s in shape]
    c = np.stack(cols, axis=1)
    if with_corners:
        corners = np.array([[(0 if (b >> i) & 1 == 0 else int(shape[i]) - 1) for i in range(4)]
                            for b in range(16)], dtype=np.int64)
        c = np.concatenate([corners, c], axis=0)
    return c.astype(np.int32)


# --------------------------------------------------------------------------------------
# Workload recipes: the five configurations as flat lists of units (pure data).
#
# A unit is one "assignment" in the paper's sense (section "Automatic Differentiation"):
# forward runs the list in order, backward runs it in reverse and ACCUMULATES into the
# gradient of every tensor that already received one.  Unit kinds:
#   conv     dst = conv(src, w)                                    (no batch-norm)
#   conv_bn  dst = relu?( bn(conv(src, w)) [+ res] )
#   pool     dst = maxpool3x3 stride 2 pad 1 (src)
# --------------------------------------------------------------------------------------

def _conv(name, src, dst, C, K, R, stride, pad, bn=True, relu=True, res=None):
    return dict(kind="conv_bn" if bn else "conv", name=name, src=src, dst=dst, C=C, K=K, R=R, S=R,
                stride=stride, pad=pad, relu=relu, res=res)


def _basic_block(units, name, src, dst, C, K, stride):
    """[3x3 -> BN -> ReLU -> 3x3 -> BN] + shortcut -> ReLU; 1x1 stride-s projection + BN when the shape changes."""
    mid = name + ".a"
    units.append(_conv(name + ".c1", src, mid, C, K, 3, stride, 1))
    res = src
    if stride != 1 or C != K:
        res = name + ".sc"
        units.append(_conv(name + ".proj", src, res, C, K, 1, stride, 0, relu=False))
    units.append(_conv(name + ".c2", mid, dst, K, K, 3, 1, 1, relu=True, res=res))


def _bottleneck_block(units, name, src, dst, C, mid_c, K, stride):
    """1x1 C->mid, 3x3 mid->mid (carries the stride), 1x1 mid->K, each with BN; shortcut added before the last ReLU."""
    a, b = name + ".a", name + ".b"
    units.append(_conv(name + ".c1", src, a, C, mid_c, 1, 1, 0))
    units.append(_conv(name + ".c2", a, b, mid_c, mid_c, 3, stride, 1))
    res = src
    if stride != 1 or C != K:
        res = name + ".sc"
        units.append(_conv(name + ".proj", src, res, C, K, 1, stride, 0, relu=False))
    units.append(_conv(name + ".c3", b, dst, mid_c, K, 1, 1, 0, relu=True, res=res))


def workload(config: int, batch: int | None = None, stage: str = "A") -> dict:
    """Recipe for configuration 1..5 (config 5 has two independent stages "A" and "B").

    Returns dict(name, dtype, seed, input=(N,C,H,W), input_dist, units=[...]).  `batch`
    overrides N (used by parity tests that run the full oracle chain at a reduced batch).
    """
    units: list = []
    if config == 1:
        N, shape, dtype, seed, dist = 8, (16, 32, 32), "f32", 1001, "normal"
        units.append(_conv("conv", "x", "y", 16, 16, 3, 1, 1, bn=False))
    elif config == 2:
        N, shape, dtype, seed, dist = 128, (64, 32, 32), "f32", 1002, "normal"
        _basic_block(units, "b1", "x", "y", 64, 64, 1)
    elif config == 3:
        N, shape, dtype, seed, dist = 256, (3, 32, 32), "bf16", 1003, "uniform"
        units.append(_conv("stem", "x", "s0", 3, 16, 3, 1, 1))
        src, C = "s0", 16
        for si, K in enumerate((16, 32, 64)):
            for bi in range(2):
                dst = f"s{si + 1}b{bi + 1}"
                _basic_block(units, dst, src, dst, C, K, 2 if (bi == 0 and K != C) else 1)
                src, C = dst, K
    elif config == 4:
        N, shape, dtype, seed, dist = 64, (3, 224, 224), "bf16", 1004, "normal"
        units.append(_conv("stem", "x", "s0", 3, 64, 7, 2, 3))
        units.append(dict(kind="pool", name="pool", src="s0", dst="p0", C=64))
        _basic_block(units, "b1", "p0", "b1", 64, 64, 1)
        _basic_block(units, "b2", "b1", "b2", 64, 64, 1)
    elif config == 5:
        dtype, dist = "bf16", "normal"
        if stage == "A":
            N, shape, seed, C = 128, (128, 112, 112), 1005, 256
        elif stage == "B":
            N, shape, seed, C = 128, (512, 28, 28), 1006, 1024
        else:
            raise ValueError("stage must be 'A' or 'B'")
        _bottleneck_block(units, "down", "x", "d", C // 2, C // 4, C, 2)
        _bottleneck_block(units, "ident", "d", "y", C, C // 4, C, 1)
    else:
        raise ValueError("config must be 1..5")
    if batch is not None:
        N = int(batch)
    name = f"config{config}" + (f"-stage{stage}" if config == 5 else "")
    return dict(name=name, config=config, dtype=dtype, seed=seed, input=(N,) + shape, input_dist=dist,
                units=units, output=units[-1]["dst"])


def tensor_shapes(wl: dict) -> dict:
    """Shape (N,C,H,W) of every activation tensor of a workload, by name (integer bookkeeping only)."""
    shapes = {"x": tuple(wl["input"])}
    for u in wl["units"]:
        N, C, H, W = shapes[u["src"]]
        if u["kind"] == "pool":
            shapes[u["dst"]] = (N, C, (H + 2 - 3) // 2 + 1, (W + 2 - 3) // 2 + 1)
        else:
            P = (H + 2 * u["pad"] - u["R"]) // u["stride"] + 1
            Q = (W + 2 * u["pad"] - u["S"]) // u["stride"] + 1
            shapes[u["dst"]] = (N, u["K"], P, Q)
    return shapes


def workload_tensors(wl: dict) -> dict:
    """Seeded float32 tensors of a workload: input x, upstream gradient dout, and per unit the filter
    w (He-normal) and batch-norm gamma = 1, beta = 0.  bf16 workloads are rounded onto the bf16 grid
    (filters and activations; gamma/beta stay float32)."""
    seed = wl["seed"]
    shapes = tensor_shapes(wl)
    x = (uniform if wl["input_dist"] == "uniform" else normal)(seed, 0, wl["input"])
    dout = normal(seed, 1, shapes[wl["output"]])
    params = {}
    for i, u in enumerate(wl["units"]):
        if u["kind"] == "pool":
            continue
        w = he_normal(seed, 100 + i, (u["K"], u["C"], u["R"], u["S"]))
        if wl["dtype"] == "bf16":
            w = to_bf16_grid(w)
        params[u["name"]] = dict(w=w, gamma=np.ones(u["K"], np.float32), beta=np.zeros(u["K"], np.float32))
    if wl["dtype"] == "bf16":
        x, dout = to_bf16_grid(x), to_bf16_grid(dout)
    return dict(x=x, dout=dout, params=params)
