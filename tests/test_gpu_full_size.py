"""Parity at the FULL configured sizes, in the launch configuration bench.py times (NHWC, the
library's own tile choice): every distinct convolution layer of configurations 2-5 runs forward,
backward-data and backward-weight on seeded tensors of the configured shape, and the results are
compared with the oracle's definition evaluated at sampled output coordinates (each output element is
an independent sum, so this is exact parity for the sampled elements; the 16 corner coordinates are
always among them).  Batch-norm + ReLU + add and max pooling are compared in full at their largest
configured shapes."""
import numpy as np
import pytest
import torch

import nsk_inputs as gen
import oracle
from paper_2409_11600_amd import binding as B
from parity import TOL, max_rel_err, on_grid, to_gpu, to_host

pytestmark = pytest.mark.gpu


def _layers():
    seen, out = set(), []
    for config, stage in ((2, "A"), (3, "A"), (4, "A"), (5, "A"), (5, "B")):
        wl = gen.workload(config, stage=stage)
        shapes = gen.tensor_shapes(wl)
        for u in wl["units"]:
            if u["kind"] == "pool":
                continue
            key = (wl["dtype"],) + shapes[u["src"]] + (u["K"], u["R"], u["stride"], u["pad"])
            if key not in seen:
                seen.add(key)
                out.append(key)
    return out


LAYERS = _layers()


def _rms_floor_err(got, want, ref_rms):
    return float(np.max(np.abs(got - want) / np.maximum(np.abs(want), ref_rms)))


@pytest.mark.parametrize("layer", LAYERS, ids=lambda l: "-".join(str(v) for v in l))
def test_conv_layer_at_full_size(layer):
    dtype, N, C, H, W, K, R, stride, pad = layer
    print(f"full-size conv {layer}", flush=True)
    seed = 3000 + LAYERS.index(layer)
    x = on_grid(gen.normal(seed, 0, (N, C, H, W)), dtype)
    w = on_grid(gen.he_normal(seed, 1, (K, C, R, R)), dtype)
    P, Q = oracle.conv2d_out_dims(x.shape, w.shape, stride, pad, 1)
    dy = on_grid(gen.normal(seed, 2, (N, K, P, Q)), dtype)
    tol = TOL[dtype]
    ws = B.Workspace()
    gx, gw, gdy = to_gpu(x, dtype, B.NSK_NHWC), to_gpu(w, dtype, B.NSK_NHWC), to_gpu(dy, dtype, B.NSK_NHWC)
    gy = B.conv2d_fwd(gx, gw, stride, pad, 1, ws=ws)
    gdx = B.conv2d_dgrad(gdy, gw, x.shape, stride, pad, 1, ws=ws)
    gdw = B.conv2d_wgrad(gx, gdy, w.shape, stride, pad, 1, ws=ws)
    torch.cuda.synchronize()
    # sampled coordinates, gathered on the device (NHWC / KRSC indexing) before the copy to the host
    n_s = 4096 if N * P * Q * K < 5e7 else 2048
    cy = gen.sample_coords(seed, 10, (N, K, P, Q), n_s)
    cx = gen.sample_coords(seed, 11, (N, C, H, W), n_s)
    cw = gen.sample_coords(seed, 12, (K, C, R, R), 256)
    pick = lambda t, c: t[tuple(torch.from_numpy(c[:, i].astype(np.int64)).cuda() for i in (0, 2, 3, 1))].float().cpu().numpy().astype(np.float64)
    got_y, got_dx, got_dw = pick(gy, cy), pick(gdx, cx), pick(gdw, cw)
    x64, w64, dy64 = x.astype(np.float64), w.astype(np.float64), dy.astype(np.float64)
    want_y = oracle.conv2d_fwd_at(x64, w64, cy, stride, pad, 1)
    want_dx = oracle.conv2d_dgrad_at(dy64, w64, x.shape, cx, stride, pad, 1)
    want_dw = oracle.conv2d_wgrad_at(x64, dy64, w.shape, cw, stride, pad, 1)
    # the floor of the relative error is the RMS of the sampled oracle values (a sample of the tensor's RMS)
    for name, got, want in (("fwd", got_y, want_y), ("dgrad", got_dx, want_dx), ("wgrad", got_dw, want_dw)):
        rms = max(float(np.sqrt(np.mean(want * want))), 1e-30)
        err = _rms_floor_err(got, want, rms)
        print(f"  {name}: max rel err {err:.2e}", flush=True)
        assert err <= tol, (name, err)
    # cells of dx that no tap reaches (strided layers) must be exact zeros
    assert np.all(got_dx[want_dx == 0.0] == 0.0)
    # structure checks that hold at any size: finite everywhere, and the adjoint identity
    # <conv(x,w),dy> = <x,dgrad(dy,w)> = <w,wgrad(x,dy)> on the device results (loose: bf16 storage)
    assert bool(torch.isfinite(gy.float()).all()) and bool(torch.isfinite(gdx.float()).all()) and bool(torch.isfinite(gdw).all())
    a = float((gy.double() * gdy.double()).sum())
    b = float((gx.double() * gdx.double()).sum())
    c = float((gw.double() * gdw.double()).sum())
    scale = float(gy.double().norm() * gdy.double().norm())
    assert abs(a - b) <= 2e-2 * scale and abs(a - c) <= 2e-2 * scale, (a, b, c, scale)


BN_FULL = [("f32", 128, 64, 32, 32), ("bf16", 256, 16, 32, 32), ("bf16", 64, 64, 112, 112), ("bf16", 128, 256, 56, 56),
           ("bf16", 128, 1024, 14, 14)]


@pytest.mark.parametrize("case", BN_FULL, ids=lambda c: "-".join(str(v) for v in c))
def test_bn_relu_add_at_full_size(case):
    dtype, N, C, H, W = case
    print(f"full-size bn {case}", flush=True)
    seed = 4000 + BN_FULL.index(case)
    shape = (N, C, H, W)
    x = on_grid(1.3 * gen.normal(seed, 0, shape) + 0.4, dtype)
    r = on_grid(gen.normal(seed, 1, shape), dtype)
    dout = on_grid(gen.normal(seed, 2, shape), dtype)
    g = (1.0 + 0.3 * gen.normal(seed, 3, (C,))).astype(np.float32)
    b = (0.2 * gen.normal(seed, 4, (C,))).astype(np.float32)
    ws = B.Workspace()
    gx, gr, gd = (to_gpu(a, dtype, B.NSK_NHWC) for a in (x, r, dout))
    gg, gb = torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda()
    out, mean, invstd = B.bn_relu_add_fwd(gx, gg, gb, gr, 1e-5, True, ws=ws)
    want_out, want_mean, want_invstd = oracle.bn_relu_add_fwd(x, g, b, r, 1e-5, True)
    tol = TOL[dtype]
    assert max_rel_err(to_host(out, B.NSK_NHWC), want_out) <= tol
    assert max_rel_err(mean.cpu().numpy(), want_mean) <= 1e-5
    assert max_rel_err(invstd.cpu().numpy(), want_invstd) <= 1e-5
    out_grid = on_grid(want_out.astype(np.float32), dtype)
    m32, i32 = want_mean.astype(np.float32), want_invstd.astype(np.float32)
    dx, dres, dg, db = B.bn_relu_add_bwd(gx, to_gpu(out_grid, dtype, B.NSK_NHWC), gd, gg, torch.from_numpy(m32).cuda(),
                                         torch.from_numpy(i32).cuda(), True, want_dresidual=True, ws=ws)
    wdx, wdres, wdg, wdb = oracle.bn_relu_add_bwd(x, out_grid, dout, g, m32, i32, True, want_dresidual=True)
    assert max_rel_err(to_host(dx, B.NSK_NHWC), wdx) <= tol
    assert np.array_equal(to_host(dres, B.NSK_NHWC), wdres)
    assert max_rel_err(dg.cpu().numpy(), wdg) <= 1e-4
    assert max_rel_err(db.cpu().numpy(), wdb) <= 1e-4


def test_maxpool_at_full_size():
    shape = (64, 64, 112, 112)
    x = on_grid(np.maximum(gen.normal(4100, 0, shape), 0.0), "bf16")
    gx = to_gpu(x, "bf16", B.NSK_NHWC)
    y, idx = B.maxpool2d_fwd(gx, 3, 2, 1)
    wy, widx = oracle.maxpool2d_fwd(x, 3, 2, 1)
    assert np.array_equal(to_host(y, B.NSK_NHWC), wy)
    assert np.array_equal(idx.cpu().permute(0, 3, 1, 2).numpy(), widx)
    dy = on_grid(gen.normal(4100, 1, wy.shape), "bf16")
    dx = B.maxpool2d_bwd(to_gpu(dy, "bf16", B.NSK_NHWC), idx, shape, 3, 2, 1)
    assert max_rel_err(to_host(dx, B.NSK_NHWC), oracle.maxpool2d_bwd(dy, widx, shape, 3, 2, 1)) <= TOL["bf16"]
