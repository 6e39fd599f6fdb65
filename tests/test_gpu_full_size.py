"""Parity at the FULL configured sizes, in the launch configuration bench.py times (NHWC, the
library's own tile choice): every distinct convolution layer of configurations 2-5 runs forward
(plain and with the statistics epilogue), backward-data (overwriting and accumulating) and
backward-weight on seeded tensors of the configured shape, and EVERY element of y, dx and dw is
compared with the oracle's full evaluation of the definition (so all border rows and all tile
boundaries of every kernel are among the compared elements).  Batch-norm + ReLU + add and max
pooling are compared in full at their largest configured shapes."""
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


def _unreached(H, W, P, Q, R, stride, pad):
    """[H, W] bool: input cells that no filter tap of any output position touches (index logic only)."""
    def axis(n, m):
        hit = np.zeros(n, dtype=bool)
        for o in range(m):
            for r in range(R):
                i = o * stride - pad + r
                if 0 <= i < n:
                    hit[i] = True
        return hit
    return ~(axis(H, P)[:, None] & axis(W, Q)[None, :])


def _full_err(got: torch.Tensor, want: np.ndarray, must_be_zero=None):
    """max_i |got_i - want_i| / max(|want_i|, rms(want)) over a whole NHWC device tensor against the oracle's NCHW
    float64 array, image by image so that the float64 temporaries stay small; also returns the number of nonzero
    elements of `got` among the cells of the [H, W] mask `must_be_zero`."""
    N = want.shape[0]
    rms = max(float(np.sqrt(np.mean(want * want))), 1e-30)
    worst, nonzero_zeros = 0.0, 0
    step = max(1, (1 << 24) // max(1, want[0].size))
    for n0 in range(0, N, step):
        g = got[n0:n0 + step].float().cpu().permute(0, 3, 1, 2).numpy().astype(np.float64)
        w = want[n0:n0 + step]
        assert g.shape == w.shape, (g.shape, w.shape)
        assert np.all(np.isfinite(g))
        worst = max(worst, float(np.max(np.abs(g - w) / np.maximum(np.abs(w), rms))))
        if must_be_zero is not None:
            assert not np.any(w[:, :, must_be_zero])
            nonzero_zeros += int(np.count_nonzero(g[:, :, must_be_zero]))
    return worst, nonzero_zeros


@pytest.mark.parametrize("layer", LAYERS, ids=lambda l: "-".join(str(v) for v in l))
def test_conv_layer_at_full_size(layer):
    dtype, N, C, H, W, K, R, stride, pad = layer
    print(f"full-size conv {layer}", flush=True)
    seed = 3000 + LAYERS.index(layer)
    x = on_grid(gen.normal(seed, 0, (N, C, H, W)), dtype)
    w = on_grid(gen.he_normal(seed, 1, (K, C, R, R)), dtype)
    P, Q = oracle.conv2d_out_dims(x.shape, w.shape, stride, pad, 1)
    dy = on_grid(gen.normal(seed, 2, (N, K, P, Q)), dtype)
    dx0 = on_grid(gen.normal(seed, 3, (N, C, H, W)), dtype)      # what the accumulating backward-data adds to
    dw0 = gen.normal(seed, 4, (K, C, R, R)).astype(np.float32)
    tol = TOL[dtype]
    ws = B.Workspace()
    gx, gw, gdy = to_gpu(x, dtype, B.NSK_NHWC), to_gpu(w, dtype, B.NSK_NHWC), to_gpu(dy, dtype, B.NSK_NHWC)
    gy = B.conv2d_fwd(gx, gw, stride, pad, 1, ws=ws)
    gy_s, stats = B.conv2d_fwd_stats(gx, gw, stride, pad, 1, ws=ws)
    gdx = B.conv2d_dgrad(gdy, gw, x.shape, stride, pad, 1, ws=ws)
    gdx_acc = to_gpu(dx0, dtype, B.NSK_NHWC)
    B.conv2d_dgrad(gdy, gw, x.shape, stride, pad, 1, out=gdx_acc, accumulate=True, ws=ws)
    gdw = B.conv2d_wgrad(gx, gdy, w.shape, stride, pad, 1, ws=ws)
    gdw_acc = to_gpu(dw0, "f32", B.NSK_NHWC)
    B.conv2d_wgrad(gx, gdy, w.shape, stride, pad, 1, out=gdw_acc, accumulate=True, ws=ws)
    torch.cuda.synchronize()

    x64, w64, dy64 = x.astype(np.float64), w.astype(np.float64), dy.astype(np.float64)
    want_y = oracle.conv2d_fwd(x64, w64, stride, pad, 1)
    err, _ = _full_err(gy, want_y)
    print(f"  fwd (all {want_y.size} elements): max rel err {err:.2e}", flush=True)
    assert err <= tol, ("fwd", err)
    # the statistics epilogue must not change y, and its partial sums must be the sums of y as stored
    assert torch.equal(gy, gy_s), "y of nsk_conv2d_fwd_stats differs from nsk_conv2d_fwd"
    rows = stats.shape[1]
    s_got = stats.double().sum(dim=1).cpu().numpy()
    y_stored = gy_s.double().reshape(-1, K)
    s_want = np.stack([y_stored.sum(dim=0).cpu().numpy(), (y_stored * y_stored).sum(dim=0).cpu().numpy()])
    M = N * P * Q
    sigma = np.sqrt(np.maximum(s_want[1] / M, 1e-30))
    # a float partial sum of at most M/rows stored values: error far below 1e-5 of M*sigma (sum) and M*sigma^2 (squares)
    assert np.max(np.abs(s_got[0] - s_want[0]) / (M * sigma)) <= 1e-5, ("stats sum", rows)
    assert np.max(np.abs(s_got[1] - s_want[1]) / (M * sigma * sigma)) <= 1e-5, ("stats sumsq", rows)
    # batch-norm fed by those partial sums against the oracle's batch-norm of the oracle's y (on the storage grid)
    g = (1.0 + 0.3 * gen.normal(seed, 5, (K,))).astype(np.float32)
    b = (0.2 * gen.normal(seed, 6, (K,))).astype(np.float32)
    gg, gb = torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda()
    y_grid = on_grid(want_y.astype(np.float32), dtype)
    want_out, want_mean, want_invstd = oracle.bn_relu_add_fwd(y_grid, g, b, None, 1e-5, True)
    mb = B.bn_mask_bytes(gy_s)
    mask = torch.empty(mb, dtype=torch.uint8, device="cuda") if mb else None
    out, mean, invstd = B.bn_relu_add_fwd(gy_s, gg, gb, None, 1e-5, True, ws=ws, relu_mask=mask, stats=stats)
    torch.cuda.synchronize()
    # the mean is compared on the scale that matters for the normalised value (a shift of the mean by d moves
    # xhat by d*invstd); stored y may differ from the oracle's by one rounding in a few elements
    stat_tol = 1e-5 if dtype == "f32" else 1e-4
    assert np.max(np.abs(mean.cpu().numpy() - want_mean) * want_invstd) <= stat_tol
    assert max_rel_err(invstd.cpu().numpy(), want_invstd) <= stat_tol
    err, _ = _full_err(out, want_out)
    print(f"  bn(relu) from the fused statistics: max rel err {err:.2e} ({rows} rows of partial sums)", flush=True)
    assert err <= tol, ("bn from stats", err)
    del want_y, want_out, y_grid, y_stored

    want_dx = oracle.conv2d_dgrad(dy64, w64, x.shape, stride, pad, 1)
    err, bad_zeros = _full_err(gdx, want_dx, _unreached(H, W, P, Q, R, stride, pad))
    print(f"  dgrad (all {want_dx.size} elements): max rel err {err:.2e}", flush=True)
    assert err <= tol, ("dgrad", err)
    assert bad_zeros == 0, "cells of dx that no tap reaches (strided layers) must be exact zeros"
    want_acc = dx0.astype(np.float64) + want_dx
    err, _ = _full_err(gdx_acc, want_acc)
    print(f"  dgrad accumulate: max rel err {err:.2e}", flush=True)
    assert err <= tol, ("dgrad accumulate", err)
    del want_dx, want_acc

    want_dw = oracle.conv2d_wgrad(x64, dy64, w.shape, stride, pad, 1)
    err = max_rel_err(to_host(gdw, B.NSK_NHWC), want_dw)
    print(f"  wgrad (all {want_dw.size} elements): max rel err {err:.2e}", flush=True)
    assert err <= tol, ("wgrad", err)
    err = max_rel_err(to_host(gdw_acc, B.NSK_NHWC), dw0.astype(np.float64) + want_dw)
    assert err <= tol, ("wgrad accumulate", err)


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
