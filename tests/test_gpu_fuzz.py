"""Seeded sweep over random small convolution problems (both types and layouts, strides 1-3 per axis, padding 0-3,
dilation 1-2, square and non-square filters, channel counts that select every kernel family), each run forward,
backward-data (overwrite and accumulate) and backward-weight (overwrite and accumulate) against the oracle.  The
size thresholds of the special kernels are lowered through their test hooks in four of the five groups, so that the
small problems the fp64 oracle can afford reach the large-tile, short-reduction, merged-class and wide-halo code
paths in shapes no hand-written case lists."""
import numpy as np
import pytest
import torch

import nsk_inputs as gen
import oracle
from paper_2409_11600_amd import binding as B
from parity import TOL, guarded, max_rel_err, on_grid, to_gpu, to_host, torch_dtype

pytestmark = pytest.mark.gpu

CHANNELS = [3, 8, 16, 24, 32, 40, 64, 64, 128, 256]
HOOKS = [
    {},
    {"NSK_PW_MIN_ROWS": "1"},
    {"NSK_BIG_MIN_TILES": "1", "NSK_WIDE_MIN_ROWS": "1"},
    {"NSK_PW_MIN_ROWS": "1", "NSK_BIG_MIN_TILES": "1", "NSK_WIDE_MIN_ROWS": "1", "NSK_STATS_ALWAYS": "1"},
    {"NSK_HALO_WIDE_ALWAYS": "1"},       # with channel counts the wide halo kernel takes (64, 128, 256 in; multiples of 64 out)
]
WIDE_HALO_GROUP = 4
CASES_PER_GROUP = 120


def _draw(rng, wide_halo=False):
    while True:
        C, K = (int(rng.choice(CHANNELS)) for _ in range(2))
        R, S = (int(rng.choice([1, 1, 2, 3, 3, 3, 5])) for _ in range(2))
        if wide_halo:     # both passes reach the kernel: C and K from its channel counts, mostly filters with taps within one pixel
            C, K = (int(rng.choice([64, 128, 128, 192, 256])) for _ in range(2))
            R, S = (int(rng.choice([2, 3, 3, 3, 4, 5])) for _ in range(2))
        if rng.random() < 0.7:
            S = R
        sh, sw = (int(rng.choice([1, 1, 1, 2, 2, 3])) for _ in range(2))
        if rng.random() < 0.7:
            sw = sh
        ph, pw = int(rng.integers(0, 1 + R // 2 + 1)), int(rng.integers(0, 1 + S // 2 + 1))
        dh, dw = (int(rng.choice([1, 1, 1, 2])) for _ in range(2))
        N = int(rng.integers(1, 5))
        H, W = int(rng.integers(4, 19)), int(rng.integers(4, 19))
        if C * K >= 128 * 128:
            N, H, W = min(N, 2), min(H, 10), min(W, 10)
        P = (H + 2 * ph - dh * (R - 1) - 1) // sh + 1
        Q = (W + 2 * pw - dw * (S - 1) - 1) // sw + 1
        if P >= 1 and Q >= 1:
            return (N, C, H, W, K, R, S, (sh, sw), (ph, pw), (dh, dw))


@pytest.mark.parametrize("group", range(len(HOOKS)))
def test_random_convolutions_match_the_oracle(group, nsk_env):
    for k, v in HOOKS[group].items():
        nsk_env(k, v)
    rng = np.random.default_rng(4200 + group)
    ws = B.Workspace()
    for case in range(CASES_PER_GROUP):
        N, C, H, W, K, R, S, st, pd, dl = shape = _draw(rng, group == WIDE_HALO_GROUP)
        dtype = "bf16" if rng.random() < 0.65 else "f32"
        layout = B.NSK_NHWC if rng.random() < 0.8 else B.NSK_NCHW
        print(f"fuzz group {group} case {case}: {shape} {dtype} layout={layout} hooks={sorted(HOOKS[group])}", flush=True)
        seed = 5000 + 100 * group + case
        x = on_grid(gen.normal(seed, 0, (N, C, H, W)), dtype)
        w = on_grid(gen.he_normal(seed, 1, (K, C, R, S)), dtype)
        P, Q = oracle.conv2d_out_dims(x.shape, w.shape, st, pd, dl)
        dy = on_grid(gen.normal(seed, 2, (N, K, P, Q)), dtype)
        base = on_grid(gen.normal(seed, 3, x.shape), dtype)
        base_w = gen.normal(seed, 4, w.shape).astype(np.float32)
        tol = TOL[dtype]
        gx, gw, gdy = to_gpu(x, dtype, layout), to_gpu(w, dtype, layout), to_gpu(dy, dtype, layout)
        y_view, y_check = guarded(gdy.shape, torch_dtype(dtype))
        B.conv2d_fwd(gx, gw, st, pd, dl, layout, out=y_view, ws=ws)
        y1, stats = B.conv2d_fwd_stats(gx, gw, st, pd, dl, layout, ws=ws)
        dx_view, dx_check = guarded(gx.shape, torch_dtype(dtype))
        B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, layout, out=dx_view, ws=ws)
        gacc = to_gpu(base, dtype, layout)
        B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, layout, out=gacc, accumulate=True, ws=ws)
        dw_view, dw_check = guarded(gw.shape, torch.float32)
        B.conv2d_wgrad(gx, gdy, w.shape, st, pd, dl, layout, out=dw_view, ws=ws)
        gdw = to_gpu(base_w, "f32", layout)
        B.conv2d_wgrad(gx, gdy, w.shape, st, pd, dl, layout, out=gdw, accumulate=True, ws=ws)
        torch.cuda.synchronize()
        for chk in (y_check, dx_check, dw_check):
            chk()
        yh = to_host(y_view, layout)
        assert max_rel_err(yh, oracle.conv2d_fwd(x, w, st, pd, dl)) <= tol, shape
        assert torch.equal(y_view, y1), shape
        sums = stats.double().sum(dim=1).cpu().numpy()
        want0, want1 = yh.sum(axis=(0, 2, 3)), (yh * yh).sum(axis=(0, 2, 3))
        assert np.max(np.abs(sums[0] - want0) / (np.sqrt(want1 * yh[:, 0].size) + 1e-30)) <= 1e-6, shape
        assert np.max(np.abs(sums[1] - want1) / (want1 + 1e-30)) <= 1e-5, shape
        want_dx = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl)
        got_dx = to_host(dx_view, layout)
        assert max_rel_err(got_dx, want_dx) <= tol, shape
        assert np.all(got_dx[want_dx == 0.0] == 0.0), shape
        assert max_rel_err(to_host(gacc, layout), oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl, into=base.astype(np.float64))) <= tol, shape
        want_dw = oracle.conv2d_wgrad(x, dy, w.shape, st, pd, dl)
        assert max_rel_err(to_host(dw_view, layout), want_dw) <= TOL["f32"] * 10, shape
        assert max_rel_err(to_host(gdw, layout), want_dw + base_w.astype(np.float64)) <= TOL["f32"] * 10, shape


BN_CHANNELS = [3, 5, 8, 16, 24, 40, 64, 128, 256, 1024]


def test_random_batch_norm_problems_match_the_oracle():
    """Random shapes through the fused batch-norm calls (plain and ReLU-mask forms), forward and backward."""
    rng = np.random.default_rng(4300)
    ws = B.Workspace()
    for case in range(80):
        C = int(rng.choice(BN_CHANNELS))
        N, H, W = int(rng.integers(1, 7)), int(rng.integers(1, 20)), int(rng.integers(1, 20))
        if N * H * W < 2:
            N = 2
        dtype = "bf16" if rng.random() < 0.5 else "f32"
        layout = B.NSK_NHWC if rng.random() < 0.75 else B.NSK_NCHW
        relu, with_res = bool(rng.random() < 0.7), bool(rng.random() < 0.5)
        shape = (N, C, H, W)
        print(f"bn fuzz case {case}: {shape} {dtype} layout={layout} relu={relu} res={with_res}", flush=True)
        seed = 6000 + case
        x = on_grid(1.3 * gen.normal(seed, 0, shape) + 0.4, dtype)
        r = on_grid(gen.normal(seed, 1, shape), dtype)
        dout = on_grid(gen.normal(seed, 2, shape), dtype)
        g = (1.0 + 0.3 * gen.normal(seed, 3, (C,))).astype(np.float32)
        b = (0.2 * gen.normal(seed, 4, (C,))).astype(np.float32)
        tol = TOL[dtype]
        gx, gr, gd = to_gpu(x, dtype, layout), to_gpu(r, dtype, layout), to_gpu(dout, dtype, layout)
        gg, gb = torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda()
        out_view, out_check = guarded(gx.shape, torch_dtype(dtype))
        mask = None
        mb = B.bn_mask_bytes(gx, layout, relu) if relu and rng.random() < 0.6 else 0     # the mask hand-over where it applies
        if mb:
            mask = torch.empty(mb, dtype=torch.uint8, device="cuda:0")
        out, mean, invstd = B.bn_relu_add_fwd(gx, gg, gb, gr if with_res else None, 1e-5, relu, layout, out=out_view, ws=ws,
                                              relu_mask=mask)
        torch.cuda.synchronize()
        out_check()
        want_out, want_mean, want_invstd = oracle.bn_relu_add_fwd(x, g, b, r if with_res else None, 1e-5, relu)
        assert max_rel_err(to_host(out, layout), want_out) <= tol, shape
        assert max_rel_err(mean.cpu().numpy(), want_mean) <= 1e-5, shape
        assert max_rel_err(invstd.cpu().numpy(), want_invstd) <= 1e-5, shape
        # backward on the GPU's own stored forward result: both sides take the ReLU mask from the same tensor
        out_h = to_host(out, layout)
        dx, dres, dg, db = B.bn_relu_add_bwd(gx, out, gd, gg, mean, invstd, relu, layout, want_dresidual=with_res, ws=ws,
                                             relu_mask=mask)
        torch.cuda.synchronize()
        wdx, wdres, wdg, wdb = oracle.bn_relu_add_bwd(x, out_h, dout, g, mean.cpu().numpy(), invstd.cpu().numpy(), relu,
                                                      want_dresidual=with_res)
        assert max_rel_err(to_host(dx, layout), wdx) <= tol, shape
        assert max_rel_err(dg.cpu().numpy(), wdg) <= 1e-4, shape
        assert max_rel_err(db.cpu().numpy(), wdb) <= 1e-4, shape
        if with_res:
            assert np.array_equal(to_host(dres, layout), wdres), shape


def test_random_max_pool_problems_match_the_oracle():
    """Random windows (1..4 per axis), strides and paddings, inputs with many tied zeros: values, first-maximum indices
    (bit exact) and the backward scatter."""
    rng = np.random.default_rng(4400)
    for case in range(60):
        R, S = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        sh, sw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        ph, pw = int(rng.integers(0, R // 2 + 1)), int(rng.integers(0, S // 2 + 1))
        if rng.random() < 0.4:
            R, S, sh, sw, ph, pw = 3, 3, 2, 2, 1, 1                      # the recipe's pool
        N, C = int(rng.integers(1, 4)), int(rng.choice([3, 8, 16, 24, 64]))
        H, W = int(rng.integers(R, 23)), int(rng.integers(S, 23))
        if rng.random() < 0.3:
            H, W = H + H % 2, W + W % 2                                  # even extents: the 2x2-block backward kernel
        dtype = "bf16" if rng.random() < 0.5 else "f32"
        layout = B.NSK_NHWC if rng.random() < 0.75 else B.NSK_NCHW
        shape = (N, C, H, W)
        print(f"pool fuzz case {case}: {shape} window {(R, S)} stride {(sh, sw)} pad {(ph, pw)} {dtype} layout={layout}", flush=True)
        x = on_grid(np.maximum(gen.normal(7000 + case, 0, shape), 0.0), dtype)
        y, idx = B.maxpool2d_fwd(to_gpu(x, dtype, layout), (R, S), (sh, sw), (ph, pw), layout)
        wy, widx = oracle.maxpool2d_fwd(x, (R, S), (sh, sw), (ph, pw))
        torch.cuda.synchronize()
        assert np.array_equal(to_host(y, layout), wy), shape
        got_idx = idx.cpu()
        if layout == B.NSK_NHWC:
            got_idx = got_idx.permute(0, 3, 1, 2)
        assert np.array_equal(got_idx.numpy(), widx), shape
        dy = on_grid(gen.normal(7000 + case, 1, wy.shape), dtype)
        dx = B.maxpool2d_bwd(to_gpu(dy, dtype, layout), idx, shape, (R, S), (sh, sw), (ph, pw), layout)
        torch.cuda.synchronize()
        assert max_rel_err(to_host(dx, layout), oracle.maxpool2d_bwd(dy, widx, shape, (R, S), (sh, sw), (ph, pw))) <= TOL[dtype], shape
