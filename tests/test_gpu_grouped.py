"""GPU parity of the grouped convolution entry points (nsk_conv2d_grouped_fwd/dgrad/wgrad) against the CPU oracle,
which defines a grouped convolution as a loop over the groups around the plain one."""
import numpy as np
import pytest
import torch

import nsk_inputs as gen
import oracle
from paper_2409_11600_amd import binding as B
from parity import TOL, guarded, max_rel_err, on_grid, to_gpu, to_host, torch_dtype

pytestmark = pytest.mark.gpu

LAYOUTS = [B.NSK_NHWC, B.NSK_NCHW]

# N, C, H, W, K, R, S, stride, pad, dilation, groups
GROUPED_SHAPES = [
    (2, 32, 12, 12, 32, 3, 3, 1, 1, 1, 2),        # two groups of 16 -> 16 (vector loads)
    (2, 64, 9, 11, 128, 3, 3, 1, 1, 1, 4),        # 16 -> 32 per group, odd extents, ragged row tile
    (2, 128, 10, 10, 128, 3, 3, 2, 1, 1, 32),     # the 32-group bottleneck shape: 4 -> 4 per group (scalar loads in bf16)
    (3, 24, 13, 9, 24, 3, 3, 1, 1, 1, 24),        # depthwise
    (2, 16, 12, 12, 32, 3, 3, 2, 1, 1, 16),       # depthwise with channel multiplier 2, stride 2
    (2, 24, 14, 12, 36, 3, 2, (2, 1), (1, 0), (1, 2), 3),   # anisotropic stride, pad, dilation; 8 -> 12 per group
    (1, 40, 9, 9, 20, 1, 1, 1, 0, 1, 5),          # 1x1, 8 -> 4 per group
    (2, 6, 10, 10, 9, 5, 5, 3, 2, 1, 3),          # stride 3 (classes without taps), odd channel counts
    (1, 256, 6, 6, 256, 3, 3, 1, 1, 1, 2),        # 128 -> 128 per group: 128-column tiles, long reduction
    (2, 16, 8, 8, 16, 3, 3, 1, 1, 1, 1),          # one group = the plain call
    (2, 128, 14, 14, 128, 3, 3, 1, 1, 1, 128),    # depthwise, several blocks of the direct kernels
    (1, 256, 9, 7, 256, 5, 5, 2, 2, 1, 256),      # depthwise 5x5 stride 2 (25 taps: three register chunks in backward-weight)
    (2, 40, 11, 13, 40, 3, 3, (2, 1), 1, (1, 2), 40),   # depthwise, anisotropic stride and dilation, 5 or 10 channel vectors
    (1, 16, 12, 12, 16, 7, 7, 1, 3, 1, 16),       # depthwise 7x7 (49 taps)
    (2, 32, 9, 11, 32, 3, 3, 1, 1, 1, 16),        # two channels per group on both sides (direct kernels)
    (1, 64, 10, 8, 64, 5, 5, 1, 2, 1, 16),        # four channels per group, 5x5
    (2, 128, 12, 12, 128, 3, 3, 1, 1, 1, 32),     # the 32-group bottleneck shape at stride 1
    (2, 32, 7, 23, 32, 3, 3, 1, 1, 1, 32),        # depthwise, output rows of 23 pixels (ragged groups of four)
    (1, 16, 9, 10, 16, 5, 3, (2, 1), (2, 1), 1, 16),    # depthwise 5x3, stride 2 down the rows only
    (2, 24, 10, 9, 24, 5, 5, 2, 2, 1, 24),        # depthwise 5x5 stride 2: backward-data classes of 3x3, 3x2, 2x3 and 2x2 taps
    (2, 64, 11, 10, 64, 3, 3, 1, 1, 1, 8),        # eight channels per group (direct kernels in bf16, generic in fp32)
    (2, 32, 9, 9, 32, 3, 3, 2, 1, 1, 4),          # the same at stride 2
    (1, 160, 8, 9, 160, 3, 3, 1, 1, 1, 40),       # four channels per group, 160 channels: three blocks of output channels, the last half empty
    (1, 72, 7, 7, 72, 5, 5, 1, 2, 1, 36),         # two channels per group, 25 taps (five register chunks in backward-weight)
]
DEPTHWISE = [2, 3, 10, 11, 12, 13, 14, 15, 16, 17, 18, 19, 20, 21, 22, 23]     # shapes the direct kernels take


def _case(i, dtype):
    N, C, H, W, K, R, S, st, pd, dl, G = GROUPED_SHAPES[i]
    x = on_grid(gen.normal(900 + i, 0, (N, C, H, W)), dtype)
    w = on_grid(gen.he_normal(900 + i, 1, (K, C // G, R, S)), dtype)
    P, Q = oracle.conv2d_out_dims(x.shape, (K, C, R, S), st, pd, dl)
    dy = on_grid(gen.normal(900 + i, 2, (N, K, P, Q)), dtype)
    return x, w, dy, st, pd, dl, G


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("i", range(len(GROUPED_SHAPES)))
def test_grouped_conv_fwd_dgrad_wgrad(i, dtype, layout):
    x, w, dy, st, pd, dl, G = _case(i, dtype)
    print(f"grouped conv case {i} {GROUPED_SHAPES[i]} {dtype} layout={layout}", flush=True)
    tol = TOL[dtype]
    ws = B.Workspace()
    gx, gw, gdy = to_gpu(x, dtype, layout), to_gpu(w, dtype, layout), to_gpu(dy, dtype, layout)

    y_view, y_check = guarded(gdy.shape, torch_dtype(dtype))
    B.conv2d_grouped_fwd(gx, gw, G, st, pd, dl, layout, out=y_view, ws=ws)
    torch.cuda.synchronize()
    y_check()
    assert max_rel_err(to_host(y_view, layout), oracle.conv2d_grouped_fwd(x, w, G, st, pd, dl)) <= tol

    dx_view, dx_check = guarded(gx.shape, torch_dtype(dtype))
    B.conv2d_grouped_dgrad(gdy, gw, x.shape, G, st, pd, dl, layout, out=dx_view, ws=ws)
    torch.cuda.synchronize()
    dx_check()
    want_dx = oracle.conv2d_grouped_dgrad(dy, w, x.shape, G, st, pd, dl)
    got_dx = to_host(dx_view, layout)
    assert max_rel_err(got_dx, want_dx) <= tol
    assert np.all(got_dx[want_dx == 0.0] == 0.0)          # cells no tap reaches are written as exact zeros

    dw_view, dw_check = guarded(gw.shape, torch.float32)
    B.conv2d_grouped_wgrad(gx, gdy, w.shape, G, st, pd, dl, layout, out=dw_view, ws=ws)
    torch.cuda.synchronize()
    dw_check()
    want_dw = oracle.conv2d_grouped_wgrad(x, dy, w.shape, G, st, pd, dl)
    assert max_rel_err(to_host(dw_view, layout), want_dw) <= tol


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("i", [0, 2, 4, 7, 10, 11, 12, 14, 15, 17, 18, 19, 20, 21, 22, 23])
def test_grouped_conv_accumulate(i, dtype, layout):
    """accumulate = 1 adds the gradients to what the buffers hold (the paper's gradient accumulation)."""
    x, w, dy, st, pd, dl, G = _case(i, dtype)
    print(f"grouped accumulate case {i} {GROUPED_SHAPES[i]} {dtype} layout={layout}", flush=True)
    tol = TOL[dtype]
    ws = B.Workspace()
    gx, gw, gdy = to_gpu(x, dtype, layout), to_gpu(w, dtype, layout), to_gpu(dy, dtype, layout)
    base = on_grid(gen.normal(900 + i, 3, x.shape), dtype)
    gacc = to_gpu(base, dtype, layout)
    B.conv2d_grouped_dgrad(gdy, gw, x.shape, G, st, pd, dl, layout, out=gacc, accumulate=True, ws=ws)
    base_w = gen.normal(900 + i, 4, w.shape).astype(np.float32)
    gdw = to_gpu(base_w, "f32", layout)
    B.conv2d_grouped_wgrad(gx, gdy, w.shape, G, st, pd, dl, layout, out=gdw, accumulate=True, ws=ws)
    torch.cuda.synchronize()
    want_acc = oracle.conv2d_grouped_dgrad(dy, w, x.shape, G, st, pd, dl, into=base.astype(np.float64))
    assert max_rel_err(to_host(gacc, layout), want_acc) <= tol
    want_dw = oracle.conv2d_grouped_wgrad(x, dy, w.shape, G, st, pd, dl, into=base_w.astype(np.float64))
    assert max_rel_err(to_host(gdw, layout), want_dw) <= tol


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("i", DEPTHWISE)
def test_depthwise_shapes_on_the_generic_kernels(i, dtype, nsk_env):
    """The direct depthwise kernels switched off: the same shapes through the generic grouped launch."""
    nsk_env("NSK_NO_DEPTHWISE", "1")
    test_grouped_conv_fwd_dgrad_wgrad(i, dtype, B.NSK_NHWC)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("i", DEPTHWISE)
def test_depthwise_shapes_on_the_per_tap_kernel(i, dtype, nsk_env):
    """The load-sharing variants of the direct kernels switched off (they take the 3-, 5- and 7-tap-wide or -high filters otherwise)."""
    nsk_env("NSK_DEPTHWISE_NO_ROWS", "1")
    test_grouped_conv_fwd_dgrad_wgrad(i, dtype, B.NSK_NHWC)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("i", DEPTHWISE)
def test_depthwise_shapes_on_the_row_sharing_kernel(i, dtype, nsk_env):
    """The column-stacked variant switched off: the row-sharing one takes the shapes it can."""
    nsk_env("NSK_DEPTHWISE_NO_COLS", "1")
    test_grouped_conv_fwd_dgrad_wgrad(i, dtype, B.NSK_NHWC)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_one_group_is_bitwise_the_plain_call(dtype):
    """groups = 1 takes the same kernels as the plain entry points."""
    x, w, dy, st, pd, dl, G = _case(9, dtype)
    layout = B.NSK_NHWC
    ws = B.Workspace()
    gx, gw, gdy = to_gpu(x, dtype, layout), to_gpu(w, dtype, layout), to_gpu(dy, dtype, layout)
    assert torch.equal(B.conv2d_grouped_fwd(gx, gw, 1, st, pd, dl, layout, ws=ws),
                       B.conv2d_fwd(gx, gw, st, pd, dl, layout, ws=ws))
    assert torch.equal(B.conv2d_grouped_dgrad(gdy, gw, x.shape, 1, st, pd, dl, layout, ws=ws),
                       B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, layout, ws=ws))
    assert torch.equal(B.conv2d_grouped_wgrad(gx, gdy, w.shape, 1, st, pd, dl, layout, ws=ws),
                       B.conv2d_wgrad(gx, gdy, w.shape, st, pd, dl, layout, ws=ws))


def test_grouped_results_are_reproducible():
    x, w, dy, st, pd, dl, G = _case(1, "bf16")
    layout = B.NSK_NHWC
    ws = B.Workspace()
    gx, gw, gdy = to_gpu(x, "bf16", layout), to_gpu(w, "bf16", layout), to_gpu(dy, "bf16", layout)
    a = B.conv2d_grouped_wgrad(gx, gdy, w.shape, G, st, pd, dl, layout, ws=ws)
    b = B.conv2d_grouped_wgrad(gx, gdy, w.shape, G, st, pd, dl, layout, ws=ws)
    assert torch.equal(a, b)


def test_random_grouped_convolutions_match_the_oracle():
    """Seeded sweep: random group counts (from 2 to depthwise), channels per group 1..32 on both sides, strides 1-3,
    padding, dilation, non-square filters; every pass, overwrite and accumulate."""
    rng = np.random.default_rng(4400)
    ws = B.Workspace()
    for case in range(100):
        while True:
            G = int(rng.choice([2, 2, 3, 4, 8, 8, 16, 32]))
            cg, kg = (int(rng.choice([1, 1, 2, 3, 4, 8, 8, 16, 32])) for _ in range(2))
            R, S = (int(rng.choice([1, 2, 3, 3, 3, 5])) for _ in range(2))
            if rng.random() < 0.7:
                S = R
            sh, sw = (int(rng.choice([1, 1, 1, 2, 2, 3])) for _ in range(2))
            if rng.random() < 0.7:
                sw = sh
            ph, pw = int(rng.integers(0, 1 + R // 2 + 1)), int(rng.integers(0, 1 + S // 2 + 1))
            dh, dw = (int(rng.choice([1, 1, 1, 2])) for _ in range(2))
            N, H, W = int(rng.integers(1, 4)), int(rng.integers(4, 15)), int(rng.integers(4, 15))
            P = (H + 2 * ph - dh * (R - 1) - 1) // sh + 1
            Q = (W + 2 * pw - dw * (S - 1) - 1) // sw + 1
            if P >= 1 and Q >= 1:
                break
        C, K, st, pd, dl = G * cg, G * kg, (sh, sw), (ph, pw), (dh, dw)
        shape = (N, C, H, W, K, R, S, st, pd, dl, G)
        dtype = "bf16" if rng.random() < 0.5 else "f32"
        layout = B.NSK_NHWC if rng.random() < 0.75 else B.NSK_NCHW
        print(f"grouped fuzz case {case}: {shape} {dtype} layout={layout}", flush=True)
        seed = 6000 + case
        x = on_grid(gen.normal(seed, 0, (N, C, H, W)), dtype)
        w = on_grid(gen.he_normal(seed, 1, (K, cg, R, S)), dtype)
        dy = on_grid(gen.normal(seed, 2, (N, K, P, Q)), dtype)
        base = on_grid(gen.normal(seed, 3, x.shape), dtype)
        base_w = gen.normal(seed, 4, w.shape).astype(np.float32)
        tol = TOL[dtype]
        gx, gw, gdy = to_gpu(x, dtype, layout), to_gpu(w, dtype, layout), to_gpu(dy, dtype, layout)
        y_view, y_check = guarded(gdy.shape, torch_dtype(dtype))
        B.conv2d_grouped_fwd(gx, gw, G, st, pd, dl, layout, out=y_view, ws=ws)
        dx_view, dx_check = guarded(gx.shape, torch_dtype(dtype))
        B.conv2d_grouped_dgrad(gdy, gw, x.shape, G, st, pd, dl, layout, out=dx_view, ws=ws)
        gacc = to_gpu(base, dtype, layout)
        B.conv2d_grouped_dgrad(gdy, gw, x.shape, G, st, pd, dl, layout, out=gacc, accumulate=True, ws=ws)
        dw_view, dw_check = guarded(gw.shape, torch.float32)
        B.conv2d_grouped_wgrad(gx, gdy, w.shape, G, st, pd, dl, layout, out=dw_view, ws=ws)
        gdw = to_gpu(base_w, "f32", layout)
        B.conv2d_grouped_wgrad(gx, gdy, w.shape, G, st, pd, dl, layout, out=gdw, accumulate=True, ws=ws)
        torch.cuda.synchronize()
        for chk in (y_check, dx_check, dw_check):
            chk()
        assert max_rel_err(to_host(y_view, layout), oracle.conv2d_grouped_fwd(x, w, G, st, pd, dl)) <= tol, shape
        want_dx = oracle.conv2d_grouped_dgrad(dy, w, x.shape, G, st, pd, dl)
        got_dx = to_host(dx_view, layout)
        assert max_rel_err(got_dx, want_dx) <= tol, shape
        assert np.all(got_dx[want_dx == 0.0] == 0.0), shape
        want_acc = oracle.conv2d_grouped_dgrad(dy, w, x.shape, G, st, pd, dl, into=base.astype(np.float64))
        assert max_rel_err(to_host(gacc, layout), want_acc) <= tol, shape
        want_dw = oracle.conv2d_grouped_wgrad(x, dy, w.shape, G, st, pd, dl)
        assert max_rel_err(to_host(dw_view, layout), want_dw) <= tol, shape
        assert max_rel_err(to_host(gdw, layout), want_dw + base_w.astype(np.float64)) <= tol, shape


# N, C, H, K, R, stride, pad, groups: the layers bench.py --grouped times
FULL_SIZE = [
    (128, 128, 56, 128, 3, 1, 1, 128),
    (128, 128, 56, 128, 3, 2, 1, 128),
    (128, 256, 28, 256, 3, 1, 1, 32),
    (128, 128, 56, 128, 3, 1, 1, 32),
]


@pytest.mark.parametrize("i", range(len(FULL_SIZE)))
def test_grouped_layers_at_full_size(i):
    """The grouped layers at the sizes bench.py --grouped times, in its launch configuration (bf16, NHWC).  Groups do
    not mix, so the oracle's plain functions on the channel runs of a few sampled groups (first, last, two in
    between) are exact parity for those groups' outputs: every element of them is compared."""
    N, C, H, K, R, st, pd, G = FULL_SIZE[i]
    print(f"full-size grouped layer {FULL_SIZE[i]}", flush=True)
    dtype, layout = "bf16", B.NSK_NHWC
    cg, kg = C // G, K // G
    x = on_grid(gen.normal(7000 + i, 0, (N, C, H, H)), dtype)
    w = on_grid(gen.he_normal(7000 + i, 1, (K, cg, R, R)), dtype)
    P, Q = oracle.conv2d_out_dims(x.shape, (K, C, R, R), st, pd, 1)
    dy = on_grid(gen.normal(7000 + i, 2, (N, K, P, Q)), dtype)
    ws = B.Workspace()
    gx, gw, gdy = to_gpu(x, dtype, layout), to_gpu(w, dtype, layout), to_gpu(dy, dtype, layout)
    gy = B.conv2d_grouped_fwd(gx, gw, G, st, pd, 1, layout, ws=ws)
    gdx = B.conv2d_grouped_dgrad(gdy, gw, x.shape, G, st, pd, 1, layout, ws=ws)
    gdw = B.conv2d_grouped_wgrad(gx, gdy, w.shape, G, st, pd, 1, layout, ws=ws)
    torch.cuda.synchronize()
    for g in sorted({0, G // 3, (2 * G) // 3, G - 1}):
        cs, ks = slice(g * cg, (g + 1) * cg), slice(g * kg, (g + 1) * kg)
        xg, wg, dyg = np.ascontiguousarray(x[:, cs]), np.ascontiguousarray(w[ks]), np.ascontiguousarray(dy[:, ks])
        got_y = gy[..., ks].float().cpu().permute(0, 3, 1, 2).numpy().astype(np.float64)
        assert max_rel_err(got_y, oracle.conv2d_fwd(xg, wg, st, pd, 1)) <= TOL[dtype], (FULL_SIZE[i], g)
        got_dx = gdx[..., cs].float().cpu().permute(0, 3, 1, 2).numpy().astype(np.float64)
        assert max_rel_err(got_dx, oracle.conv2d_dgrad(dyg, wg, xg.shape, st, pd, 1)) <= TOL[dtype], (FULL_SIZE[i], g)
        got_dw = gdw[ks].cpu().permute(0, 3, 1, 2).numpy().astype(np.float64)
        assert max_rel_err(got_dw, oracle.conv2d_wgrad(xg, dyg, wg.shape, st, pd, 1)) <= TOL["f32"] * 10, (FULL_SIZE[i], g)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_depthwise_channels_do_not_leak_into_each_other(dtype):
    """An infinity in one channel of a depthwise layer's input reaches that channel's outputs only: every other channel
    keeps its bits (the kernels pack two bf16 channels per dword, so this is a property worth pinning)."""
    N, C, H, W = 2, 16, 9, 11
    x = on_grid(gen.normal(7100, 0, (N, C, H, W)), dtype)
    w = on_grid(gen.he_normal(7100, 1, (C, 1, 3, 3)), dtype)
    x_inf = x.copy()
    x_inf[1, 5, 4, 6] = np.inf
    layout = B.NSK_NHWC
    ws = B.Workspace()
    gw = to_gpu(w, dtype, layout)
    y0 = B.conv2d_grouped_fwd(to_gpu(x, dtype, layout), gw, C, 1, 1, 1, layout, ws=ws)
    y1 = B.conv2d_grouped_fwd(to_gpu(x_inf, dtype, layout), gw, C, 1, 1, 1, layout, ws=ws)
    dx0 = B.conv2d_grouped_dgrad(to_gpu(x, dtype, layout), gw, (N, C, H, W), C, 1, 1, 1, layout, ws=ws)
    dx1 = B.conv2d_grouped_dgrad(to_gpu(x_inf, dtype, layout), gw, (N, C, H, W), C, 1, 1, 1, layout, ws=ws)
    torch.cuda.synchronize()
    others = [c for c in range(C) if c != 5]
    for a, b in ((y0, y1), (dx0, dx1)):
        assert torch.equal(a[..., others], b[..., others])
        assert bool(torch.isfinite(a).all()) and not bool(torch.isfinite(b[..., 5]).all())
