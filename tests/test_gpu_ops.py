"""GPU parity of every libnsk entry point against the CPU oracle, element by element, on shapes
that span several tiles and ragged tails (through the C ABI via the ctypes binding)."""
import numpy as np
import pytest
import torch

import nsk_inputs as gen
import oracle
from paper_2409_11600_amd import binding as B
from parity import TOL, guarded, max_rel_err, on_grid, to_gpu, to_host, torch_dtype

pytestmark = pytest.mark.gpu

LAYOUTS = [B.NSK_NHWC, B.NSK_NCHW]

# N, C, H, W, K, R, S, stride, pad, dilation
CONV_SHAPES = [
    (3, 16, 20, 20, 16, 3, 3, 1, 1, 1),        # config-1-like, several M tiles
    (2, 64, 17, 19, 64, 3, 3, 1, 1, 1),        # odd extents, ragged M tail
    (2, 32, 16, 16, 64, 3, 3, 2, 1, 1),        # stride-2 downsample
    (2, 16, 15, 15, 32, 1, 1, 2, 0, 1),        # 1x1 stride-2 projection, odd extent
    (2, 3, 30, 30, 16, 3, 3, 1, 1, 1),         # 3-channel stem (scalar gather)
    (1, 3, 37, 41, 64, 7, 7, 2, 3, 1),         # 7x7 stride-2 pad-3 stem
    (2, 128, 9, 9, 256, 1, 1, 1, 0, 1),        # bottleneck expand, 128x128 tiles
    (2, 256, 9, 9, 64, 1, 1, 1, 0, 1),         # bottleneck reduce
    (1, 72, 11, 13, 40, 3, 3, 1, 1, 1),        # channels not a multiple of the tile sizes
    (2, 24, 14, 12, 20, 3, 2, (2, 1), (1, 0), (1, 2)),   # anisotropic stride, pad, dilation
    (1, 8, 12, 12, 8, 3, 3, 1, 2, 2),          # dilation 2
    (1, 5, 9, 9, 7, 3, 3, 3, 1, 1),            # stride 3, odd channel counts (scalar paths)
    (2, 3, 38, 42, 64, 7, 7, 2, 3, 1),         # 7x7 stride-2 stem, even extents (space-to-depth path)
    (1, 4, 20, 16, 24, 5, 5, 2, 2, 1),         # 5x5 stride-2, 4 channels (space-to-depth, 3x3 coarse taps)
    (2, 1, 12, 18, 16, 3, 3, 2, 1, 1),         # 3x3 stride-2, single channel (space-to-depth, 2x2 coarse taps)
    (1, 64, 6, 66, 64, 3, 3, 1, 1, 1),         # 64->64 on a 66-wide image: too wide for the input ring, single-group halo kernel
    (2, 64, 16, 32, 64, 3, 3, 1, 1, 1),        # 64->64 on 32-wide images with H % 8 == 0: the row-aligned fp32 kernels
    (3, 3, 17, 19, 32, 3, 3, 1, 1, 1),         # 3 -> 32 stride-1 stem, odd extents (direct kernels for few channels)
    (2, 16, 11, 13, 3, 3, 3, 1, 1, 1),         # 16 -> 3: few OUTPUT channels (the same kernels with the roles swapped)
    (2, 2, 9, 9, 8, 3, 3, 2, 1, 1),            # 2 -> 8, stride 2 on odd extents (backward-data classes on the direct kernel)
    (1, 4, 10, 12, 64, 5, 5, 1, 2, (1, 2)),    # 4 -> 64, 5x5 with dilation
]
FEW_CHANNELS = [4, 17, 18, 19, 20]


def _conv_case(i, dtype):
    N, C, H, W, K, R, S, st, pd, dl = CONV_SHAPES[i]
    x = on_grid(gen.normal(500 + i, 0, (N, C, H, W)), dtype)
    w = on_grid(gen.he_normal(500 + i, 1, (K, C, R, S)), dtype)
    P, Q = oracle.conv2d_out_dims(x.shape, w.shape, st, pd, dl)
    dy = on_grid(gen.normal(500 + i, 2, (N, K, P, Q)), dtype)
    return x, w, dy, st, pd, dl


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("i", range(len(CONV_SHAPES)))
def test_conv_fwd_dgrad_wgrad(i, dtype, layout):
    x, w, dy, st, pd, dl = _conv_case(i, dtype)
    print(f"conv case {i} {CONV_SHAPES[i]} {dtype} layout={layout}", flush=True)
    tol = TOL[dtype]
    ws = B.Workspace()
    gx, gw, gdy = to_gpu(x, dtype, layout), to_gpu(w, dtype, layout), to_gpu(dy, dtype, layout)

    y_view, y_check = guarded(gdy.shape, torch_dtype(dtype))
    B.conv2d_fwd(gx, gw, st, pd, dl, layout, out=y_view, ws=ws)
    torch.cuda.synchronize()
    y_check()
    assert max_rel_err(to_host(y_view, layout), oracle.conv2d_fwd(x, w, st, pd, dl)) <= tol

    dx_view, dx_check = guarded(gx.shape, torch_dtype(dtype))
    B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, layout, out=dx_view, ws=ws)
    torch.cuda.synchronize()
    dx_check()
    want_dx = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl)
    got_dx = to_host(dx_view, layout)
    assert max_rel_err(got_dx, want_dx) <= tol
    assert np.all(got_dx[want_dx == 0.0] == 0.0)          # cells no tap reaches are written as exact zeros

    dw_view, dw_check = guarded(gw.shape, torch.float32)
    B.conv2d_wgrad(gx, gdy, w.shape, st, pd, dl, layout, out=dw_view, ws=ws)
    torch.cuda.synchronize()
    dw_check()
    assert max_rel_err(to_host(dw_view, layout), oracle.conv2d_wgrad(x, dy, w.shape, st, pd, dl)) <= tol


# Shapes with channel counts that are multiples of 64: routed through the large-tile bf16 kernel by lowering
# its tile-count threshold (at their full sizes these layers take it on their own).
WIDE_SHAPES = [
    (2, 128, 9, 9, 256, 1, 1, 1, 0, 1),        # 1x1, two column blocks, ragged row block
    (3, 256, 10, 9, 64, 1, 1, 1, 0, 1),        # 1x1, 64-column variant, four k-tiles
    (2, 64, 18, 14, 128, 3, 3, 2, 1, 1),       # 3x3 stride 2 (four parity classes in backward-data)
    (2, 128, 11, 13, 128, 3, 3, 1, 1, 1),      # 3x3 stride 1, 18 k-tiles, padding on every side
    (4, 64, 16, 16, 192, 1, 1, 2, 0, 1),       # 1x1 stride 2, 192 columns (half-empty second column block)
    (1, 64, 33, 17, 64, 3, 3, 1, 2, 2),        # dilation 2
    (2, 3, 20, 24, 64, 7, 7, 2, 3, 1),         # image stem: space-to-depth, then the large-tile backward-weight kernel on 16 channels
    (2, 32, 12, 10, 64, 3, 3, 2, 1, 1),        # 32 input channels (four taps per 128-column tile)
    (4, 16, 12, 12, 16, 3, 3, 1, 1, 1),        # 16 -> 16: a quarter of the 64-row backward-weight tile is live
    (4, 16, 12, 12, 32, 3, 3, 2, 1, 1),        # 16 -> 32 stride 2
    (3, 32, 9, 9, 32, 3, 3, 1, 1, 1),          # 32 -> 32
    (4, 16, 10, 10, 32, 1, 1, 2, 0, 1),        # 1x1 projection, 16 columns
    (2, 24, 9, 9, 40, 3, 3, 1, 1, 1),          # 40 output channels, 24 input channels
    (2, 128, 10, 10, 128, 3, 3, 2, 1, 1),      # stride 2, 128 columns: the four backward-data classes in one launch
    (3, 64, 9, 11, 64, 3, 3, 2, 1, 1),         # the same with 64 columns on odd extents (classes of different sizes)
    (2, 64, 8, 8, 128, 2, 2, 2, 0, 1),         # 2x2 stride 2: four one-tap classes
]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("i", range(len(WIDE_SHAPES)))
def test_conv_wide_layers_large_tile_kernel(i, layout, nsk_env):
    nsk_env("NSK_BIG_MIN_TILES", "1")
    nsk_env("NSK_WIDE_MIN_ROWS", "1")
    N, C, H, W, K, R, S, st, pd, dl = WIDE_SHAPES[i]
    print(f"wide conv case {i} {WIDE_SHAPES[i]} layout={layout}", flush=True)
    dtype = "bf16"
    x = on_grid(gen.normal(700 + i, 0, (N, C, H, W)), dtype)
    w = on_grid(gen.he_normal(700 + i, 1, (K, C, R, S)), dtype)
    P, Q = oracle.conv2d_out_dims(x.shape, w.shape, st, pd, dl)
    dy = on_grid(gen.normal(700 + i, 2, (N, K, P, Q)), dtype)
    base = on_grid(gen.normal(700 + i, 3, x.shape), dtype)
    tol = TOL[dtype]
    ws = B.Workspace()
    gx, gw, gdy = to_gpu(x, dtype, layout), to_gpu(w, dtype, layout), to_gpu(dy, dtype, layout)
    y_view, y_check = guarded(gdy.shape, torch_dtype(dtype))
    B.conv2d_fwd(gx, gw, st, pd, dl, layout, out=y_view, ws=ws)
    dx_view, dx_check = guarded(gx.shape, torch_dtype(dtype))
    B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, layout, out=dx_view, ws=ws)
    gacc = to_gpu(base, dtype, layout)
    B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, layout, out=gacc, accumulate=True, ws=ws)
    torch.cuda.synchronize()
    y_check()
    dx_check()
    assert max_rel_err(to_host(y_view, layout), oracle.conv2d_fwd(x, w, st, pd, dl)) <= tol
    want_dx = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl)
    got_dx = to_host(dx_view, layout)
    assert max_rel_err(got_dx, want_dx) <= tol
    assert np.all(got_dx[want_dx == 0.0] == 0.0)
    want_acc = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl, into=base.astype(np.float64))
    assert max_rel_err(to_host(gacc, layout), want_acc) <= tol
    # backward-weight through the large-tile kernel, overwrite and accumulate
    dw_view, dw_check = guarded(gw.shape, torch.float32)
    B.conv2d_wgrad(gx, gdy, w.shape, st, pd, dl, layout, out=dw_view, ws=ws)
    base_w = gen.normal(700 + i, 4, w.shape).astype(np.float32)
    gdw = to_gpu(base_w, "f32", layout)
    B.conv2d_wgrad(gx, gdy, w.shape, st, pd, dl, layout, out=gdw, accumulate=True, ws=ws)
    torch.cuda.synchronize()
    dw_check()
    want_dw = oracle.conv2d_wgrad(x, dy, w.shape, st, pd, dl)
    assert max_rel_err(to_host(dw_view, layout), want_dw) <= TOL["f32"] * 10   # fp32 sums of exact bf16 products
    assert max_rel_err(to_host(gdw, layout), want_dw + base_w.astype(np.float64)) <= TOL["f32"] * 10


# 3x3 stride-1 bf16 layers with 128 or 256 input channels for the kernel that stages whole image rows (all channels, with
# halo) once and streams the filter from L2 into MFMA operand registers.  NSK_HALO_WIDE_ALWAYS lifts its size
# thresholds so that these small shapes take it.
HALO_WIDE_SHAPES = [
    (3, 128, 14, 14, 128),       # one image per tile (14 rows of 16 padded positions), one column block
    (2, 256, 14, 14, 256),       # the bottleneck-stage layer itself: two column blocks
    (2, 128, 9, 11, 256),        # the tile ends inside its last position tile
    (1, 256, 20, 13, 128),       # two tiles per image, the second with fewer rows
    (2, 128, 30, 30, 128),       # 32 padded positions per row: 7 rows per tile, 5 tiles per image (ragged last one)
    (3, 256, 7, 7, 128),         # a tile of 7 rows of 9 padded positions: two of the seven position tiles are live
    (1, 128, 5, 100, 128),       # wide rows: two rows per tile, halo of 103 positions on each side
    (1, 128, 3, 220, 128),       # one row per tile
    (2, 64, 12, 12, 128),        # 64 input channels: a single channel group, nothing left for the moving wavefront
    (2, 128, 10, 10, 64),        # 64 output channels: blocks of two multiplying wavefronts
    (2, 256, 9, 9, 192),         # 192 output channels: three such blocks per tile
]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("i", range(len(HALO_WIDE_SHAPES)))
def test_conv_wide_halo_kernel(i, layout, nsk_env):
    nsk_env("NSK_HALO_WIDE_ALWAYS", "1")
    N, C, H, W, K = HALO_WIDE_SHAPES[i]
    print(f"wide halo conv case {i} {HALO_WIDE_SHAPES[i]} layout={layout}", flush=True)
    dtype, st, pd, dl = "bf16", 1, 1, 1
    x = on_grid(gen.normal(1300 + i, 0, (N, C, H, W)), dtype)
    w = on_grid(gen.he_normal(1300 + i, 1, (K, C, 3, 3)), dtype)
    dy = on_grid(gen.normal(1300 + i, 2, (N, K, H, W)), dtype)
    base = on_grid(gen.normal(1300 + i, 3, x.shape), dtype)
    tol = TOL[dtype]
    ws = B.Workspace()
    gx, gw, gdy = to_gpu(x, dtype, layout), to_gpu(w, dtype, layout), to_gpu(dy, dtype, layout)
    y_view, y_check = guarded(gdy.shape, torch_dtype(dtype))
    B.conv2d_fwd(gx, gw, st, pd, dl, layout, out=y_view, ws=ws)
    y1, stats = B.conv2d_fwd_stats(gx, gw, st, pd, dl, layout, ws=ws)
    y2, _ = B.conv2d_fwd_stats(gx, gw, st, pd, dl, layout, ws=ws)
    if C == K:       # backward-data of a C -> K layer is a K -> C layer: the kernel needs 128..512 channels there too
        dx_view, dx_check = guarded(gx.shape, torch_dtype(dtype))
        B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, layout, out=dx_view, ws=ws)
        gacc = to_gpu(base, dtype, layout)
        B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, layout, out=gacc, accumulate=True, ws=ws)
    torch.cuda.synchronize()
    y_check()
    want_y = oracle.conv2d_fwd(x, w, st, pd, dl)
    assert max_rel_err(to_host(y_view, layout), want_y) <= tol
    assert torch.equal(y1, y2) and torch.equal(y1.flatten(), y_view.reshape(y1.shape).flatten())   # reproducible; same as plain
    yh = to_host(y1, layout)
    sums = stats.double().sum(dim=1).cpu().numpy()
    want0, want1 = yh.sum(axis=(0, 2, 3)), (yh * yh).sum(axis=(0, 2, 3))
    assert np.max(np.abs(sums[0] - want0) / (np.sqrt(want1 * yh[:, 0].size) + 1e-30)) <= 1e-6
    assert np.max(np.abs(sums[1] - want1) / (want1 + 1e-30)) <= 1e-5
    if C == K:
        dx_check()
        want_dx = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl)
        assert max_rel_err(to_host(dx_view, layout), want_dx) <= tol
        want_acc = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl, into=base.astype(np.float64))
        assert max_rel_err(to_host(gacc, layout), want_acc) <= tol



# Backward-data of strided layers through the same kernel: the residue classes of the output position (four for
# stride 2) are stride-1 convolutions over the same dy tiles and share one launch.  N, C, H, W, K, R, stride, pad
HALO_WIDE_STRIDED = [
    (2, 128, 28, 28, 128, 3, 2, 1),      # 3x3 stride 2: classes with 4, 2, 2 and 1 taps
    (2, 256, 14, 14, 256, 3, 2, 1),      # 7x7 dy grid, two column blocks
    (1, 256, 27, 25, 128, 3, 2, 1),      # odd extents: classes of different sizes
    (2, 128, 12, 20, 128, 2, 2, 0),      # 2x2 stride 2: four one-tap classes
    (1, 128, 16, 16, 128, 4, 2, 1),      # 4x4 stride 2: four taps in every class
    (1, 128, 20, 18, 128, 3, (2, 1), 1), # stride 2 along rows only: two classes with 6 and 3 taps
    (2, 64, 20, 24, 64, 3, 2, 1),        # 64 -> 64: one channel group, blocks of two multiplying wavefronts
    (1, 192, 14, 14, 64, 3, 2, 1),       # 192 output channels of the backward pass: three blocks per tile
]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("i", range(len(HALO_WIDE_STRIDED)))
def test_conv_wide_halo_kernel_strided_backward_data(i, layout, nsk_env):
    nsk_env("NSK_HALO_WIDE_ALWAYS", "1")
    N, C, H, W, K, R, st, pd = HALO_WIDE_STRIDED[i]
    print(f"wide halo strided dgrad case {i} {HALO_WIDE_STRIDED[i]} layout={layout}", flush=True)
    dtype, dl = "bf16", 1
    x_shape = (N, C, H, W)
    w = on_grid(gen.he_normal(1400 + i, 1, (K, C, R, R)), dtype)
    P, Q = oracle.conv2d_out_dims(x_shape, w.shape, st, pd, dl)
    dy = on_grid(gen.normal(1400 + i, 2, (N, K, P, Q)), dtype)
    base = on_grid(gen.normal(1400 + i, 3, x_shape), dtype)
    tol = TOL[dtype]
    ws = B.Workspace()
    gw, gdy = to_gpu(w, dtype, layout), to_gpu(dy, dtype, layout)
    dx_view, dx_check = guarded(x_shape if layout == B.NSK_NCHW else (N, H, W, C), torch_dtype(dtype))
    B.conv2d_dgrad(gdy, gw, x_shape, st, pd, dl, layout, out=dx_view, ws=ws)
    again = torch.empty_like(dx_view)
    B.conv2d_dgrad(gdy, gw, x_shape, st, pd, dl, layout, out=again, ws=ws)
    gacc = to_gpu(base, dtype, layout)
    B.conv2d_dgrad(gdy, gw, x_shape, st, pd, dl, layout, out=gacc, accumulate=True, ws=ws)
    torch.cuda.synchronize()
    dx_check()
    want_dx = oracle.conv2d_dgrad(dy, w, x_shape, st, pd, dl)
    got_dx = to_host(dx_view, layout)
    assert max_rel_err(got_dx, want_dx) <= tol
    assert np.all(got_dx[want_dx == 0.0] == 0.0)
    assert torch.equal(again, dx_view)
    want_acc = oracle.conv2d_dgrad(dy, w, x_shape, st, pd, dl, into=base.astype(np.float64))
    assert max_rel_err(to_host(gacc, layout), want_acc) <= tol


# The forward pass of 3x3 stride-2 pad-1 layers with 128 or 256 input channels on even extents: the same kernel on the
# four parity planes of the input, staged one after the other (two moving wavefronts, requests two stages ahead) and
# merged into one set of accumulators.  N, C, H, W, K
HALO_WIDE_FWD_S2 = [
    (2, 256, 28, 28, 256),       # the bottleneck-stage layer itself: one image per tile, two column blocks
    (3, 128, 28, 28, 128),       # two channel groups: a plane's first group lands on the columns read two stages before
    (2, 128, 18, 22, 64),        # the tile ends inside its last position tile; blocks of two multiplying wavefronts
    (1, 256, 40, 26, 128),       # two tiles per image, the second with fewer rows
    (2, 128, 8, 56, 192),        # seven rows of 30 padded positions per tile; three column blocks of 64
    (1, 128, 12, 58, 128),       # 31 padded positions per row: the most staged rows the two moving wavefronts take (288)
]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("i", range(len(HALO_WIDE_FWD_S2)))
def test_conv_wide_halo_kernel_stride2_forward(i, layout, nsk_env):
    nsk_env("NSK_HALO_WIDE_ALWAYS", "1")
    N, C, H, W, K = HALO_WIDE_FWD_S2[i]
    print(f"wide halo stride-2 forward case {i} {HALO_WIDE_FWD_S2[i]} layout={layout}", flush=True)
    dtype, st, pd, dl = "bf16", 2, 1, 1
    x = on_grid(gen.normal(1450 + i, 0, (N, C, H, W)), dtype)
    w = on_grid(gen.he_normal(1450 + i, 1, (K, C, 3, 3)), dtype)
    ws = B.Workspace()
    gx, gw = to_gpu(x, dtype, layout), to_gpu(w, dtype, layout)
    out_shape = (N, K, H // 2, W // 2) if layout == B.NSK_NCHW else (N, H // 2, W // 2, K)
    y_view, y_check = guarded(out_shape, torch_dtype(dtype))
    B.conv2d_fwd(gx, gw, st, pd, dl, layout, out=y_view, ws=ws)
    y1, stats = B.conv2d_fwd_stats(gx, gw, st, pd, dl, layout, ws=ws)
    y2, _ = B.conv2d_fwd_stats(gx, gw, st, pd, dl, layout, ws=ws)
    torch.cuda.synchronize()
    y_check()
    want_y = oracle.conv2d_fwd(x, w, st, pd, dl)
    assert max_rel_err(to_host(y_view, layout), want_y) <= TOL[dtype]
    assert torch.equal(y1, y2) and torch.equal(y1.flatten(), y_view.reshape(y1.shape).flatten())   # reproducible; same as plain
    yh = to_host(y1, layout)
    sums = stats.double().sum(dim=1).cpu().numpy()
    want0, want1 = yh.sum(axis=(0, 2, 3)), (yh * yh).sum(axis=(0, 2, 3))
    assert np.max(np.abs(sums[0] - want0) / (np.sqrt(want1 * yh[:, 0].size) + 1e-30)) <= 1e-6
    assert np.max(np.abs(sums[1] - want1) / (want1 + 1e-30)) <= 1e-5
    # the kernels that take the layer otherwise
    nsk_env("NSK_NO_HALO_WIDE", "1")
    y3 = B.conv2d_fwd(gx, gw, st, pd, dl, layout, ws=ws)
    assert max_rel_err(to_host(y3, layout), want_y) <= TOL[dtype]



# Short-reduction bf16 layers (1, 2 or 4 taps, at most 256 reduction indices) for the kernel that keeps the filter
# in LDS and loads pixels straight into MFMA operands.
PW_SHAPES = [
    (2, 128, 9, 9, 256, 1, 1, 1, 0, 1),        # four column chunks forward, 256 input channels (32-pixel tiles) backward
    (3, 256, 10, 9, 64, 1, 1, 1, 0, 1),        # 256 -> 64 and back
    (4, 64, 16, 16, 192, 1, 1, 2, 0, 1),       # stride 2, three column chunks (backward takes the generic kernel)
    (2, 64, 15, 13, 64, 1, 1, 2, 0, 1),        # stride 2 on odd extents: ragged residue classes in backward-data
    (5, 128, 7, 7, 128, 1, 1, 1, 0, 1),        # ragged last tile
    (1, 64, 6, 6, 64, 1, 1, 1, 1, 1),          # padded 1x1: source positions outside the image read as zero
    (4, 64, 250, 260, 64, 1, 1, 1, 0, 1),      # several tiles per wavefront (both register sets, prefetch across tiles)
    (2, 64, 18, 14, 64, 3, 3, 2, 1, 1),        # backward-data classes with 1, 2, 2 and 4 taps on 64 channels
    (2, 64, 17, 15, 64, 3, 3, 2, 1, 1),        # the same on odd extents
    (2, 64, 12, 12, 128, 3, 3, 2, 1, 1),       # 128 channels: classes with 1 and 2 taps (the 4-tap class is generic)
    (2, 64, 12, 14, 64, 2, 2, 2, 0, 1),        # 2x2 stride-2 filter: four taps forward, one tap per class backward
    (1, 128, 9, 9, 64, 1, 2, 1, 0, 1),         # two taps of 128 channels forward
    # narrow outputs (16 and 32 channels): the layers of the CIFAR-sized network
    (4, 16, 12, 12, 16, 3, 3, 1, 1, 1),        # 16 -> 16 3x3: half of each MFMA tile is padding
    (4, 16, 12, 12, 32, 3, 3, 2, 1, 1),        # 16 -> 32 stride 2; backward-data classes of 1, 2, 4 taps on 32 channels
    (4, 16, 10, 10, 32, 1, 1, 2, 0, 1),        # its projection shortcut (zero fill of the 2x2 cells in backward-data)
    (3, 32, 9, 9, 32, 3, 3, 1, 1, 1),          # 32 -> 32 3x3
    (3, 32, 10, 10, 64, 3, 3, 2, 1, 1),        # 32 -> 64 stride 2: 64-channel chunk forward, 32-channel outputs backward
    (3, 32, 11, 9, 64, 1, 1, 2, 0, 1),         # and its projection, odd extents
    (2, 64, 9, 9, 16, 1, 1, 1, 0, 1),          # 64 -> 16: four k-steps, 16-channel output
    (2, 16, 8, 8, 16, 2, 2, 2, 0, 1),          # 2x2 stride 2 on 16 channels: four taps forward
    (2, 32, 6, 7, 32, 1, 2, 1, 0, 1),          # two taps of 32 channels
    (300, 16, 32, 32, 16, 3, 3, 1, 1, 1),      # the CIFAR layer itself at more than full batch: several tiles per wavefront
    # outputs too wide for one block's LDS: column groups
    (2, 256, 9, 9, 1024, 1, 1, 1, 0, 1),       # 256 -> 1024: eight groups of 128 columns
    (3, 128, 8, 8, 512, 1, 1, 1, 0, 1),        # 128 -> 512: two groups of 256 columns
    (2, 1024, 6, 6, 256, 1, 1, 1, 0, 1),       # 1024 -> 256: backward-data (also accumulating) in eight groups
    (40, 256, 14, 14, 1024, 1, 1, 1, 0, 1),    # the bottleneck layer itself at reduced batch: several tiles per wavefront
    (2, 512, 7, 7, 256, 1, 1, 1, 0, 1),        # 512 channels in one tap (32 k-steps), four groups of 64 columns
    (2, 512, 8, 8, 1024, 1, 1, 2, 0, 1),       # the stride-2 projection: sixteen groups
]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("i", range(len(PW_SHAPES)))
def test_conv_pointwise_kernel(i, layout, nsk_env):
    nsk_env("NSK_PW_MIN_ROWS", "1")
    N, C, H, W, K, R, S, st, pd, dl = PW_SHAPES[i]
    if layout == B.NSK_NCHW and N * H * W > 100000:
        pytest.skip("large case once (NHWC)")
    print(f"pointwise conv case {i} {PW_SHAPES[i]} layout={layout}", flush=True)
    dtype = "bf16"
    x = on_grid(gen.normal(1100 + i, 0, (N, C, H, W)), dtype)
    w = on_grid(gen.he_normal(1100 + i, 1, (K, C, R, S)), dtype)
    P, Q = oracle.conv2d_out_dims(x.shape, w.shape, st, pd, dl)
    dy = on_grid(gen.normal(1100 + i, 2, (N, K, P, Q)), dtype)
    tol = TOL[dtype]
    ws = B.Workspace()
    gx, gw, gdy = to_gpu(x, dtype, layout), to_gpu(w, dtype, layout), to_gpu(dy, dtype, layout)
    y_view, y_check = guarded(gdy.shape, torch_dtype(dtype))
    B.conv2d_fwd(gx, gw, st, pd, dl, layout, out=y_view, ws=ws)
    y1, stats = B.conv2d_fwd_stats(gx, gw, st, pd, dl, layout, ws=ws)
    dx_view, dx_check = guarded(gx.shape, torch_dtype(dtype))
    B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, layout, out=dx_view, ws=ws)
    torch.cuda.synchronize()
    y_check()
    dx_check()
    assert torch.equal(y_view, y1)
    # one row of partial sums per wavefront of this kernel's fixed grid: the forward pass really took it
    # (nine taps into 128 channels and the 1024-channel input take other kernels; split outputs have fewer row shares)
    assert stats.shape[1] in (1024, 512, 256, 128, 64) or (C, K, R) in ((64, 128, 3), (1024, 256, 1))
    yh = to_host(y_view, layout)
    assert max_rel_err(yh, oracle.conv2d_fwd(x, w, st, pd, dl)) <= tol
    sums = stats.double().sum(dim=1).cpu().numpy()             # [2, K]
    want0, want1 = yh.sum(axis=(0, 2, 3)), (yh * yh).sum(axis=(0, 2, 3))
    assert np.max(np.abs(sums[0] - want0) / (np.sqrt(want1 * yh[:, 0].size) + 1e-30)) <= 1e-6
    assert np.max(np.abs(sums[1] - want1) / (want1 + 1e-30)) <= 1e-5
    want_dx = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl)
    got_dx = to_host(dx_view, layout)
    assert max_rel_err(got_dx, want_dx) <= tol
    assert np.all(got_dx[want_dx == 0.0] == 0.0)
    # accumulating backward-data (old values fetched one chunk ahead, one rounding of old + sum)
    base = on_grid(gen.normal(1100 + i, 3, x.shape), dtype)
    gacc = to_gpu(base, dtype, layout)
    B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, layout, out=gacc, accumulate=True, ws=ws)
    torch.cuda.synchronize()
    want_acc = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl, into=base.astype(np.float64))
    assert max_rel_err(to_host(gacc, layout), want_acc) <= tol
    # a second run gives the same bits (fixed summation order, no atomics), partial sums included
    y2, stats2 = B.conv2d_fwd_stats(gx, gw, st, pd, dl, layout, ws=ws)
    dx2 = B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, layout, ws=ws)
    torch.cuda.synchronize()
    assert torch.equal(y2, y1) and torch.equal(stats2, stats) and torch.equal(dx2, dx_view)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("i", [1, 2, 3, 4, 8, 12, 13, 15, 16, 17, 18, 19, 20])
def test_conv_gradients_accumulate(i, dtype, layout):
    x, w, dy, st, pd, dl = _conv_case(i, dtype)
    ws = B.Workspace()
    base_x = on_grid(gen.normal(600 + i, 0, x.shape), dtype)
    base_w = gen.normal(600 + i, 1, w.shape)
    gdx = to_gpu(base_x, dtype, layout)
    gdw = to_gpu(base_w, "f32", layout)
    gx, gw, gdy = to_gpu(x, dtype, layout), to_gpu(w, dtype, layout), to_gpu(dy, dtype, layout)
    B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, layout, out=gdx, accumulate=True, ws=ws)
    B.conv2d_wgrad(gx, gdy, w.shape, st, pd, dl, layout, out=gdw, accumulate=True, ws=ws)
    torch.cuda.synchronize()
    want_dx = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl, into=base_x.astype(np.float64))
    want_dw = oracle.conv2d_wgrad(x, dy, w.shape, st, pd, dl, into=base_w.astype(np.float64))
    assert max_rel_err(to_host(gdx, layout), want_dx) <= TOL[dtype]
    assert max_rel_err(to_host(gdw, layout), want_dw) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_halo_backward_weight_many_chunks_per_block(dtype, nsk_env):
    """3x3 64->64 backward-weight on enough positions that every block of the halo kernel walks several chunks (the
    double-buffered hand-over between its moving and its multiplying wavefronts), against the oracle; the variant
    without split roles must give the same bits."""
    N, C, H, W, K = 8, 64, 46, 46, 64
    print(f"halo backward-weight, many chunks: {(N, C, H, W, K)} {dtype}", flush=True)
    x = on_grid(gen.normal(880, 0, (N, C, H, W)), dtype)
    dy = on_grid(gen.normal(880, 2, (N, K, H, W)), dtype)
    layout = B.NSK_NHWC
    ws = B.Workspace()
    gx, gdy = to_gpu(x, dtype, layout), to_gpu(dy, dtype, layout)
    dw_view, dw_check = guarded((K, 3, 3, C), torch.float32)
    B.conv2d_wgrad(gx, gdy, (K, C, 3, 3), 1, 1, 1, layout, out=dw_view, ws=ws)
    torch.cuda.synchronize()
    dw_check()
    want = oracle.conv2d_wgrad(x, dy, (K, C, 3, 3), 1, 1, 1)
    assert max_rel_err(to_host(dw_view, layout), want) <= TOL["f32"] * 10   # fp32 sums of exact products
    nsk_env("NSK_WH_NO_SPLIT", "1")
    plain = B.conv2d_wgrad(gx, gdy, (K, C, 3, 3), 1, 1, 1, layout, ws=ws)
    torch.cuda.synchronize()
    assert torch.equal(plain, dw_view)


# bf16 3x3 stride-1 64->64 layers, forward and backward-data: the filter-stationary kernel (128- or 256-position
# tiles; blocks that walk several tiles; ragged last tile; images wider than the 256-position ring allows) and, with
# NSK_NO_FS, the kernels that keep the filter in LDS.  N, H, W
FS_SHAPES = [(3, 20, 24), (16, 56, 56), (5, 7, 61), (2, 9, 66), (40, 8, 8), (1, 1, 1), (9, 33, 17)]


@pytest.mark.parametrize("no_fs", [False, True], ids=["filter_in_registers", "filter_in_lds"])
@pytest.mark.parametrize("i", range(len(FS_SHAPES)))
def test_conv_64_to_64_kernels(i, no_fs, nsk_env):
    N, H, W = FS_SHAPES[i]
    if no_fs:
        nsk_env("NSK_NO_FS", "1")
    print(f"64->64 case {FS_SHAPES[i]} no_fs={no_fs}", flush=True)
    x = on_grid(gen.normal(1500 + i, 0, (N, 64, H, W)), "bf16")
    w = on_grid(gen.he_normal(1500 + i, 1, (64, 64, 3, 3)), "bf16")
    dy = on_grid(gen.normal(1500 + i, 2, (N, 64, H, W)), "bf16")
    ws = B.Workspace()
    gx, gw, gdy = (to_gpu(a, "bf16", B.NSK_NHWC) for a in (x, w, dy))
    y, check_y = guarded((N, H, W, 64), torch.bfloat16)
    dx, check_dx = guarded((N, H, W, 64), torch.bfloat16)
    B.conv2d_fwd(gx, gw, 1, 1, 1, out=y, ws=ws)
    B.conv2d_dgrad(gdy, gw, (N, 64, H, W), 1, 1, 1, out=dx, ws=ws)
    y_s, stats = B.conv2d_fwd_stats(gx, gw, 1, 1, 1, ws=ws)
    torch.cuda.synchronize()
    check_y()
    check_dx()
    want_y = oracle.conv2d_fwd(x, w, 1, 1, 1)
    assert max_rel_err(to_host(y, B.NSK_NHWC), want_y) <= TOL["bf16"]
    assert max_rel_err(to_host(dx, B.NSK_NHWC), oracle.conv2d_dgrad(dy, w, x.shape, 1, 1, 1)) <= TOL["bf16"]
    assert torch.equal(y, y_s)
    # the partial sums against the oracle's y on the storage grid (a stored value may differ from it by one rounding)
    y_grid = on_grid(want_y.astype(np.float32), "bf16")
    sums = stats.double().sum(dim=1).cpu().numpy()
    M = N * H * W
    sigma = np.sqrt((y_grid * y_grid).sum(axis=(0, 2, 3)) / M) + 1e-30
    assert np.max(np.abs(sums[0] - y_grid.sum(axis=(0, 2, 3))) / (M * sigma)) <= 1e-3
    assert np.max(np.abs(sums[1] - (y_grid * y_grid).sum(axis=(0, 2, 3))) / (M * sigma * sigma)) <= 1e-3
    # accumulating backward-data (one rounding of old + sum)
    old = on_grid(gen.normal(1500 + i, 3, (N, 64, H, W)), "bf16")
    acc = to_gpu(old, "bf16", B.NSK_NHWC)
    B.conv2d_dgrad(gdy, gw, (N, 64, H, W), 1, 1, 1, out=acc, accumulate=True, ws=ws)
    assert max_rel_err(to_host(acc, B.NSK_NHWC), oracle.conv2d_dgrad(dy, w, x.shape, 1, 1, 1, into=old.astype(np.float64))) <= TOL["bf16"]


# bf16 3x3 stride-2 pad-1 64->64 layers on even extents: backward-data of all four residue classes in one launch of
# the filter-stationary kernel (blocks that walk several tiles, ragged last tile, tiles that span many small images);
# with NSK_NO_FS the same problems on the kernels that take the classes otherwise.  N, H, W
FS_S2_SHAPES = [(8, 112, 112), (20, 60, 68), (70, 30, 34), (300, 14, 14), (2100, 4, 6)]


@pytest.mark.parametrize("no_fs", [False, True], ids=["filter_in_registers", "other_kernels"])
@pytest.mark.parametrize("i", range(len(FS_S2_SHAPES)))
def test_conv_64_to_64_stride2_backward_data(i, no_fs, nsk_env):
    N, H, W = FS_S2_SHAPES[i]
    if no_fs:
        nsk_env("NSK_NO_FS", "1")
    print(f"64->64 stride 2 dgrad case {FS_S2_SHAPES[i]} no_fs={no_fs}", flush=True)
    w = on_grid(gen.he_normal(1600 + i, 1, (64, 64, 3, 3)), "bf16")
    dy = on_grid(gen.normal(1600 + i, 2, (N, 64, H // 2, W // 2)), "bf16")
    ws = B.Workspace()
    gw, gdy = to_gpu(w, "bf16", B.NSK_NHWC), to_gpu(dy, "bf16", B.NSK_NHWC)
    dx, check_dx = guarded((N, H, W, 64), torch.bfloat16)
    B.conv2d_dgrad(gdy, gw, (N, 64, H, W), 2, 1, 1, out=dx, ws=ws)
    torch.cuda.synchronize()
    check_dx()
    want = oracle.conv2d_dgrad(dy, w, (N, 64, H, W), 2, 1, 1)
    assert max_rel_err(to_host(dx, B.NSK_NHWC), want) <= TOL["bf16"]
    dx2 = B.conv2d_dgrad(gdy, gw, (N, 64, H, W), 2, 1, 1, ws=ws)
    assert torch.equal(dx, dx2)


# The forward pass of the same layers: the filter-stationary kernel on four parity planes of the input (one tile per
# block, several tiles per block, ragged last tile, tiles over many small images, the widest image its rings hold
# (174 columns: all of the LDS) and one that is wider and goes elsewhere), plain and with the batch-norm statistics.  N, H, W
FS_S2_FWD_SHAPES = FS_S2_SHAPES + [(24, 112, 112), (90, 60, 68), (6, 124, 124), (6, 64, 174), (6, 64, 178)]


@pytest.mark.parametrize("no_fs", [False, True], ids=["filter_in_registers", "other_kernels"])
@pytest.mark.parametrize("i", range(len(FS_S2_FWD_SHAPES)))
def test_conv_64_to_64_stride2_forward(i, no_fs, nsk_env):
    N, H, W = FS_S2_FWD_SHAPES[i]
    if no_fs:
        nsk_env("NSK_NO_FS", "1")
    print(f"64->64 stride 2 forward case {FS_S2_FWD_SHAPES[i]} no_fs={no_fs}", flush=True)
    x = on_grid(gen.normal(1700 + i, 0, (N, 64, H, W)), "bf16")
    w = on_grid(gen.he_normal(1700 + i, 1, (64, 64, 3, 3)), "bf16")
    ws = B.Workspace()
    gx, gw = to_gpu(x, "bf16", B.NSK_NHWC), to_gpu(w, "bf16", B.NSK_NHWC)
    y, check_y = guarded((N, H // 2, W // 2, 64), torch.bfloat16)
    B.conv2d_fwd(gx, gw, 2, 1, 1, out=y, ws=ws)
    y_s, stats = B.conv2d_fwd_stats(gx, gw, 2, 1, 1, ws=ws)
    torch.cuda.synchronize()
    check_y()
    want_y = oracle.conv2d_fwd(x, w, 2, 1, 1)
    assert max_rel_err(to_host(y, B.NSK_NHWC), want_y) <= TOL["bf16"]
    assert torch.equal(y, y_s)
    y_grid = on_grid(want_y.astype(np.float32), "bf16")
    sums = stats.double().sum(dim=1).cpu().numpy()
    M = N * (H // 2) * (W // 2)
    sigma = np.sqrt((y_grid * y_grid).sum(axis=(0, 2, 3)) / M) + 1e-30
    assert np.max(np.abs(sums[0] - y_grid.sum(axis=(0, 2, 3))) / (M * sigma)) <= 1e-3
    assert np.max(np.abs(sums[1] - (y_grid * y_grid).sum(axis=(0, 2, 3))) / (M * sigma * sigma)) <= 1e-3
    y2 = B.conv2d_fwd(gx, gw, 2, 1, 1, ws=ws)
    assert torch.equal(y, y2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_conv_is_bitwise_reproducible(dtype):
    x, w, dy, st, pd, dl = _conv_case(1, dtype)
    ws = B.Workspace()
    gx, gw, gdy = to_gpu(x, dtype, B.NSK_NHWC), to_gpu(w, dtype, B.NSK_NHWC), to_gpu(dy, dtype, B.NSK_NHWC)
    a = [B.conv2d_fwd(gx, gw, st, pd, dl, ws=ws), B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, ws=ws),
         B.conv2d_wgrad(gx, gdy, w.shape, st, pd, dl, ws=ws)]
    b = [B.conv2d_fwd(gx, gw, st, pd, dl, ws=ws), B.conv2d_dgrad(gdy, gw, x.shape, st, pd, dl, ws=ws),
         B.conv2d_wgrad(gx, gdy, w.shape, st, pd, dl, ws=ws)]
    torch.cuda.synchronize()
    for u, v in zip(a, b):
        assert torch.equal(u.view(torch.uint8 if u.dtype != torch.float32 else torch.float32).flatten(),
                           v.view(torch.uint8 if v.dtype != torch.float32 else torch.float32).flatten())


# N, C, H, W
# Shapes for the convolution + batch-norm statistics hand-over: one per kernel family with a statistics epilogue,
# plus shapes that take the separate reduction pass.
STATS_SHAPES = [
    ("bf16", (3, 64, 20, 24, 64, 3, 3, 1, 1, 1)),      # bf16 3x3 64->64 (two-group halo kernel), several tiles per block
    ("f32", (2, 64, 16, 32, 64, 3, 3, 1, 1, 1)),       # fp32 row-aligned halo kernel
    ("bf16", (2, 128, 9, 9, 256, 1, 1, 1, 0, 1)),      # generic kernel, 128x128 tiles
    ("bf16", (2, 32, 16, 16, 64, 3, 3, 2, 1, 1)),      # generic kernel, 128x64 tiles, stride 2
    ("f32", (2, 16, 15, 15, 32, 1, 1, 2, 0, 1)),       # generic kernel, fp32, 256x32 tiles, ragged
    ("bf16", (2, 3, 20, 24, 64, 7, 7, 2, 3, 1)),       # image stem (space-to-depth + halo kernel)
    ("bf16", (1, 5, 9, 9, 7, 3, 3, 3, 1, 1)),          # scalar epilogue: separate reduction pass
    ("f32", (2, 3, 30, 30, 16, 3, 3, 1, 1, 1)),        # 3-channel stem on the generic path
]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("big", [False, True])
@pytest.mark.parametrize("i", range(len(STATS_SHAPES)))
def test_conv_statistics_feed_the_batch_norm(i, big, layout, nsk_env):
    """nsk_conv2d_fwd_stats leaves per-channel partial sums of its stored output; nsk_bn_relu_add_fwd_stats takes its
    batch statistics from them.  y must equal the plain forward bit for bit, the partial sums must add up to the
    sums of the stored y, and the batch-norm results must agree with the plain call (which reads y once more) and
    with the oracle."""
    dtype, (N, C, H, W, K, R, S, st, pd, dl) = STATS_SHAPES[i]
    nsk_env("NSK_STATS_ALWAYS", "1")     # the generic kernel's statistics epilogue also for short reductions
    if big:
        if dtype != "bf16" or C % 64 or K % 64:
            pytest.skip("the large-tile kernel takes bf16 layers with channel counts that are multiples of 64")
        nsk_env("NSK_BIG_MIN_TILES", "1")
    print(f"stats case {STATS_SHAPES[i]} big={big} layout={layout}", flush=True)
    x = on_grid(gen.normal(900 + i, 0, (N, C, H, W)), dtype)
    w = on_grid(gen.he_normal(900 + i, 1, (K, C, R, S)), dtype)
    g = (1.0 + 0.3 * gen.normal(900 + i, 3, (K,))).astype(np.float32)
    b = (0.2 * gen.normal(900 + i, 4, (K,))).astype(np.float32)
    ws = B.Workspace()
    gx, gw = to_gpu(x, dtype, layout), to_gpu(w, dtype, layout)
    gg, gb = torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda()
    y0 = B.conv2d_fwd(gx, gw, st, pd, dl, layout, ws=ws)
    y1, stats = B.conv2d_fwd_stats(gx, gw, st, pd, dl, layout, ws=ws)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    yh = to_host(y1, layout)                                   # NCHW float64 of the stored values
    sums = stats.double().sum(dim=1).cpu().numpy()             # [2, K]
    want0, want1 = yh.sum(axis=(0, 2, 3)), (yh * yh).sum(axis=(0, 2, 3))
    scale0 = np.sqrt(want1 * yh[:, 0].size) + 1e-30            # sum of n terms of rms r: compare on the scale n*r... sqrt(n*sum sq)
    assert np.max(np.abs(sums[0] - want0) / scale0) <= 1e-6
    assert np.max(np.abs(sums[1] - want1) / (want1 + 1e-30)) <= 1e-5
    out0, mean0, inv0 = B.bn_relu_add_fwd(y1, gg, gb, None, 1e-5, True, layout, ws=ws)
    out1, mean1, inv1 = B.bn_relu_add_fwd(y1, gg, gb, None, 1e-5, True, layout, ws=ws, stats=stats)
    torch.cuda.synchronize()
    assert max_rel_err(mean1.cpu().numpy(), mean0.cpu().numpy()) <= 1e-5
    assert max_rel_err(inv1.cpu().numpy(), inv0.cpu().numpy()) <= 1e-5
    # the oracle's batch-norm of the ORACLE's convolution output (on the storage grid); the mean is compared on the
    # scale that matters for the normalised value (a shift of the mean by d moves xhat by d * invstd)
    y_want = on_grid(oracle.conv2d_fwd(x, w, st, pd, dl).astype(np.float32), dtype)
    want_out, want_mean, want_inv = oracle.bn_relu_add_fwd(y_want, g, b, None, 1e-5, True)
    stat_tol = 1e-5 if dtype == "f32" else 2e-4
    assert np.max(np.abs(mean1.cpu().numpy() - want_mean) * want_inv) <= stat_tol
    assert max_rel_err(inv1.cpu().numpy(), want_inv) <= stat_tol
    assert max_rel_err(to_host(out1, layout), want_out) <= TOL[dtype]


@pytest.mark.parametrize("dtype,offset,least", [("f32", 6.0, 25), ("f32", 20.0, 80), ("bf16", 3.0, 12)])
def test_fused_statistics_with_a_strongly_offset_convolution_output(dtype, offset, least):
    """The statistics epilogues add UNSHIFTED float partial sums and the variance is E[y^2] - E[y]^2 in double
    precision, which loses accuracy as |mean| / sigma grows.  A padded 3x3 layer cannot get there (its border
    outputs see fewer taps, which bounds |mean| / sigma near 7), a 1x1 layer can: an all-positive input
    (N(0,1) + offset) through a 1x1 filter with a positive mean gives channel means of tens to more than a hundred
    standard deviations.  A float partial sum of y^2 is good to about half an ulp (3e-8), which is 3e-8 * (mean /
    sigma)^2 of the variance: the fused chain must stay inside 4e-8 * (mean / sigma)^2 against the oracle (the header states
    it: 1e-4 of invstd at about 80 standard deviations)."""
    N, C, H, W, K = 4, 64, 16, 32, 64
    x = on_grid(gen.normal(950, 0, (N, C, H, W)) + offset, dtype)
    w = on_grid(gen.he_normal(950, 1, (K, C, 1, 1)) + 0.05, dtype)
    g = (1.0 + 0.3 * gen.normal(950, 3, (K,))).astype(np.float32)
    b = (0.2 * gen.normal(950, 4, (K,))).astype(np.float32)
    y_want = on_grid(oracle.conv2d_fwd(x, w, 1, 0, 1).astype(np.float32), dtype)
    want_out, want_mean, want_inv = oracle.bn_relu_add_fwd(y_want, g, b, None, 1e-5, True)
    ratio = float(np.max(np.abs(want_mean) * want_inv))
    print(f"offset {offset} {dtype}: |mean| / sigma up to {ratio:.0f}", flush=True)
    assert ratio > least
    ws = B.Workspace()
    gx, gw = to_gpu(x, dtype, B.NSK_NHWC), to_gpu(w, dtype, B.NSK_NHWC)
    y, stats = B.conv2d_fwd_stats(gx, gw, 1, 0, 1, ws=ws)
    out, mean, inv = B.bn_relu_add_fwd(y, torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda(), None, 1e-5, True,
                                       ws=ws, stats=stats)
    torch.cuda.synchronize()
    assert max_rel_err(to_host(y, B.NSK_NHWC), y_want) <= TOL[dtype]
    stat_tol = max(1e-5, 4e-8 * ratio * ratio) if dtype == "f32" else 2e-3
    assert max_rel_err(inv.cpu().numpy(), want_inv) <= stat_tol
    assert np.max(np.abs(mean.cpu().numpy() - want_mean) * want_inv) <= stat_tol
    # out = gamma * xhat + beta with xhat = (y - mean) * invstd: relative errors d_inv of invstd and d_mean * invstd
    # of the mean move out by gamma * (|xhat| * d_inv + d_mean * invstd)
    out_tol = TOL[dtype] if dtype == "bf16" else TOL[dtype] + 2 * stat_tol
    assert max_rel_err(to_host(out, B.NSK_NHWC), want_out) <= out_tol


# conv -> batch-norm -> ReLU -> conv with the normalised activation never stored: the second convolution and its
# backward-weight call apply it to the raw output of the first on load, the batch-norm's backward pass takes the ReLU
# mask from there.  dtype, (N, C, H, W) of the raw tensor, K, R, stride, pad of the consuming convolution
ACT_SHAPES = [
    ("f32", (4, 64, 16, 32), 64, 3, 1, 1),      # fp32 3x3 64->64 on 32-wide images: kernels with the fused operand load
    ("f32", (128, 64, 32, 32), 64, 3, 1, 1),    # the same at the size of the configured block: several tiles per block
    ("bf16", (3, 64, 20, 24), 64, 3, 1, 1),     # no fused load for this layer: activation applied into the workspace
    ("f32", (2, 16, 15, 17), 32, 3, 2, 1),      # strided consumer, generic kernels
    ("bf16", (2, 256, 9, 9), 64, 1, 1, 0),      # 1x1 consumer
]


@pytest.mark.parametrize("i", range(len(ACT_SHAPES)))
def test_fused_activation_calls(i):
    dtype, shape, K, R, stride, pad = ACT_SHAPES[i]
    N, C, H, W = shape
    print(f"fused activation case {ACT_SHAPES[i]}", flush=True)
    seed = 1700 + i
    y_raw = on_grid(1.3 * gen.normal(seed, 0, shape) + 0.2, dtype)
    g = (1.0 + 0.3 * gen.normal(seed, 1, (C,))).astype(np.float32)
    b = (0.2 * gen.normal(seed, 2, (C,))).astype(np.float32)
    w = on_grid(gen.he_normal(seed, 3, (K, C, R, R)), dtype)
    # the oracle's chain: batch-norm + ReLU (stored on the grid), then the convolution and its backward passes
    a_want, mean_want, inv_want = oracle.bn_relu_add_fwd(y_raw, g, b, None, 1e-5, True)
    a_grid = on_grid(a_want.astype(np.float32), dtype)
    z_want = oracle.conv2d_fwd(a_grid, w, stride, pad, 1)
    dz = on_grid(gen.normal(seed, 4, z_want.shape), dtype)
    dw_want = oracle.conv2d_wgrad(a_grid, dz, w.shape, stride, pad, 1)
    da = on_grid(gen.normal(seed, 5, shape), dtype)                       # gradient arriving at the activation
    m32, i32 = mean_want.astype(np.float32), inv_want.astype(np.float32)
    dy_want, _, dg_want, db_want = oracle.bn_relu_add_bwd(y_raw, a_grid, da, g, m32, i32, True, want_dresidual=False)
    # input of nsk_bn_fwd_coeffs: one row of partial sums of the raw tensor (exact sums, rounded to float)
    y64 = y_raw.astype(np.float64)
    stats = np.stack([y64.sum(axis=(0, 2, 3)), (y64 * y64).sum(axis=(0, 2, 3))]).astype(np.float32).reshape(2, 1, C)
    ws = B.Workspace()
    gy, gw = to_gpu(y_raw, dtype, B.NSK_NHWC), to_gpu(w, dtype, B.NSK_NHWC)
    gg, gb = torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda()
    mean, inv, coeffs = B.bn_fwd_coeffs(gy, gg, gb, torch.from_numpy(stats).cuda(), 1e-5, ws=ws)
    assert max_rel_err(mean.cpu().numpy(), mean_want) <= 1e-5
    assert max_rel_err(inv.cpu().numpy(), inv_want) <= 1e-5
    z, zstats = B.conv2d_fwd_act(gy, coeffs, gw, stride, pad, 1, want_stats=True, ws=ws)
    z_plain = B.conv2d_fwd_act(gy, coeffs, gw, stride, pad, 1, ws=ws)
    dw = B.conv2d_wgrad_act(gy, coeffs, to_gpu(dz, dtype, B.NSK_NHWC), w.shape, stride, pad, 1, ws=ws)
    dy, dg, db = B.bn_relu_bwd_act(gy, coeffs, to_gpu(da, dtype, B.NSK_NHWC), gg, mean, inv, ws=ws)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert max_rel_err(to_host(z, B.NSK_NHWC), z_want) <= tol
    assert torch.equal(z, z_plain)
    zs = zstats.double().sum(dim=1).cpu().numpy()
    zh = to_host(z, B.NSK_NHWC)
    assert np.max(np.abs(zs[0] - zh.sum(axis=(0, 2, 3))) / (np.sqrt((zh * zh).sum(axis=(0, 2, 3)) * zh[:, 0].size) + 1e-30)) <= 1e-5
    assert max_rel_err(to_host(dw, B.NSK_NHWC), dw_want) <= tol
    assert max_rel_err(to_host(dy, B.NSK_NHWC), dy_want) <= tol
    assert max_rel_err(dg.cpu().numpy(), dg_want) <= 1e-4
    assert max_rel_err(db.cpu().numpy(), db_want) <= 1e-4


BN_SHAPES = [(4, 64, 9, 11), (3, 16, 16, 16), (2, 256, 7, 7), (2, 1024, 5, 5), (5, 24, 6, 7), (2, 3, 10, 10),
             (3, 40, 33, 17)]


def _bn_case(i, dtype):
    shape = BN_SHAPES[i]
    x = on_grid(1.7 * gen.normal(700 + i, 0, shape) + 0.6, dtype)
    r = on_grid(gen.normal(700 + i, 1, shape), dtype)
    dout = on_grid(gen.normal(700 + i, 2, shape), dtype)
    g = (1.0 + 0.3 * gen.normal(700 + i, 3, (shape[1],))).astype(np.float32)
    b = (0.2 * gen.normal(700 + i, 4, (shape[1],))).astype(np.float32)
    return x, r, dout, g, b


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("relu,with_res", [(True, True), (True, False), (False, True), (False, False)])
@pytest.mark.parametrize("i", range(len(BN_SHAPES)))
def test_bn_relu_add_fwd_bwd(i, relu, with_res, dtype, layout):
    x, r, dout, g, b = _bn_case(i, dtype)
    print(f"bn case {BN_SHAPES[i]} relu={relu} res={with_res} {dtype} layout={layout}", flush=True)
    tol = TOL[dtype]
    ws = B.Workspace()
    gx, gr, gd = to_gpu(x, dtype, layout), to_gpu(r, dtype, layout), to_gpu(dout, dtype, layout)
    gg, gb = torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda()
    rm = torch.full((x.shape[1],), 0.5, device="cuda:0")
    rv = torch.full((x.shape[1],), 2.0, device="cuda:0")
    out_view, out_check = guarded(gx.shape, torch_dtype(dtype))
    out, mean, invstd = B.bn_relu_add_fwd(gx, gg, gb, gr if with_res else None, 1e-5, relu, layout,
                                          running_mean=rm, running_var=rv, out=out_view, ws=ws)
    torch.cuda.synchronize()
    out_check()
    orm, orv = np.full(x.shape[1], 0.5), np.full(x.shape[1], 2.0)
    want_out, want_mean, want_invstd = oracle.bn_relu_add_fwd(x, g, b, r if with_res else None, 1e-5, relu,
                                                              running_mean=orm, running_var=orv)
    got_out = to_host(out, layout)
    assert max_rel_err(got_out, want_out) <= tol
    assert max_rel_err(mean.cpu().numpy(), want_mean) <= 1e-5
    assert max_rel_err(invstd.cpu().numpy(), want_invstd) <= 1e-5
    assert max_rel_err(rm.cpu().numpy(), orm) <= 1e-5
    assert max_rel_err(rv.cpu().numpy(), orv) <= 1e-5

    # backward from the oracle's stored forward result (on the storage grid), so that both sides take
    # the ReLU mask from the same `out`
    out_grid = on_grid(want_out.astype(np.float32), dtype)
    g_out = to_gpu(out_grid, dtype, layout)
    dx_view, dx_check = guarded(gx.shape, torch_dtype(dtype))
    dx, dres, dg, db = B.bn_relu_add_bwd(gx, g_out, gd, gg, torch.from_numpy(want_mean.astype(np.float32)).cuda(),
                                         torch.from_numpy(want_invstd.astype(np.float32)).cuda(), relu, layout,
                                         dx=dx_view, want_dresidual=with_res, ws=ws)
    torch.cuda.synchronize()
    dx_check()
    wdx, wdres, wdg, wdb = oracle.bn_relu_add_bwd(x, out_grid, dout, g, want_mean.astype(np.float32),
                                                  want_invstd.astype(np.float32), relu, want_dresidual=with_res)
    assert max_rel_err(to_host(dx, layout), wdx) <= tol
    assert max_rel_err(dg.cpu().numpy(), wdg) <= 1e-4
    assert max_rel_err(db.cpu().numpy(), wdb) <= 1e-4
    if with_res:
        assert np.array_equal(to_host(dres, layout), wdres)      # a masked copy: exact
    else:
        assert dres is None


POOL_SHAPES = [(2, 64, 20, 20), (1, 16, 13, 17), (2, 5, 9, 9), (1, 8, 6, 6)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("with_res", [True, False])
@pytest.mark.parametrize("i", [0, 1, 2, 3])
def test_bn_relu_mask_calls_match_the_plain_calls(i, with_res, dtype):
    """The *_mask entry points hand the ReLU mask from forward to backward (one byte per 16-byte vector): the mask must
    equal out > 0 element for element and every result must equal the plain calls bit for bit (same kernels, same
    order of operations)."""
    x, r, dout, g, b = _bn_case(i, dtype)
    layout = B.NSK_NHWC
    print(f"bn mask case {BN_SHAPES[i]} res={with_res} {dtype}", flush=True)
    ws = B.Workspace()
    gx, gr, gd = to_gpu(x, dtype, layout), to_gpu(r, dtype, layout), to_gpu(dout, dtype, layout)
    gg, gb = torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda()
    res = gr if with_res else None
    nbytes = B.bn_mask_bytes(gx, layout, True)
    vec = 8 if dtype == "bf16" else 4
    assert nbytes == gx.numel() // vec
    assert B.bn_mask_bytes(gx, layout, False) == 0 and B.bn_mask_bytes(gx, B.NSK_NCHW, True) == 0
    raw_mask = torch.full((nbytes + 1024,), 0xAA, dtype=torch.uint8, device="cuda:0")   # canaries on both sides
    mask_view = raw_mask[512:512 + nbytes]

    def mask_check():
        assert bool((raw_mask[:512] == 0xAA).all()) and bool((raw_mask[512 + nbytes:] == 0xAA).all())

    out0, mean0, inv0 = B.bn_relu_add_fwd(gx, gg, gb, res, 1e-5, True, layout, ws=ws)
    out1, mean1, inv1 = B.bn_relu_add_fwd(gx, gg, gb, res, 1e-5, True, layout, ws=ws, relu_mask=mask_view)
    torch.cuda.synchronize()
    mask_check()
    assert torch.equal(out0, out1) and torch.equal(mean0, mean1) and torch.equal(inv0, inv1)
    bits = (out1.reshape(-1, vec).float() > 0).to(torch.int32)
    want_mask = (bits << torch.arange(vec, device="cuda:0", dtype=torch.int32)).sum(dim=1).to(torch.uint8)
    assert torch.equal(mask_view, want_mask)
    dx0, dr0, dg0, db0 = B.bn_relu_add_bwd(gx, out0, gd, gg, mean0, inv0, True, layout, want_dresidual=with_res, ws=ws)
    dx1, dr1, dg1, db1 = B.bn_relu_add_bwd(gx, None, gd, gg, mean0, inv0, True, layout, want_dresidual=with_res, ws=ws,
                                           relu_mask=mask_view)
    torch.cuda.synchronize()
    assert torch.equal(dx0, dx1) and torch.equal(dg0, dg1) and torch.equal(db0, db1)
    if with_res:
        assert torch.equal(dr0, dr1)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("i", range(len(POOL_SHAPES)))
def test_maxpool_fwd_bwd(i, dtype, layout):
    shape = POOL_SHAPES[i]
    x = on_grid(np.maximum(gen.normal(800 + i, 0, shape), 0.0), dtype)     # post-ReLU-like: many tied zeros
    gx = to_gpu(x, dtype, layout)
    y, idx = B.maxpool2d_fwd(gx, 3, 2, 1, layout)
    wy, widx = oracle.maxpool2d_fwd(x, 3, 2, 1)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(y, layout), wy)
    got_idx = idx.cpu()
    if layout == B.NSK_NHWC:
        got_idx = got_idx.permute(0, 3, 1, 2)
    assert np.array_equal(got_idx.numpy(), widx)
    dy = on_grid(gen.normal(800 + i, 1, wy.shape), dtype)
    dx = B.maxpool2d_bwd(to_gpu(dy, dtype, layout), idx, shape, 3, 2, 1, layout)
    torch.cuda.synchronize()
    assert max_rel_err(to_host(dx, layout), oracle.maxpool2d_bwd(dy, widx, shape, 3, 2, 1)) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("i", [0, 1, 3])
def test_maxpool_3x3_on_the_general_kernel(i, dtype, nsk_env):
    """The 3x3 fast path of the forward pool switched off: the general kernel must give the same bits."""
    nsk_env("NSK_POOL_GENERAL", "1")
    test_maxpool_fwd_bwd(i, dtype, B.NSK_NHWC)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("i", FEW_CHANNELS)
def test_few_channel_shapes_on_the_generic_kernels(i, dtype, nsk_env):
    """The direct kernels for layers with at most four channels on one side switched off."""
    nsk_env("NSK_NO_TINY", "1")
    test_conv_fwd_dgrad_wgrad(i, dtype, B.NSK_NHWC)

