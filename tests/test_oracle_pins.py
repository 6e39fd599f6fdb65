"""Pins for the CPU oracle: things fixed by mathematics or by an independent library routine.

The paper prints no numeric example of its convolution / batch-norm path (it hands the
work to a vendor library, section "Experiments and Discussion"), so the oracle is pinned by
hand-derived closed forms (tests/golden), the 1x1-convolution == matrix-product identity
(the paper's `@` operator multiplies by the transposed weight, section "Automatic
Differentiation"), the adjoint identity, finite differences, structural identities
(stride = subsampling, dilation = zero-stuffed filter), scipy's correlate2d and torch's
CPU float64 operators with autograd.  None of these re-types the oracle's loops.
"""
import os

import numpy as np
import pytest
import scipy.signal
import torch
import torch.nn.functional as F

import nsk_inputs as gen
import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")

# (N, C, H, W, K, R, S, stride, pad, dilation): tiny shapes incl. stride 2, pad 3, dilation 2,
# non-square images and filters, C = 3, odd extents.
SHAPES = [
    (2, 3, 7, 9, 4, 3, 3, (1, 1), (1, 1), (1, 1)),
    (2, 4, 8, 8, 5, 3, 3, (2, 2), (1, 1), (1, 1)),
    (1, 3, 13, 11, 6, 7, 7, (2, 2), (3, 3), (1, 1)),
    (2, 5, 9, 7, 3, 1, 1, (2, 2), (0, 0), (1, 1)),
    (2, 2, 10, 9, 3, 3, 2, (1, 2), (2, 0), (2, 1)),
    (1, 4, 6, 6, 4, 3, 3, (1, 1), (2, 2), (2, 2)),
    (3, 6, 5, 5, 2, 1, 1, (1, 1), (0, 0), (1, 1)),
    (1, 2, 9, 12, 3, 2, 3, (3, 2), (1, 2), (1, 2)),
]


def _rand(seed, *shapes):
    return [gen.normal(seed, i, s).astype(np.float64) for i, s in enumerate(shapes)]


def _case(i):
    N, C, H, W, K, R, S, st, pd, dl = SHAPES[i]
    x, w = _rand(100 + i, (N, C, H, W), (K, C, R, S))
    P, Q = oracle.conv2d_out_dims(x.shape, w.shape, st, pd, dl)
    dy = gen.normal(100 + i, 9, (N, K, P, Q)).astype(np.float64)
    return x, w, dy, st, pd, dl


# ----------------------------------------------------------------------------- conv forward

def test_out_dims_formula_cases():
    # 224 -> 112 for 7x7 s2 p3 ; 112 -> 56 for 3x3 s2 p1 ; filter larger than padded image -> 0
    assert oracle.conv2d_out_dims((1, 3, 224, 224), (64, 3, 7, 7), 2, 3, 1) == (112, 112)
    assert oracle.conv2d_out_dims((1, 3, 112, 112), (1, 3, 3, 3), 2, 1, 1) == (56, 56)
    assert oracle.conv2d_out_dims((1, 1, 2, 2), (1, 1, 5, 5), 1, 0, 1) == (0, 0)
    assert oracle.conv2d_out_dims((1, 1, 7, 7), (1, 1, 3, 3), 1, 0, 2) == (3, 3)


def test_golden_ones_3x3():
    want = np.loadtxt(os.path.join(GOLD, "conv_ones_3x3_pad1.txt"))
    y = oracle.conv2d_fwd(np.ones((1, 1, 3, 3)), np.ones((1, 1, 3, 3)), 1, 1, 1)
    assert np.array_equal(y[0, 0], want)


def test_golden_ramp_stride2_no_flip():
    want = np.loadtxt(os.path.join(GOLD, "conv_ramp_2x2_stride2.txt"))
    x = np.arange(16.0).reshape(1, 1, 4, 4)
    w = np.array([[1.0, 2.0], [3.0, 4.0]]).reshape(1, 1, 2, 2)
    y = oracle.conv2d_fwd(x, w, 2, 0, 1)
    assert np.array_equal(y[0, 0], want)


def test_delta_filter_shifts_the_image():
    x = _rand(7, (2, 3, 6, 5))[0]
    for r in range(3):
        for s in range(3):
            w = np.zeros((3, 3, 3, 3))
            for c in range(3):
                w[c, c, r, s] = 1.0
            y = oracle.conv2d_fwd(x, w, 1, 1, 1)
            want = np.zeros_like(x)
            xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)))
            want[:] = xp[:, :, r:r + 6, s:s + 5]
            assert np.array_equal(y, want)


def test_1x1_conv_is_matmul_with_transposed_weight():
    x, w = _rand(11, (3, 6, 5, 4), (7, 6, 1, 1))
    y = oracle.conv2d_fwd(x, w, 1, 0, 1)
    X = x.transpose(0, 2, 3, 1).reshape(-1, 6)       # [M, C]
    Y = X @ w.reshape(7, 6).T                        # [M, K] = X . W^T
    want = Y.reshape(3, 5, 4, 7).transpose(0, 3, 1, 2)
    np.testing.assert_allclose(y, want, rtol=1e-13, atol=1e-13)


def test_valid_correlation_matches_scipy():
    x, w = _rand(12, (2, 3, 9, 8), (4, 3, 3, 4))
    y = oracle.conv2d_fwd(x, w, 1, 0, 1)
    for n in range(2):
        for k in range(4):
            want = sum(scipy.signal.correlate2d(x[n, c], w[k, c], mode="valid") for c in range(3))
            np.testing.assert_allclose(y[n, k], want, rtol=1e-12, atol=1e-12)


def test_stride_is_subsampling_and_dilation_is_zero_stuffing():
    x, w = _rand(13, (2, 3, 11, 10), (4, 3, 3, 3))
    full = oracle.conv2d_fwd(x, w, 1, 1, 1)
    strided = oracle.conv2d_fwd(x, w, (2, 3), 1, 1)
    assert np.array_equal(strided, full[:, :, ::2, ::3])
    stuffed = np.zeros((4, 3, 5, 5))
    stuffed[:, :, ::2, ::2] = w
    a = oracle.conv2d_fwd(x, w, 1, 2, 2)
    b = oracle.conv2d_fwd(x, stuffed, 1, 2, 1)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)


def test_linearity_and_shift_equivariance():
    x1, x2, w = _rand(14, (1, 2, 8, 8), (1, 2, 8, 8), (3, 2, 3, 3))
    y = oracle.conv2d_fwd(2.0 * x1 - 3.0 * x2, w, 1, 0, 1)
    want = 2.0 * oracle.conv2d_fwd(x1, w, 1, 0, 1) - 3.0 * oracle.conv2d_fwd(x2, w, 1, 0, 1)
    np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-12)
    # shifting the image by one pixel shifts the valid output by one pixel
    ys = oracle.conv2d_fwd(x1[:, :, 1:, 1:], w, 1, 0, 1)
    y0 = oracle.conv2d_fwd(x1, w, 1, 0, 1)
    assert np.array_equal(ys, y0[:, :, 1:, 1:])


@pytest.mark.parametrize("i", range(len(SHAPES)))
def test_fwd_matches_torch_float64(i):
    x, w, dy, st, pd, dl = _case(i)
    y = oracle.conv2d_fwd(x, w, st, pd, dl)
    want = F.conv2d(torch.from_numpy(x), torch.from_numpy(w), None, st, pd, dl).numpy()
    assert y.shape == want.shape
    np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------------------- conv backward

@pytest.mark.parametrize("i", range(len(SHAPES)))
def test_adjoint_identity(i):
    x, w, dy, st, pd, dl = _case(i)
    y = oracle.conv2d_fwd(x, w, st, pd, dl)
    dx = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl)
    dw = oracle.conv2d_wgrad(x, dy, w.shape, st, pd, dl)
    a, b, c = np.vdot(y, dy), np.vdot(x, dx), np.vdot(w, dw)
    scale = np.sqrt(np.vdot(y, y) * np.vdot(dy, dy))
    assert abs(a - b) <= 1e-12 * scale
    assert abs(a - c) <= 1e-12 * scale


@pytest.mark.parametrize("i", range(len(SHAPES)))
def test_gradients_match_central_differences(i):
    # L = <conv(x,w), dy> is bilinear, so a central difference is exact up to rounding.
    x, w, dy, st, pd, dl = _case(i)
    dx = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl)
    dw = oracle.conv2d_wgrad(x, dy, w.shape, st, pd, dl)
    rng = np.random.default_rng(i)
    h = 0.5
    for _ in range(12):
        j = tuple(rng.integers(0, s) for s in x.shape)
        e = np.zeros_like(x)
        e[j] = h
        fd = (np.vdot(oracle.conv2d_fwd(x + e, w, st, pd, dl), dy)
              - np.vdot(oracle.conv2d_fwd(x - e, w, st, pd, dl), dy)) / (2 * h)
        assert abs(fd - dx[j]) <= 1e-10 * max(1.0, abs(fd))
        j = tuple(rng.integers(0, s) for s in w.shape)
        e = np.zeros_like(w)
        e[j] = h
        fd = (np.vdot(oracle.conv2d_fwd(x, w + e, st, pd, dl), dy)
              - np.vdot(oracle.conv2d_fwd(x, w - e, st, pd, dl), dy)) / (2 * h)
        assert abs(fd - dw[j]) <= 1e-10 * max(1.0, abs(fd))


@pytest.mark.parametrize("i", range(len(SHAPES)))
def test_gradients_match_torch_autograd(i):
    x, w, dy, st, pd, dl = _case(i)
    tx = torch.from_numpy(x).requires_grad_(True)
    tw = torch.from_numpy(w).requires_grad_(True)
    F.conv2d(tx, tw, None, st, pd, dl).backward(torch.from_numpy(dy))
    dx = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl)
    dw = oracle.conv2d_wgrad(x, dy, w.shape, st, pd, dl)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dw, tw.grad.numpy(), rtol=1e-12, atol=1e-12)


def test_dgrad_of_1x1_stride2_is_zero_off_the_sampling_grid():
    N, C, H, W, K, R, S, st, pd, dl = SHAPES[3]
    x, w, dy, st, pd, dl = _case(3)
    dx = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl)
    assert np.all(dx[:, :, 1::2, :] == 0.0)
    assert np.all(dx[:, :, :, 1::2] == 0.0)
    # on the grid it is the transposed 1x1 matmul
    want = np.einsum("nkpq,kc->ncpq", dy, w[:, :, 0, 0])
    np.testing.assert_allclose(dx[:, :, ::2, ::2], want, rtol=1e-13, atol=1e-13)


def test_accumulate_adds_to_existing_gradient():
    x, w, dy, st, pd, dl = _case(1)
    dx = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl)
    dw = oracle.conv2d_wgrad(x, dy, w.shape, st, pd, dl)
    bx, bw = _rand(55, x.shape, w.shape)
    ax, aw = bx.copy(), bw.copy()
    oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl, into=ax)
    oracle.conv2d_wgrad(x, dy, w.shape, st, pd, dl, into=aw)
    np.testing.assert_allclose(ax, bx + dx, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(aw, bw + dw, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("i", range(len(SHAPES)))
def test_sampled_evaluation_equals_full(i):
    x, w, dy, st, pd, dl = _case(i)
    y = oracle.conv2d_fwd(x, w, st, pd, dl)
    dx = oracle.conv2d_dgrad(dy, w, x.shape, st, pd, dl)
    dw = oracle.conv2d_wgrad(x, dy, w.shape, st, pd, dl)
    cy = gen.sample_coords(1, 0, y.shape, 64)
    cx = gen.sample_coords(1, 1, x.shape, 64)
    cw = gen.sample_coords(1, 2, w.shape, 64)
    np.testing.assert_allclose(oracle.conv2d_fwd_at(x, w, cy, st, pd, dl), y[tuple(cy.T)], rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.conv2d_dgrad_at(dy, w, x.shape, cx, st, pd, dl), dx[tuple(cx.T)],
                               rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.conv2d_wgrad_at(x, dy, w.shape, cw, st, pd, dl), dw[tuple(cw.T)],
                               rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------------------- batch-norm + ReLU + add

def _bn_case(seed, shape=(4, 5, 6, 7)):
    x = 2.0 * gen.normal(seed, 0, shape).astype(np.float64) + 0.7
    r = gen.normal(seed, 1, shape).astype(np.float64)
    g = 1.0 + 0.3 * gen.normal(seed, 2, (shape[1],)).astype(np.float64)
    b = 0.2 * gen.normal(seed, 3, (shape[1],)).astype(np.float64)
    dout = gen.normal(seed, 4, shape).astype(np.float64)
    return x, r, g, b, dout


def test_bn_closed_forms():
    x, r, g, b, _ = _bn_case(21)
    eps = 1e-5
    out, mean, invstd = oracle.bn_relu_add_fwd(x, g, b, None, eps, relu=False)
    np.testing.assert_allclose(mean, x.mean(axis=(0, 2, 3)), rtol=1e-13, atol=1e-13)
    var = x.var(axis=(0, 2, 3))            # numpy's default is the biased variance
    np.testing.assert_allclose(invstd, 1.0 / np.sqrt(var + eps), rtol=1e-13)
    np.testing.assert_allclose(out.mean(axis=(0, 2, 3)), b, atol=1e-13)
    np.testing.assert_allclose(out.var(axis=(0, 2, 3)), g * g * var / (var + eps), rtol=1e-12)
    # constant input -> out == beta ; affine change of x leaves out unchanged up to eps
    const = np.full_like(x, 3.25)
    oc, _, _ = oracle.bn_relu_add_fwd(const, g, b, None, eps, relu=False)
    np.testing.assert_allclose(oc, np.broadcast_to(b[None, :, None, None], x.shape), atol=1e-12)
    o1, _, _ = oracle.bn_relu_add_fwd(x, g, b, None, 0.0, relu=False)
    o2, _, _ = oracle.bn_relu_add_fwd(5.0 * x - 2.0, g, b, None, 0.0, relu=False)
    np.testing.assert_allclose(o1, o2, rtol=1e-11, atol=1e-11)


def test_bn_relu_and_residual_order():
    x, r, g, b, _ = _bn_case(22)
    plain, _, _ = oracle.bn_relu_add_fwd(x, g, b, None, 1e-5, relu=False)
    both, _, _ = oracle.bn_relu_add_fwd(x, g, b, r, 1e-5, relu=True)
    assert np.all(both >= 0.0)
    np.testing.assert_allclose(both, np.maximum(plain + r, 0.0), rtol=0, atol=1e-14)


def test_bn_running_stats_use_unbiased_variance():
    x, r, g, b, _ = _bn_case(23)
    rm = np.full(5, 0.5)
    rv = np.full(5, 2.0)
    oracle.bn_relu_add_fwd(x, g, b, None, 1e-5, relu=False, momentum=0.1, running_mean=rm, running_var=rv)
    np.testing.assert_allclose(rm, 0.9 * 0.5 + 0.1 * x.mean(axis=(0, 2, 3)), rtol=1e-13)
    np.testing.assert_allclose(rv, 0.9 * 2.0 + 0.1 * x.var(axis=(0, 2, 3), ddof=1), rtol=1e-13)


@pytest.mark.parametrize("relu,with_res", [(False, False), (True, False), (True, True), (False, True)])
def test_bn_matches_torch_autograd(relu, with_res):
    x, r, g, b, dout = _bn_case(24)
    eps = 1e-5
    tx = torch.from_numpy(x).requires_grad_(True)
    tg = torch.from_numpy(g).requires_grad_(True)
    tb = torch.from_numpy(b).requires_grad_(True)
    tr = torch.from_numpy(r).requires_grad_(True)
    z = F.batch_norm(tx, None, None, tg, tb, training=True, momentum=0.1, eps=eps)
    if with_res:
        z = z + tr
    if relu:
        z = torch.relu(z)
    z.backward(torch.from_numpy(dout))
    out, mean, invstd = oracle.bn_relu_add_fwd(x, g, b, r if with_res else None, eps, relu=relu)
    np.testing.assert_allclose(out, z.detach().numpy(), rtol=1e-11, atol=1e-11)
    dx, dres, dg, db = oracle.bn_relu_add_bwd(x, out, dout, g, mean, invstd, relu=relu, want_dresidual=with_res)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(dg, tg.grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-10, atol=1e-10)
    if with_res:
        np.testing.assert_allclose(dres, tr.grad.numpy(), rtol=0, atol=1e-13)
    else:
        assert dres is None


def test_bn_backward_invariants_and_add_rule():
    x, r, g, b, dout = _bn_case(25)
    out, mean, invstd = oracle.bn_relu_add_fwd(x, g, b, None, 1e-5, relu=False)
    dx, _, dg, db = oracle.bn_relu_add_bwd(x, out, dout, g, mean, invstd, relu=False)
    xhat = (x - mean[None, :, None, None]) * invstd[None, :, None, None]
    assert np.abs(dx.sum(axis=(0, 2, 3))).max() < 1e-11
    # sum(xhat^2)/M = var/(var+eps), so sum(dx*xhat) = gamma*invstd*dgamma*eps*invstd^2 (zero only at eps = 0)
    np.testing.assert_allclose((dx * xhat).sum(axis=(0, 2, 3)), g * invstd * dg * 1e-5 * invstd ** 2,
                               rtol=1e-6, atol=1e-12)
    np.testing.assert_allclose(db, dout.sum(axis=(0, 2, 3)), rtol=1e-12)
    np.testing.assert_allclose(dg, (dout * xhat).sum(axis=(0, 2, 3)), rtol=1e-11, atol=1e-11)
    # the gradient of the add goes unchanged to the residual operand, masked by the ReLU
    out2, mean, invstd = oracle.bn_relu_add_fwd(x, g, b, r, 1e-5, relu=True)
    _, dres, _, _ = oracle.bn_relu_add_bwd(x, out2, dout, g, mean, invstd, relu=True, want_dresidual=True)
    assert np.array_equal(dres, np.where(out2 > 0.0, dout, 0.0))


def test_bn_backward_central_differences():
    x, r, g, b, dout = _bn_case(26, (2, 3, 4, 5))
    eps = 1e-5

    def loss(xv, gv, bv, rv):
        o, _, _ = oracle.bn_relu_add_fwd(xv, gv, bv, rv, eps, relu=True)
        return np.vdot(o, dout)

    out, mean, invstd = oracle.bn_relu_add_fwd(x, g, b, r, eps, relu=True)
    z_plain, _, _ = oracle.bn_relu_add_fwd(x, g, b, r, eps, relu=False)
    dx, dres, dg, db = oracle.bn_relu_add_bwd(x, out, dout, g, mean, invstd, relu=True, want_dresidual=True)
    h = 1e-5
    if np.abs(z_plain).min() < 100 * h:      # a pre-activation sits on the ReLU kink: FD is not valid
        pytest.skip("a pre-activation is too close to zero for this seed")
    rng = np.random.default_rng(0)
    for _ in range(10):
        j = tuple(rng.integers(0, s) for s in x.shape)
        e = np.zeros_like(x)
        e[j] = h
        fd = (loss(x + e, g, b, r) - loss(x - e, g, b, r)) / (2 * h)
        assert abs(fd - dx[j]) < 1e-6 * max(1.0, abs(fd))
        fd = (loss(x, g, b, r + e) - loss(x, g, b, r - e)) / (2 * h)
        assert abs(fd - dres[j]) < 1e-6 * max(1.0, abs(fd))
    for c in range(3):
        e = np.zeros(3)
        e[c] = h
        fd = (loss(x, g + e, b, r) - loss(x, g - e, b, r)) / (2 * h)
        assert abs(fd - dg[c]) < 1e-6 * max(1.0, abs(fd))
        fd = (loss(x, g, b + e, r) - loss(x, g, b - e, r)) / (2 * h)
        assert abs(fd - db[c]) < 1e-6 * max(1.0, abs(fd))


# ----------------------------------------------------------------------------- max pooling

def test_maxpool_golden_ties():
    x = np.array([[5, 5, 1, 0], [5, 2, 1, 7], [0, 0, 7, 7], [3, 0, 7, 1]], dtype=np.float64).reshape(1, 1, 4, 4)
    lines = [l for l in open(os.path.join(GOLD, "maxpool_ties_4x4.txt")) if not l.startswith("#")]
    want_y = np.array(lines[0].split()[1:], dtype=np.float64).reshape(2, 2)
    want_i = np.array(lines[1].split()[1:], dtype=np.int8).reshape(2, 2)
    y, idx = oracle.maxpool2d_fwd(x, 3, 2, 1)
    assert np.array_equal(y[0, 0], want_y)
    assert np.array_equal(idx[0, 0], want_i)
    const, ci = oracle.maxpool2d_fwd(np.full((1, 1, 5, 5), 2.0), 3, 2, 1)
    assert np.all(const == 2.0)
    # constant image: the first in-image tap of every window wins
    assert np.array_equal(ci[0, 0], np.array([[4, 3, 3], [1, 0, 0], [1, 0, 0]], dtype=np.int8))


@pytest.mark.parametrize("shape,win,st,pd", [((2, 3, 9, 8), 3, 2, 1), ((1, 2, 12, 12), 3, 2, 1), ((2, 2, 7, 7), 2, 2, 0)])
def test_maxpool_matches_torch(shape, win, st, pd):
    x = gen.normal(31, 0, shape).astype(np.float64)
    y, idx = oracle.maxpool2d_fwd(x, win, st, pd)
    tx = torch.from_numpy(x).requires_grad_(True)
    ty, ti = F.max_pool2d(tx, win, st, pd, return_indices=True)
    assert np.array_equal(y, ty.detach().numpy())
    # torch returns the flat h*W+w position; convert the oracle's window position to it
    P, Q = y.shape[2:]
    p = np.arange(P)[:, None]
    q = np.arange(Q)[None, :]
    flat = (p * st - pd + idx // win) * shape[3] + (q * st - pd + idx % win)
    assert np.array_equal(flat, ti.numpy())
    dy = gen.normal(31, 1, y.shape).astype(np.float64)
    ty.backward(torch.from_numpy(dy))
    dx = oracle.maxpool2d_bwd(dy, idx, shape, win, st, pd)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=0, atol=1e-14)
    np.testing.assert_allclose(dx.sum(), dy.sum(), rtol=1e-12)


# ----------------------------------------------------------------------------- bf16 grid

def test_bf16_rounding_golden_and_torch():
    for line in open(os.path.join(GOLD, "bf16_rounding.txt")):
        if line.startswith("#") or not line.strip():
            continue
        src, want = line.split()
        got = oracle.round_bf16(np.array([eval(src)]))[0]
        assert got == eval(want), (src, got)
    a = gen.normal(41, 0, (4096,)) * np.float32(37.0)
    ours = oracle.round_bf16(a.astype(np.float64))
    theirs = torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(ours, theirs)
    assert np.array_equal(gen.to_bf16_grid(a).astype(np.float64), theirs)


# ---------------------------------------------------------------------------------------------- grouped convolution
@pytest.mark.parametrize("case", [(2, 8, 7, 9, 12, 3, 2, 1, 1, 1), (1, 6, 8, 8, 6, 3, 6, 2, 1, 1), (2, 4, 9, 7, 8, 2, 4, (2, 1), (0, 1), (1, 2)),
                                  (1, 12, 6, 6, 4, 1, 4, 1, 0, 1)])
def test_grouped_convolution_matches_torch_float64_with_autograd(case):
    """Forward against torch's CPU float64 grouped convolution, both gradients against its autograd (depthwise included:
    groups == C)."""
    N, C, H, W, K, R, G, st, pd, dl = case
    rng = np.random.default_rng(77 + C + K)
    x = rng.standard_normal((N, C, H, W))
    w = rng.standard_normal((K, C // G, R, R))
    tx, tw = torch.from_numpy(x).requires_grad_(True), torch.from_numpy(w).requires_grad_(True)
    ty = F.conv2d(tx, tw, None, st, pd, dl, groups=G)
    y = oracle.conv2d_grouped_fwd(x, w, G, st, pd, dl)
    assert y.shape == tuple(ty.shape) and np.max(np.abs(y - ty.detach().numpy())) <= 1e-12 * max(1.0, np.abs(y).max())
    dy = rng.standard_normal(y.shape)
    ty.backward(torch.from_numpy(dy))
    dx = oracle.conv2d_grouped_dgrad(dy, w, x.shape, G, st, pd, dl)
    dw = oracle.conv2d_grouped_wgrad(x, dy, w.shape, G, st, pd, dl)
    assert np.max(np.abs(dx - tx.grad.numpy())) <= 1e-12 * max(1.0, np.abs(dx).max())
    assert np.max(np.abs(dw - tw.grad.numpy())) <= 1e-12 * max(1.0, np.abs(dw).max())
    base = rng.standard_normal(x.shape)
    assert np.allclose(oracle.conv2d_grouped_dgrad(dy, w, x.shape, G, st, pd, dl, into=base), base + dx, rtol=0, atol=1e-12)


def test_grouped_convolution_with_one_group_is_the_plain_one_and_groups_do_not_mix():
    rng = np.random.default_rng(5)
    x, w = rng.standard_normal((1, 4, 5, 5)), rng.standard_normal((6, 4, 3, 3))
    assert np.array_equal(oracle.conv2d_grouped_fwd(x, w, 1, 1, 1, 1), oracle.conv2d_fwd(x, w, 1, 1, 1))
    w2 = rng.standard_normal((6, 2, 3, 3))
    y = oracle.conv2d_grouped_fwd(x, w2, 2, 1, 1, 1)
    x_other = x.copy()
    x_other[:, 2:] += 10.0                      # changing the second group's input ...
    y_other = oracle.conv2d_grouped_fwd(x_other, w2, 2, 1, 1, 1)
    assert np.array_equal(y[:, :3], y_other[:, :3]) and not np.allclose(y[:, 3:], y_other[:, 3:])   # ... moves its outputs only
