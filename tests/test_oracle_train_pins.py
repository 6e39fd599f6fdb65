"""Pins for the oracle of the training-step tail (global average pool, fully connected layer, softmax cross-entropy,
SGD with momentum, AdamW, gradient clip): closed forms, invariants, finite differences, the convolution oracle (a
different implementation: C loops) on the 1x1 case, and torch's CPU float64 operators and optimizers.  None of these
re-types the oracle's formulas; each is chosen so that a dropped term, a wrong sign or a transposed operand fails.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import nsk_inputs as gen
import oracle
from oracle import train as T


def _r(seed, k, shape):
    return gen.normal(seed, k, shape).astype(np.float64)


# ----------------------------------------------------------------------------- global average pool

def test_avgpool_closed_forms():
    x = np.zeros((2, 3, 4, 5))
    x[0, 1] = 7.0                                   # constant plane -> its value
    x[1, 2] = np.arange(20.0).reshape(4, 5)         # ramp 0..19 -> 9.5
    y = T.global_avgpool_fwd(x)
    assert y.shape == (2, 3)
    assert y[0, 1] == 7.0 and y[1, 2] == 9.5 and y[0, 0] == 0.0


def test_avgpool_matches_torch_and_adjoint():
    x, dy = _r(1, 0, (3, 5, 6, 7)), _r(1, 1, (3, 5))
    tx = torch.tensor(x, requires_grad=True)
    ty = F.adaptive_avg_pool2d(tx, 1)[:, :, 0, 0]
    ty.backward(torch.tensor(dy))
    np.testing.assert_allclose(T.global_avgpool_fwd(x), ty.detach().numpy(), rtol=1e-14, atol=1e-15)
    dx = T.global_avgpool_bwd(dy, x.shape)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-14, atol=1e-16)
    # <A x, dy> == <x, A^T dy>
    assert abs((T.global_avgpool_fwd(x) * dy).sum() - (x * dx).sum()) <= 1e-12
    base = _r(1, 2, x.shape)
    np.testing.assert_allclose(T.global_avgpool_bwd(dy, x.shape, into=base), base + dx, rtol=0, atol=1e-15)


# ----------------------------------------------------------------------------- fully connected layer

def test_linear_is_the_1x1_convolution_on_a_1x1_image():
    """x @ w with w transposed (section "Automatic Differentiation") == the convolution oracle (C loops) with R=S=H=W=1."""
    x, w, dy = _r(2, 0, (5, 7)), _r(2, 1, (4, 7)), _r(2, 2, (5, 4))
    y = T.linear_fwd(x, w)
    np.testing.assert_allclose(y, oracle.conv2d_fwd(x[:, :, None, None], w[:, :, None, None])[:, :, 0, 0], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(T.linear_dgrad(dy, w),
                               oracle.conv2d_dgrad(dy[:, :, None, None], w[:, :, None, None], (5, 7, 1, 1))[:, :, 0, 0],
                               rtol=1e-13, atol=1e-13)
    dw, db = T.linear_wgrad(x, dy)
    np.testing.assert_allclose(dw, oracle.conv2d_wgrad(x[:, :, None, None], dy[:, :, None, None], (4, 7, 1, 1))[:, :, 0, 0],
                               rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(db, dy.sum(0), rtol=1e-14)


def test_linear_hand_example_and_transposition():
    # w is [outputs][inputs]: y[0] = 1*1 + 2*2 + 3*3 = 14, y[1] = 1*0 + 2*1 + 3*0 = 2 (+ bias)
    x = np.array([[1.0, 2.0, 3.0]])
    w = np.array([[1.0, 2.0, 3.0], [0.0, 1.0, 0.0]])
    assert T.linear_fwd(x, w).tolist() == [[14.0, 2.0]]
    assert T.linear_fwd(x, w, np.array([0.5, -2.0])).tolist() == [[14.5, 0.0]]
    assert T.linear_dgrad(np.array([[1.0, 10.0]]), w).tolist() == [[1.0, 12.0, 3.0]]
    dw, db = T.linear_wgrad(x, np.array([[1.0, 10.0]]))
    assert dw.tolist() == [[1.0, 2.0, 3.0], [10.0, 20.0, 30.0]] and db.tolist() == [1.0, 10.0]


def test_linear_matches_torch_autograd_and_accumulates():
    x, w, b, dy = _r(3, 0, (6, 9)), _r(3, 1, (5, 9)), _r(3, 2, (5,)), _r(3, 3, (6, 5))
    tx, tw, tb = (torch.tensor(a, requires_grad=True) for a in (x, w, b))
    F.linear(tx, tw, tb).backward(torch.tensor(dy))
    np.testing.assert_allclose(T.linear_fwd(x, w, b), F.linear(tx, tw, tb).detach().numpy(), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(T.linear_dgrad(dy, w), tx.grad.numpy(), rtol=1e-13, atol=1e-13)
    dw, db = T.linear_wgrad(x, dy)
    np.testing.assert_allclose(dw, tw.grad.numpy(), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-13, atol=1e-13)
    bx, bw, bb = _r(3, 4, x.shape), _r(3, 5, w.shape), _r(3, 6, b.shape)
    np.testing.assert_allclose(T.linear_dgrad(dy, w, into=bx), bx + tx.grad.numpy(), rtol=1e-13, atol=1e-13)
    dw2, db2 = T.linear_wgrad(x, dy, into_dw=bw, into_db=bb)
    np.testing.assert_allclose(dw2, bw + dw, rtol=0, atol=1e-14)
    np.testing.assert_allclose(db2, bb + db, rtol=0, atol=1e-14)


# ----------------------------------------------------------------------------- softmax cross-entropy

def test_xent_closed_forms():
    K = 10
    loss, per = T.softmax_xent_fwd(np.zeros((4, K)), [0, 3, 9, 5])
    assert abs(loss - np.log(K)) <= 1e-15 and np.allclose(per, np.log(K))
    # two classes, logits (a, 0), label 0: loss = log(1 + exp(-a))
    a = 1.7
    loss, _ = T.softmax_xent_fwd(np.array([[a, 0.0]]), [0])
    assert abs(loss - np.log1p(np.exp(-a))) <= 1e-15
    # a confident right answer costs ~0, a confident wrong one ~ the margin
    assert T.softmax_xent_fwd(np.array([[50.0, 0.0]]), [0])[0] < 1e-20
    assert abs(T.softmax_xent_fwd(np.array([[50.0, 0.0]]), [1])[0] - 50.0) < 1e-12


def test_xent_shift_invariance_and_large_logits():
    z = _r(4, 0, (5, 7)) * 3.0
    lab = [1, 0, 6, 3, 3]
    l0, _ = T.softmax_xent_fwd(z, lab)
    l1, _ = T.softmax_xent_fwd(z + 1e4, lab)          # naive exp would overflow
    assert np.isfinite(l1) and abs(l0 - l1) <= 1e-9
    np.testing.assert_allclose(T.softmax_xent_bwd(z, lab), T.softmax_xent_bwd(z + 1e4, lab), atol=1e-12)


def test_xent_gradient_rows_sum_to_zero_and_match_finite_differences():
    z = _r(5, 0, (4, 6))
    lab = np.array([2, 5, 0, 2])
    dz = T.softmax_xent_bwd(z, lab, dloss=1.5)
    np.testing.assert_allclose(dz.sum(axis=1), 0.0, atol=1e-16)
    assert np.all(dz[np.arange(4), lab] < 0) and np.all(np.delete(dz[0], 2) > 0)
    h = 1e-6
    for (n, k) in [(0, 2), (1, 0), (3, 5), (2, 3)]:
        zp, zm = z.copy(), z.copy()
        zp[n, k] += h
        zm[n, k] -= h
        fd = 1.5 * (T.softmax_xent_fwd(zp, lab)[0] - T.softmax_xent_fwd(zm, lab)[0]) / (2 * h)
        assert abs(fd - dz[n, k]) <= 1e-9


def test_xent_matches_torch():
    z = _r(6, 0, (8, 10)) * 2.0
    lab = np.array([3, 1, 4, 1, 5, 9, 2, 6])
    tz = torch.tensor(z, requires_grad=True)
    tl = F.cross_entropy(tz, torch.tensor(lab))
    tl.backward()
    assert abs(T.softmax_xent_fwd(z, lab)[0] - tl.item()) <= 1e-14
    np.testing.assert_allclose(T.softmax_xent_bwd(z, lab), tz.grad.numpy(), rtol=1e-12, atol=1e-16)


# ----------------------------------------------------------------------------- optimizers

def test_sgd_closed_form_constant_gradient():
    """With a constant gradient and no decay: v_t = g (1 - mu^t) / (1 - mu), w_t = w_0 - lr * sum_s v_s."""
    g, mu, lr = 0.25, 0.9, 0.1
    w, v = np.array([1.0]), np.array([0.0])
    vs = []
    for t in range(1, 6):
        w, v, gz = T.sgd_momentum_step(w, np.array([g]), v, lr, mu, 0.0)
        vs.append(g * (1 - mu ** t) / (1 - mu))
        assert abs(v[0] - vs[-1]) <= 1e-15
        assert abs(w[0] - (1.0 - lr * sum(vs))) <= 1e-15
        assert gz.tolist() == [0.0]                 # the gradient buffer is cleared (section "Caching and Pooling")


def test_sgd_weight_decay_and_scale_terms():
    # one step from v = 0: w' = w - lr * (s*g + wd*w)
    w, v, _ = T.sgd_momentum_step(np.array([2.0]), np.array([3.0]), np.array([0.0]), 0.5, 0.9, 0.1, grad_scale=0.5)
    assert abs(v[0] - (1.5 + 0.2)) <= 1e-15 and abs(w[0] - (2.0 - 0.5 * 1.7)) <= 1e-15


@pytest.mark.parametrize("wd", [0.0, 1e-2])
def test_sgd_matches_torch(wd):
    w0 = _r(7, 0, (37,))
    gs = [_r(7, 1 + t, (37,)) for t in range(4)]
    tw = torch.tensor(w0.copy(), requires_grad=True)
    opt = torch.optim.SGD([tw], lr=0.05, momentum=0.9, weight_decay=wd)
    w, v = w0.copy(), np.zeros_like(w0)
    for g in gs:
        tw.grad = torch.tensor(g.copy())
        opt.step()
        w, v, _ = T.sgd_momentum_step(w, g, v, 0.05, 0.9, wd)
        np.testing.assert_allclose(w, tw.detach().numpy(), rtol=1e-13, atol=1e-15)


def test_adamw_first_step_is_a_signed_step():
    """From m = v = 0 the bias-corrected ratio is g / (|g| + eps): every weight moves by ~lr against its gradient's sign."""
    g = np.array([3.0, -0.02, 1e-3])
    w, m, v, gz = T.adamw_step(np.zeros(3), g, np.zeros(3), np.zeros(3), 1, lr=0.01, eps=1e-12)
    np.testing.assert_allclose(w, -0.01 * np.sign(g), rtol=1e-8)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-15)
    np.testing.assert_allclose(v, 0.001 * g * g, rtol=1e-12)
    assert not gz.any()
    # zero gradient: only the decoupled decay acts, multiplicatively
    w, _, _, _ = T.adamw_step(np.array([2.0]), np.array([0.0]), np.zeros(1), np.zeros(1), 1, lr=0.1, weight_decay=0.5)
    assert abs(w[0] - 2.0 * (1 - 0.05)) <= 1e-15


@pytest.mark.parametrize("wd", [0.0, 1e-4, 0.1])
def test_adamw_matches_torch(wd):
    w0 = _r(8, 0, (29,))
    gs = [_r(8, 1 + t, (29,)) for t in range(5)]
    tw = torch.tensor(w0.copy(), requires_grad=True)
    opt = torch.optim.AdamW([tw], lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=wd)
    w, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    for t, g in enumerate(gs, start=1):
        tw.grad = torch.tensor(g.copy())
        opt.step()
        w, m, v, _ = T.adamw_step(w, g, m, v, t, 1e-3, 0.9, 0.999, 1e-8, wd)
        np.testing.assert_allclose(w, tw.detach().numpy(), rtol=1e-12, atol=1e-15)


def test_clip_scale_closed_form_and_torch():
    g1, g2 = np.array([3.0, 0.0]), np.array([[0.0, 4.0]])      # global norm 5
    assert T.clip_scale([g1, g2], 10.0) == 1.0
    assert abs(T.clip_scale([g1, g2], 2.5) - 2.5 / (5.0 + 1e-6)) <= 1e-15
    a, b = _r(9, 0, (11,)) * 4, _r(9, 1, (3, 5)) * 4
    ta, tb = torch.tensor(a.copy(), requires_grad=True), torch.tensor(b.copy(), requires_grad=True)
    ta.grad, tb.grad = torch.tensor(a.copy()), torch.tensor(b.copy())
    torch.nn.utils.clip_grad_norm_([ta, tb], 5.0)
    s = T.clip_scale([a, b], 5.0)
    np.testing.assert_allclose(a * s, ta.grad.numpy(), rtol=1e-12)
    np.testing.assert_allclose(b * s, tb.grad.numpy(), rtol=1e-12)
