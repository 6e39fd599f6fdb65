"""Pins for the oracle of the recurrent workload (embedding, GRU layer, gradients through time): torch's CPU float64
`nn.GRU` / `F.embedding` with autograd (an independent implementation of the same gate convention), closed forms,
and central finite differences.  A wrong gate order, a reset gate applied on the wrong side, a dropped bias or a
transposed weight fails at least one of them."""
import numpy as np
import torch
import torch.nn.functional as F

import nsk_inputs as gen
from oracle import gru as G


def _r(seed, k, shape, scale=1.0):
    return scale * gen.normal(seed, k, shape).astype(np.float64)


def _params(seed, E, H):
    return (_r(seed, 0, (3 * H, E), 0.4), _r(seed, 1, (3 * H, H), 0.4), _r(seed, 2, (3 * H,), 0.3), _r(seed, 3, (3 * H,), 0.3))


def test_embedding_hand_example_and_torch():
    table = np.arange(12.0).reshape(4, 3)
    out = G.embedding_fwd([2, 0, 2], table)
    assert out.tolist() == [[6.0, 7.0, 8.0], [0.0, 1.0, 2.0], [6.0, 7.0, 8.0]]
    dt = G.embedding_bwd([2, 0, 2], np.array([[1.0, 1, 1], [10, 10, 10], [100, 100, 100]]), 4)
    assert dt.tolist() == [[10.0] * 3, [0.0] * 3, [101.0] * 3, [0.0] * 3]      # duplicates add up, untouched rows stay 0
    tok = (gen.uniform(11, 0, (40,)) * 9).astype(np.int64) % 9
    tab, dout = _r(11, 1, (9, 5)), _r(11, 2, (40, 5))
    tt = torch.tensor(tab, requires_grad=True)
    F.embedding(torch.tensor(tok), tt).backward(torch.tensor(dout))
    np.testing.assert_allclose(G.embedding_bwd(tok, dout, 9), tt.grad.numpy(), rtol=1e-14, atol=1e-14)
    base = _r(11, 3, (9, 5))
    np.testing.assert_allclose(G.embedding_bwd(tok, dout, 9, into=base), base + tt.grad.numpy(), rtol=1e-14, atol=1e-14)


def test_gates_closed_forms():
    H = 3
    zeros = np.zeros((2, 3 * H))
    h_prev = np.array([[1.0, -2.0, 0.5], [0.0, 3.0, -1.0]])
    # all pre-activations zero: r = z = 1/2, n = tanh(0) = 0, h' = h/2
    h, r, z, n, q = G.gru_gates_fwd(zeros, zeros, np.zeros(3 * H), np.zeros(3 * H), h_prev)
    assert np.all(r == 0.5) and np.all(z == 0.5) and np.all(n == 0.0) and np.array_equal(h, 0.5 * h_prev)
    # update gate saturated to 1: the state is carried over unchanged; to 0: the state becomes the candidate
    big = np.zeros(3 * H)
    big[H:2 * H] = 50.0
    h, *_ = G.gru_gates_fwd(zeros, zeros, big, np.zeros(3 * H), h_prev)
    np.testing.assert_allclose(h, h_prev, atol=1e-15)
    gi = zeros.copy()
    gi[:, 2 * H:] = 0.7
    h, *_ = G.gru_gates_fwd(gi, zeros, -big, np.zeros(3 * H), h_prev)
    np.testing.assert_allclose(h, np.tanh(0.7), atol=1e-15)
    # the reset gate multiplies the RECURRENT candidate term (including its bias), not the input term
    b_hh = np.zeros(3 * H)
    b_hh[2 * H:] = 2.0
    b_ih = np.zeros(3 * H)
    b_ih[:H] = -50.0                        # r -> 0
    h, r, z, n, q = G.gru_gates_fwd(gi, zeros, b_ih, b_hh, h_prev)
    np.testing.assert_allclose(n, np.tanh(0.7), atol=1e-12)      # the 2.0 is gated away, the 0.7 is not
    assert np.all(q == 2.0)


def test_layer_matches_torch_gru_forward_and_backward():
    T, N, E, H = 7, 4, 5, 6
    w_ih, w_hh, b_ih, b_hh = _params(21, E, H)
    x, h0, dh_all = _r(21, 4, (T, N, E)), _r(21, 5, (N, H)), _r(21, 6, (T, N, H))
    gru = torch.nn.GRU(E, H).double()
    with torch.no_grad():
        gru.weight_ih_l0.copy_(torch.tensor(w_ih)); gru.weight_hh_l0.copy_(torch.tensor(w_hh))
        gru.bias_ih_l0.copy_(torch.tensor(b_ih)); gru.bias_hh_l0.copy_(torch.tensor(b_hh))
    tx, th0 = torch.tensor(x, requires_grad=True), torch.tensor(h0, requires_grad=True)
    out, _ = gru(tx, th0[None])
    out.backward(torch.tensor(dh_all))
    fwd = G.gru_forward(x, h0, w_ih, w_hh, b_ih, b_hh)
    np.testing.assert_allclose(fwd["h"][1:], out.detach().numpy(), rtol=1e-12, atol=1e-13)
    bwd = G.gru_backward(x, fwd, w_ih, w_hh, dh_all)
    np.testing.assert_allclose(bwd["dx"], tx.grad.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(bwd["dh0"], th0.grad.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(bwd["dw_ih"], gru.weight_ih_l0.grad.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(bwd["dw_hh"], gru.weight_hh_l0.grad.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(bwd["db_ih"], gru.bias_ih_l0.grad.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(bwd["db_hh"], gru.bias_hh_l0.grad.numpy(), rtol=1e-11, atol=1e-13)


def test_backward_matches_finite_differences():
    T, N, E, H = 4, 2, 3, 3
    w_ih, w_hh, b_ih, b_hh = _params(31, E, H)
    x, h0, dh_all = _r(31, 4, (T, N, E)), _r(31, 5, (N, H)), _r(31, 6, (T, N, H))

    def loss(x_, h0_, w_ih_, w_hh_, b_ih_, b_hh_):
        return float((G.gru_forward(x_, h0_, w_ih_, w_hh_, b_ih_, b_hh_)["h"][1:] * dh_all).sum())

    bwd = G.gru_backward(x, G.gru_forward(x, h0, w_ih, w_hh, b_ih, b_hh), w_ih, w_hh, dh_all)
    args = [x, h0, w_ih, w_hh, b_ih, b_hh]
    grads = [bwd["dx"], bwd["dh0"], bwd["dw_ih"], bwd["dw_hh"], bwd["db_ih"], bwd["db_hh"]]
    eps = 1e-6
    for k, (a, g) in enumerate(zip(args, grads)):
        for idx in [tuple(0 for _ in a.shape), tuple(s - 1 for s in a.shape), tuple(s // 2 for s in a.shape)]:
            ap, am = [v.copy() for v in args], [v.copy() for v in args]
            ap[k][idx] += eps
            am[k][idx] -= eps
            fd = (loss(*ap) - loss(*am)) / (2 * eps)
            assert abs(fd - g[idx]) <= 1e-7 * max(1.0, abs(fd)), (k, idx)
