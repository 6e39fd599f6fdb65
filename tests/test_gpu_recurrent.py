"""GPU parity of the recurrent workload against oracle/gru.py: embedding lookup and its gradient, the fused GRU gate
kernels, and the whole classifier (embedding -> GRU -> output layer -> cross entropy) forward, backward through time
and one clipped AdamW step."""
import numpy as np
import pytest
import torch

import nsk_inputs as gen
from oracle import gru as G
from oracle import train as T
from paper_2409_11600_amd import binding as B
from paper_2409_11600_amd.recurrent import GpuGruClassifier
from parity import TOL, guarded, max_rel_err, on_grid, torch_dtype

pytestmark = pytest.mark.gpu


def dev(a, dtype="f32"):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0", dtype=torch_dtype(dtype))


def host(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,E,V", [(40, 8, 9), (1000, 64, 50), (10000, 256, 32768), (7, 5, 3)])
def test_embedding_lookup_and_its_gradient(n, E, V, dtype):
    print(f"embedding case n={n} E={E} V={V} {dtype}", flush=True)
    tokens = (gen.uniform(8000 + n, 0, (n,)) * V).astype(np.int32) % V
    tokens[: min(n, 5)] = tokens[0]                      # duplicates for certain
    table = on_grid(gen.normal(8000 + n, 1, (V, E)), dtype)
    dout = on_grid(gen.normal(8000 + n, 2, (n, E)), dtype)
    gt = torch.from_numpy(tokens).cuda()
    out_view, out_check = guarded((n, E), torch_dtype(dtype))
    B.embedding_fwd(gt, dev(table, dtype), out=out_view)
    dt_view, dt_check = guarded((V, E), torch.float32)
    B.embedding_bwd(gt, dev(dout, dtype), V, dtable=dt_view)
    base = gen.normal(8000 + n, 3, (V, E)).astype(np.float32)
    gacc = dev(base)
    B.embedding_bwd(gt, dev(dout, dtype), V, dtable=gacc, accumulate=True)
    again = B.embedding_bwd(gt, dev(dout, dtype), V)
    torch.cuda.synchronize()
    out_check()
    dt_check()
    assert np.array_equal(host(out_view), G.embedding_fwd(tokens, table))             # a copy: exact
    want = G.embedding_bwd(tokens, dout, V)
    assert max_rel_err(host(dt_view), want) <= 1e-5
    assert np.all(host(dt_view)[want == 0.0] == 0.0)
    assert max_rel_err(host(gacc), G.embedding_bwd(tokens, dout, V, into=base.astype(np.float64))) <= 1e-5
    assert torch.equal(again, dt_view)                                                # position order, no atomics


def test_embedding_flags_a_token_out_of_range():
    table = dev(np.ones((4, 8)))
    tok = torch.tensor([0, 4, -1, 3], dtype=torch.int32).cuda()
    out = B.embedding_fwd(tok, table)
    d = B.embedding_bwd(tok, dev(np.ones((4, 8))), 4)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert np.all(o[0] == 1) and np.all(np.isnan(o[1])) and np.all(np.isnan(o[2])) and np.all(o[3] == 1)
    assert d.cpu().numpy().sum(axis=1).tolist() == [8.0, 0.0, 0.0, 8.0]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,H", [(50, 256), (4, 8), (3, 40), (1, 8)])
def test_gru_gate_kernels(N, H, dtype):
    print(f"gru gates case N={N} H={H} {dtype}", flush=True)
    s = 8100 + N
    gi, gh = on_grid(gen.normal(s, 0, (N, 3 * H)), dtype), on_grid(gen.normal(s, 1, (N, 3 * H)), dtype)
    b_ih, b_hh = (0.3 * gen.normal(s, 2, (3 * H,))).astype(np.float32), (0.3 * gen.normal(s, 3, (3 * H,))).astype(np.float32)
    h_prev, dh1, dh2 = (on_grid(gen.normal(s, 4 + k, (N, H)), dtype) for k in range(3))
    tol = TOL[dtype]
    h_view, h_check = guarded((N, H), torch_dtype(dtype))
    _, saved = B.gru_gates_fwd(dev(gi, dtype), dev(gh, dtype), dev(b_ih), dev(b_hh), dev(h_prev, dtype), h_new=h_view)
    torch.cuda.synchronize()
    h_check()
    wh, r, z, n, q = G.gru_gates_fwd(gi, gh, b_ih, b_hh, h_prev)
    assert max_rel_err(host(h_view), wh) <= tol
    sv = host(saved)
    for k, want in enumerate((r, z, n, q)):
        assert max_rel_err(sv[:, k * H:(k + 1) * H], want) <= tol
    # backward from the values the forward kernel stored (both sides differentiate the same stored gates)
    rs, zs, ns, qs = (sv[:, k * H:(k + 1) * H] for k in range(4))
    dgi, dgh, dhd = B.gru_gates_bwd(saved, dev(h_prev, dtype), dev(dh1, dtype), dev(dh2, dtype))
    dgi1, _, _ = B.gru_gates_bwd(saved, dev(h_prev, dtype), dev(dh1, dtype))
    torch.cuda.synchronize()
    wgi, wgh, wd = G.gru_gates_bwd(rs, zs, ns, qs, h_prev, dh1.astype(np.float64) + dh2)
    assert max_rel_err(host(dgi), wgi) <= tol and max_rel_err(host(dgh), wgh) <= tol and max_rel_err(host(dhd), wd) <= tol
    assert max_rel_err(host(dgi1), G.gru_gates_bwd(rs, zs, ns, qs, h_prev, dh1)[0]) <= tol


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,H", [(50, 256), (4, 8), (3, 40), (1, 4), (64, 128), (130, 20)])
def test_gru_fused_step_kernels(N, H, dtype):
    """nsk_gru_step_fwd / bwd: the recurrent product and the gate arithmetic of a step in one launch, against the
    oracle's product followed by its gate functions."""
    print(f"gru fused step case N={N} H={H} {dtype}", flush=True)
    assert B.gru_step_supported(N, H)
    s = 8400 + N
    gi = on_grid(gen.normal(s, 0, (N, 3 * H)), dtype)
    w_hh = on_grid(gen.normal(s, 1, (3 * H, H)) / np.sqrt(H), dtype)
    b_ih, b_hh = (0.3 * gen.normal(s, 2, (3 * H,))).astype(np.float32), (0.3 * gen.normal(s, 3, (3 * H,))).astype(np.float32)
    h_prev, dh_a, dhd_next = (on_grid(gen.normal(s, 4 + k, (N, H)), dtype) for k in range(3))
    dgh_next = on_grid(gen.normal(s, 7, (N, 3 * H)), dtype)
    tol = TOL[dtype]
    h_view, h_check = guarded((N, H), torch_dtype(dtype))
    s_view, s_check = guarded((N, 4 * H), torch_dtype(dtype))
    g_w, g_h = dev(w_hh, dtype), dev(h_prev, dtype)
    g_wt = dev(np.ascontiguousarray(w_hh.T), dtype)
    B.gru_step_fwd(dev(gi, dtype), g_w, dev(b_ih), dev(b_hh), g_h, h_new=h_view, saved=s_view)
    torch.cuda.synchronize()
    h_check()
    s_check()
    wh, r, z, n, q = G.gru_gates_fwd(gi, h_prev.astype(np.float64) @ w_hh.astype(np.float64).T, b_ih, b_hh, h_prev)
    assert max_rel_err(host(h_view), wh) <= tol
    sv = host(s_view)
    for k, want in enumerate((r, z, n, q)):
        assert max_rel_err(sv[:, k * H:(k + 1) * H], want) <= tol
    # backward from the stored gates, with all three gradient sources, then with each of them alone
    rs, zs, ns, qs = (sv[:, k * H:(k + 1) * H] for k in range(4))
    rec = dgh_next.astype(np.float64) @ w_hh.astype(np.float64)
    cases = [(dh_a, dhd_next, dgh_next), (dh_a, None, None), (None, dhd_next, None), (None, None, dgh_next)]
    for a, d, g in cases:
        outs = [guarded(sh, torch_dtype(dtype)) for sh in ((N, 3 * H), (N, 3 * H), (N, H))]
        B.gru_step_bwd(s_view, g_h, g_wt, dh_a=None if a is None else dev(a, dtype), dh_direct_next=None if d is None else dev(d, dtype),
                       dgh_next=None if g is None else dev(g, dtype), dgi=outs[0][0], dgh=outs[1][0], dh_direct=outs[2][0])
        torch.cuda.synchronize()
        for _, check in outs:
            check()
        dh = np.zeros((N, H)) + (0 if a is None else a) + (0 if d is None else d) + (0 if g is None else rec)
        for (view, _), want in zip(outs, G.gru_gates_bwd(rs, zs, ns, qs, h_prev, dh)):
            assert max_rel_err(host(view), want) <= tol
    assert not B.gru_step_supported(300, 256) and not B.gru_step_supported(8, 6)


def _model(seed, T_, N, E, H, V, K):
    tokens = ((gen.uniform(seed, 0, (T_, N)) * V).astype(np.int32)) % V
    labels = ((gen.uniform(seed, 1, (N,)) * K).astype(np.int32)) % K
    p = dict(table=gen.normal(seed, 2, (V, E)), w_ih=gen.normal(seed, 3, (3 * H, E)) / np.sqrt(E),
             w_hh=gen.normal(seed, 4, (3 * H, H)) / np.sqrt(H), b_ih=0.1 * gen.normal(seed, 5, (3 * H,)),
             b_hh=0.1 * gen.normal(seed, 6, (3 * H,)), w_out=gen.normal(seed, 7, (K, H)) / np.sqrt(H),
             b_out=0.1 * gen.normal(seed, 8, (K,)))
    return tokens, labels, {k: v.astype(np.float32) for k, v in p.items()}


def _oracle_step(tokens, labels, p):
    """Forward to the loss and backward through time with the oracle's primitives, in float64."""
    T_, N = tokens.shape
    V, E = p["table"].shape
    x = G.embedding_fwd(tokens.reshape(-1), p["table"]).reshape(T_, N, E)
    fwd = G.gru_forward(x, np.zeros((N, p["w_hh"].shape[1])), p["w_ih"], p["w_hh"], p["b_ih"], p["b_hh"])
    hT = fwd["h"][-1]
    logits = T.linear_fwd(hT, p["w_out"], p["b_out"])
    loss, _ = T.softmax_xent_fwd(logits, labels)
    dlogits = T.softmax_xent_bwd(logits, labels)
    dw_out, db_out = T.linear_wgrad(hT, dlogits)
    dh_all = np.zeros_like(fwd["h"][1:])
    dh_all[-1] = T.linear_dgrad(dlogits, p["w_out"])
    bwd = G.gru_backward(x, fwd, p["w_ih"], p["w_hh"], dh_all)
    grads = dict(table=G.embedding_bwd(tokens.reshape(-1), bwd["dx"].reshape(T_ * N, E), V), w_ih=bwd["dw_ih"],
                 w_hh=bwd["dw_hh"], b_ih=bwd["db_ih"], b_hh=bwd["db_hh"], w_out=dw_out, b_out=db_out)
    return loss, fwd, grads


@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("shape", [(6, 4, 16, 16, 50, 2), (12, 8, 32, 24, 100, 3)])
def test_gru_classifier_forward_backward_and_adamw_step_match_the_oracle(shape, fused):
    T_, N, E, H, V, K = shape
    print(f"gru classifier T={T_} N={N} E={E} H={H} V={V} K={K} (f32) fused steps={fused}", flush=True)
    tokens, labels, p = _model(8200 + T_, T_, N, E, H, V, K)
    m = GpuGruClassifier(tokens, labels, **p, dtype="f32", lr=1e-3, weight_decay=1e-4, clip=0.05)
    assert m.fused_steps
    m.fused_steps = fused       # False: one product and one gate kernel per step and direction
    m.forward()
    m.backward()
    torch.cuda.synchronize()
    loss, fwd, grads = _oracle_step(tokens, labels, p)
    assert abs(float(m.loss.item()) - loss) <= 1e-5 * abs(loss)
    assert max_rel_err(host(m.h), fwd["h"]) <= TOL["f32"]
    for k in m.order:
        assert max_rel_err(host(m.grad[k]), grads[k]) <= 2 * TOL["f32"], k
    gh = {k: host(m.grad[k]) for k in m.order}
    m.update()
    torch.cuda.synchronize()
    s = T.clip_scale([gh[k] for k in m.order], 0.05)
    assert s < 1.0 and abs(float(m.scale.item()) - s) <= 1e-5 * s
    b1, b2 = float(np.float32(0.9)), float(np.float32(0.999))
    for k in m.order:
        wd = 1e-4 if k in ("table", "w_ih", "w_hh", "w_out") else 0.0
        want, _, _, _ = T.adamw_step(p[k], gh[k], np.zeros_like(gh[k]), np.zeros_like(gh[k]), 1, 1e-3, b1, b2, 1e-8, wd, grad_scale=s)
        assert max_rel_err(host(m.master[k]) - p[k], want - p[k]) <= 1e-3, k
        assert not m.grad[k].any()


def test_bf16_gru_classifier_tracks_the_oracle_and_learns():
    T_, N, E, H, V, K = 10, 16, 32, 32, 64, 2
    tokens, labels, p = _model(8300, T_, N, E, H, V, K)
    m = GpuGruClassifier(tokens, labels, **p, dtype="bf16", lr=1e-2, weight_decay=0.0, clip=5.0)
    q = {k: (gen.to_bf16_grid(v) if k in ("table", "w_ih", "w_hh", "w_out") else v) for k, v in p.items()}
    loss, _, _ = _oracle_step(tokens, labels, q)
    losses = []
    for _ in range(30):
        m.step()
        torch.cuda.synchronize()
        losses.append(float(m.loss.item()))
    assert abs(losses[0] - loss) <= 2e-2 * abs(loss)
    assert np.all(np.isfinite(losses)) and losses[-1] < 0.7 * losses[0]
    for k in ("table", "w_ih", "w_hh", "w_out"):
        assert torch.equal(m.w[k], m.master[k].to(torch.bfloat16))
