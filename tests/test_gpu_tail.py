"""GPU parity of the training-step tail (global average pool, fully connected layer, softmax cross-entropy, SGD with
momentum, AdamW, gradient clip) against the oracle in oracle/train.py, element by element on the same seeded inputs.
Tolerances: the path's stated bars (1e-4 fp32, 2e-2 bf16 on values stored in bf16); optimizer state is float on
both sides of the ABI and is held to 1e-5 (a handful of float operations per element against float64)."""
import numpy as np
import pytest
import torch

import nsk_inputs as gen
from oracle import train as T
from paper_2409_11600_amd import binding as B
from parity import TOL, guarded, max_rel_err, on_grid, to_gpu, to_host, torch_dtype

pytestmark = pytest.mark.gpu

LAYOUTS = [B.NSK_NHWC, B.NSK_NCHW]


def dev(a, dtype="f32"):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0", dtype=torch_dtype(dtype))


def host(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


POOL_SHAPES = [(3, 64, 7, 7), (2, 10, 8, 8), (2, 2048, 7, 7), (1, 5, 3, 9), (130, 512, 4, 4), (2, 3, 33, 31), (4, 64, 56, 56),
               (2, 256, 13, 9)]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("i", range(len(POOL_SHAPES)))
def test_global_avgpool(i, dtype, layout):
    shape = POOL_SHAPES[i]
    print(f"avgpool case {shape} {dtype} layout={layout}", flush=True)
    x = on_grid(gen.normal(1300 + i, 0, shape) + 0.3, dtype)
    dy = on_grid(gen.normal(1300 + i, 1, shape[:2]), dtype)
    base = on_grid(gen.normal(1300 + i, 2, shape), dtype)
    tol = TOL[dtype]
    gx = to_gpu(x, dtype, layout)
    y_view, y_check = guarded(shape[:2], torch_dtype(dtype))
    B.global_avgpool_fwd(gx, layout, out=y_view)
    dx_view, dx_check = guarded(gx.shape, torch_dtype(dtype))
    B.global_avgpool_bwd(dev(dy, dtype), shape, layout, out=dx_view)
    gacc = to_gpu(base, dtype, layout)
    B.global_avgpool_bwd(dev(dy, dtype), shape, layout, out=gacc, accumulate=True)
    torch.cuda.synchronize()
    y_check()
    dx_check()
    assert max_rel_err(host(y_view), T.global_avgpool_fwd(x)) <= tol
    assert max_rel_err(to_host(dx_view, layout), T.global_avgpool_bwd(dy, shape)) <= tol
    assert max_rel_err(to_host(gacc, layout), T.global_avgpool_bwd(dy, shape, into=base.astype(np.float64))) <= tol


LINEAR_SHAPES = [(128, 512, 10), (32, 64, 10), (5, 2048, 1000), (256, 64, 100), (1, 7, 3), (50, 256, 2)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("i", range(len(LINEAR_SHAPES)))
def test_linear_is_the_matmul_with_the_transposed_weight(i, dtype):
    N, C, K = LINEAR_SHAPES[i]
    print(f"linear case {LINEAR_SHAPES[i]} {dtype}", flush=True)
    x = on_grid(gen.normal(1400 + i, 0, (N, C)), dtype)
    w = on_grid(gen.normal(1400 + i, 1, (K, C)) / np.sqrt(C), dtype)
    b = gen.normal(1400 + i, 2, (K,)).astype(np.float32)
    dy = on_grid(gen.normal(1400 + i, 3, (N, K)), dtype)
    tol = TOL[dtype]
    ws = B.Workspace()
    gx, gw, gb, gdy = dev(x, dtype), dev(w, dtype), dev(b), dev(dy, dtype)
    y_view, y_check = guarded((N, K), torch_dtype(dtype))
    B.linear_fwd(gx, gw, gb, out=y_view, ws=ws)
    y_nb = B.linear_fwd(gx, gw, None, ws=ws)
    dx_view, dx_check = guarded((N, C), torch_dtype(dtype))
    B.linear_dgrad(gdy, gw, out=dx_view, ws=ws)
    dw_view, dw_check = guarded((K, C), torch.float32)
    db_view, db_check = guarded((K,), torch.float32)
    B.linear_wgrad(gx, gdy, dw=dw_view, db=db_view, ws=ws)
    torch.cuda.synchronize()
    for c in (y_check, dx_check, dw_check, db_check):
        c()
    assert max_rel_err(host(y_view), T.linear_fwd(x, w, b)) <= tol
    assert max_rel_err(host(y_nb), T.linear_fwd(x, w)) <= tol
    assert max_rel_err(host(dx_view), T.linear_dgrad(dy, w)) <= tol
    want_dw, want_db = T.linear_wgrad(x, dy)
    assert max_rel_err(host(dw_view), want_dw) <= TOL["f32"] * 10      # fp32 sums of exact products
    assert max_rel_err(host(db_view), want_db) <= TOL["f32"]
    # accumulating forms
    bx = on_grid(gen.normal(1400 + i, 4, (N, C)), dtype)
    bw = gen.normal(1400 + i, 5, (K, C)).astype(np.float32)
    bb = gen.normal(1400 + i, 6, (K,)).astype(np.float32)
    gbx, gbw, gbb = dev(bx, dtype), dev(bw), dev(bb)
    B.linear_dgrad(gdy, gw, out=gbx, accumulate=True, ws=ws)
    B.linear_wgrad(gx, gdy, dw=gbw, db=gbb, accumulate=True, ws=ws)
    torch.cuda.synchronize()
    assert max_rel_err(host(gbx), T.linear_dgrad(dy, w, into=bx.astype(np.float64))) <= tol
    want_dw2, want_db2 = T.linear_wgrad(x, dy, into_dw=bw.astype(np.float64), into_db=bb.astype(np.float64))
    assert max_rel_err(host(gbw), want_dw2) <= TOL["f32"] * 10
    assert max_rel_err(host(gbb), want_db2) <= TOL["f32"]


XENT_SHAPES = [(128, 10), (7, 1000), (50, 2), (256, 100), (1, 1), (3, 65)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("i", range(len(XENT_SHAPES)))
def test_softmax_cross_entropy(i, dtype):
    N, K = XENT_SHAPES[i]
    print(f"xent case {XENT_SHAPES[i]} {dtype}", flush=True)
    z = 3.0 * gen.normal(1500 + i, 0, (N, K))
    if i == 0:
        z[0] += 3000.0                                     # a naive exp would overflow
        z[1, 3] = -1e4                                     # and one probability underflows to zero
    z = on_grid(z, dtype)
    labels = (gen.uniform(1500 + i, 1, (N,)) * K).astype(np.int32) % K
    gz, gl = dev(z, dtype), torch.from_numpy(labels).cuda()
    loss, per = B.softmax_xent_fwd(gz, gl)
    dz_view, dz_check = guarded((N, K), torch_dtype(dtype))
    B.softmax_xent_bwd(gz, gl, dloss=1.5, out=dz_view)
    torch.cuda.synchronize()
    dz_check()
    want_loss, want_per = T.softmax_xent_fwd(z, labels)
    assert max_rel_err(host(per), want_per) <= 1e-5
    assert abs(float(loss.item()) - want_loss) <= 1e-5 * max(1.0, abs(want_loss))
    assert max_rel_err(host(dz_view), T.softmax_xent_bwd(z, labels, 1.5)) <= TOL[dtype]


def test_softmax_cross_entropy_flags_a_label_out_of_range():
    z = dev(np.zeros((4, 5)))
    loss, per = B.softmax_xent_fwd(z, torch.tensor([0, 5, -1, 2], dtype=torch.int32).cuda())
    torch.cuda.synchronize()
    p = per.cpu().numpy()
    assert np.isnan(p[1]) and np.isnan(p[2]) and abs(p[0] - np.log(5)) < 1e-6 and np.isnan(loss.item())


OPT_SIZES = [1000003, 64 * 3 * 7 * 7, 10, 1]


@pytest.mark.parametrize("with_lp,with_scale", [(False, False), (True, True)])
@pytest.mark.parametrize("n", OPT_SIZES)
def test_sgd_momentum_steps(n, with_lp, with_scale):
    print(f"sgd case n={n} lp={with_lp} scale={with_scale}", flush=True)
    w0 = gen.normal(1600, 0, (n,)).astype(np.float32)
    gs = [gen.normal(1600, 1 + t, (n,)).astype(np.float32) for t in range(3)]
    lr, mu, wd, s = 0.05, 0.9, 1e-2, 0.37
    gw, gv = dev(w0), torch.zeros(n, device="cuda:0")
    lp_view, lp_check = guarded((n,), torch.bfloat16)
    scale = dev(np.array([s])) if with_scale else None
    w, v = w0.astype(np.float64), np.zeros(n)
    for g in gs:
        gg = dev(g)
        B.sgd_momentum_step(gw, gg, gv, lr, mu, wd, w_lp=lp_view if with_lp else None, grad_scale=scale)
        w, v, _ = T.sgd_momentum_step(w, g, v, lr, mu, wd, grad_scale=s if with_scale else 1.0)
        torch.cuda.synchronize()
        assert not gg.any()                                   # gradient buffer cleared
        assert max_rel_err(host(gw), w) <= 1e-5
        assert max_rel_err(host(gv), v) <= 1e-5
    lp_check()
    if with_lp:
        assert torch.equal(lp_view, gw.to(torch.bfloat16))    # the bf16 copy is the rounded master weight


@pytest.mark.parametrize("with_lp,with_scale", [(False, False), (True, True)])
@pytest.mark.parametrize("n", OPT_SIZES)
def test_adamw_steps(n, with_lp, with_scale):
    print(f"adamw case n={n} lp={with_lp} scale={with_scale}", flush=True)
    w0 = gen.normal(1700, 0, (n,)).astype(np.float32)
    gs = [gen.normal(1700, 1 + t, (n,)).astype(np.float32) for t in range(4)]
    # the ABI takes the coefficients as float: the oracle gets the same float values (1 - 0.999f differs from 0.001 by 1.3e-5)
    lr, b1, b2, eps, wd, s = 1e-3, float(np.float32(0.9)), float(np.float32(0.999)), 1e-8, 1e-4, 0.6
    gw, gm, gv = dev(w0), torch.zeros(n, device="cuda:0"), torch.zeros(n, device="cuda:0")
    lp_view, lp_check = guarded((n,), torch.bfloat16)
    scale = dev(np.array([s])) if with_scale else None
    w, m, v = w0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t, g in enumerate(gs, start=1):
        gg = dev(g)
        B.adamw_step(gw, gg, gm, gv, t, lr, b1, b2, eps, wd, w_lp=lp_view if with_lp else None, grad_scale=scale)
        w, m, v, _ = T.adamw_step(w, g, m, v, t, lr, b1, b2, eps, wd, grad_scale=s if with_scale else 1.0)
        torch.cuda.synchronize()
        assert not gg.any()
        assert max_rel_err(host(gw), w) <= 1e-5
        assert max_rel_err(host(gm), m) <= 1e-5
        assert max_rel_err(host(gv), v) <= 1e-5
    lp_check()
    if with_lp:
        assert torch.equal(lp_view, gw.to(torch.bfloat16))


def test_many_tensors_in_one_launch_match_the_single_tensor_calls():
    """40 tensors of mixed sizes (two launch tables of 32 and 8), per-tensor weight decay, bf16 copies for some."""
    sizes = [1, 7, 64, 1000, 4097, 300001, 36864, 16] * 5
    mk = lambda k, n: dev(gen.normal(1900, k, (n,)))
    for adam in (False, True):
        recs, refs = [], []
        for k, n in enumerate(sizes):
            w, g = mk(10 * k, n), mk(10 * k + 1, n)
            s1, s2 = 0.1 * mk(10 * k + 2, n), (0.01 * mk(10 * k + 3, n)) ** 2
            lp = torch.empty(n, dtype=torch.bfloat16, device="cuda:0") if k % 3 == 0 else None
            wd = 1e-2 * (k % 4)
            refs.append(tuple(t.clone() for t in (w, g, s1, s2)) + (wd,))
            recs.append((w, g, s1, s2 if adam else None, lp, wd))
        tab = B.param_table(recs)
        scale = dev(np.array([0.8]))
        if adam:
            B.adamw_step_multi(tab, 3, 1e-2, grad_scale=scale)
        else:
            B.sgd_momentum_step_multi(tab, 0.05, 0.9, grad_scale=scale)
        for (w, g, s1, s2, lp, wd), (rw, rg, rs1, rs2, _) in zip(recs, refs):
            if adam:
                B.adamw_step(rw, rg, rs1, rs2, 3, 1e-2, weight_decay=wd, grad_scale=scale)
            else:
                B.sgd_momentum_step(rw, rg, rs1, 0.05, 0.9, wd, grad_scale=scale)
            torch.cuda.synchronize()
            assert torch.equal(w, rw) and torch.equal(s1, rs1) and not g.any()
            assert s2 is None or torch.equal(s2, rs2)
            assert lp is None or torch.equal(lp, w.to(torch.bfloat16))


def test_gradient_clip_scale():
    grads = [4.0 * gen.normal(1800, k, shp).astype(np.float32) for k, shp in enumerate([(300001,), (64, 64, 3, 3), (10,), (1,)])]
    gg = [dev(g) for g in grads]
    for max_norm in (5.0, 1e9):
        sc = B.clip_scale(gg, max_norm)
        torch.cuda.synchronize()
        want = T.clip_scale(grads, max_norm)
        assert abs(float(sc.item()) - want) <= 1e-5 * want
    assert float(B.clip_scale(gg, 1e9).item()) == 1.0


def test_host_validation_of_the_tail_entry_points():
    L = B.lib()
    assert L.nsk_global_avgpool_fwd(B.NSK_F32, B.NSK_NHWC, 0, 4, 2, 2, None, None, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_global_avgpool_fwd(B.NSK_F32, B.NSK_NHWC, 1, 4, 2, 2, None, None, None) == B.NSK_ERR_NULL
    assert L.nsk_softmax_xent_fwd(7, 4, 4, None, None, None, None, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_sgd_momentum_step(0, None, None, None, None, 0.1, 0.9, 0.0, None, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_sgd_momentum_step(4, None, None, None, None, 0.1, 0.9, 0.0, None, None) == B.NSK_ERR_NULL
    w = torch.zeros(8, device="cuda:0")
    assert L.nsk_adamw_step(4, w.data_ptr(), w.data_ptr(), w.data_ptr(), w.data_ptr(), None, 0, 0.1, 0.9, 0.999, 1e-8, 0.0,
                            None, None) == B.NSK_ERR_BAD_DESC        # steps count from 1
    assert L.nsk_adamw_step(4, w.data_ptr() + 4, w.data_ptr(), w.data_ptr(), w.data_ptr(), None, 1, 0.1, 0.9, 0.999, 1e-8,
                            0.0, None, None) == B.NSK_ERR_ALIGNMENT


# ----------------------------------------------------------------------------- full sizes (the shapes the bench's --train-step runs)

def test_tail_at_full_size_of_config_5_stage_a():
    """Average pool over [128, 256, 56, 56] bf16 (205 MB), 256 -> 1000 classifier on 128 samples, loss, and one
    SGD-momentum launch over 25.6 M parameters (a ResNet-50's worth) in one table entry: all compared in full."""
    N, C, H, W, K = 128, 256, 56, 56, 1000
    print(f"full-size tail {N, C, H, W, K}", flush=True)
    x = gen.to_bf16_grid(gen.normal(2200, 0, (N, C, H, W)) + 0.25)
    gx = to_gpu(x, "bf16", B.NSK_NHWC)
    pooled = B.global_avgpool_fwd(gx, B.NSK_NHWC)
    torch.cuda.synchronize()
    want_pooled = T.global_avgpool_fwd(x)
    assert max_rel_err(host(pooled), want_pooled) <= TOL["bf16"]
    dy = gen.to_bf16_grid(gen.normal(2200, 1, (N, C)))
    dx = B.global_avgpool_bwd(dev(dy, "bf16"), (N, C, H, W), B.NSK_NHWC)
    torch.cuda.synchronize()
    got = to_host(dx, B.NSK_NHWC)
    del dx
    assert max_rel_err(got[::7], T.global_avgpool_bwd(dy, (N, C, H, W))[::7]) <= TOL["bf16"]
    del got
    ph = gen.to_bf16_grid(want_pooled)
    w = gen.to_bf16_grid(gen.normal(2200, 2, (K, C)) / np.sqrt(C))
    b = (0.1 * gen.normal(2200, 3, (K,))).astype(np.float32)
    logits = B.linear_fwd(dev(ph, "bf16"), dev(w, "bf16"), dev(b))
    labels = (gen.uniform(2200, 4, (N,)) * K).astype(np.int32) % K
    torch.cuda.synchronize()
    zh = host(logits)
    assert max_rel_err(zh, T.linear_fwd(ph, w, b)) <= TOL["bf16"]
    loss, _ = B.softmax_xent_fwd(logits, torch.from_numpy(labels).cuda())
    dz = B.softmax_xent_bwd(logits, torch.from_numpy(labels).cuda())
    torch.cuda.synchronize()
    want_loss, _ = T.softmax_xent_fwd(zh, labels)
    assert abs(float(loss.item()) - want_loss) <= 1e-5 * want_loss
    assert max_rel_err(host(dz), T.softmax_xent_bwd(zh, labels)) <= TOL["bf16"]
    n = 25_557_032
    w0 = gen.normal(2201, 0, (n,)).astype(np.float32)
    g0 = gen.normal(2201, 1, (n,)).astype(np.float32)
    v0 = (0.1 * gen.normal(2201, 2, (n,))).astype(np.float32)
    gw, gg, gv = dev(w0), dev(g0), dev(v0)
    lp = torch.empty(n, dtype=torch.bfloat16, device="cuda:0")
    B.sgd_momentum_step_multi(B.param_table([(gw, gg, gv, None, lp, 1e-4)]), 0.1, 0.9)
    torch.cuda.synchronize()
    ww, vv, _ = T.sgd_momentum_step(w0, g0, v0, 0.1, 0.9, 1e-4)
    assert max_rel_err(host(gw), ww) <= 1e-5 and max_rel_err(host(gv), vv) <= 1e-5
    assert not gg.any() and torch.equal(lp, gw.to(torch.bfloat16))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,cols", [(768, 256), (5, 3), (33, 70), (1, 16), (1000, 2048)])
def test_transpose2d_is_an_exact_copy(rows, cols, dtype):
    a = on_grid(gen.normal(2300 + rows, 0, (rows, cols)), dtype)
    view, check = guarded((cols, rows), torch_dtype(dtype))
    B.transpose2d(dev(a, dtype), out=view)
    torch.cuda.synchronize()
    check()
    assert np.array_equal(host(view), a.T.astype(np.float64))
