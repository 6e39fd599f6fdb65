"""The entry point that allocates nothing: nsk_bn_relu_add_fwd_static keeps its partial sums in a device array of
the library instead of a caller workspace.  It must give exactly what nsk_bn_relu_add_fwd gives (same kernels), on
two calls in a row that share the array, the second on a smaller tensor, and must meet the oracle's bar."""
import ctypes

import numpy as np
import pytest
import torch

import nsk_inputs as gen
import oracle
from paper_2409_11600_amd import binding as B
from parity import TOL, max_rel_err, on_grid, to_gpu, to_host

# (N, C, H, W) of the first and of the second, smaller call
PAIRS = [("bf16", (16, 256, 28, 28), (3, 64, 9, 11)), ("f32", (32, 64, 32, 32), (2, 24, 7, 5)),
         ("bf16", (8, 1024, 14, 14), (8, 16, 32, 32))]


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,first,second", PAIRS)
def test_static_scratch_call_equals_the_workspace_call(dtype, first, second):
    print(f"no-alloc bn {dtype} {first} then {second}", flush=True)
    assert B.lib().nsk_static_scratch_bytes() == 8 << 20
    ws = B.Workspace()
    for k, shape in enumerate((first, second)):
        seed = 7100 + 10 * PAIRS.index((dtype, first, second)) + k
        x = on_grid(1.3 * gen.normal(seed, 0, shape) + 0.4, dtype)
        r = on_grid(gen.normal(seed, 1, shape), dtype)
        g = (1.0 + 0.3 * gen.normal(seed, 3, (shape[1],))).astype(np.float32)
        b = (0.2 * gen.normal(seed, 4, (shape[1],))).astype(np.float32)
        gx, gr = to_gpu(x, dtype, B.NSK_NHWC), to_gpu(r, dtype, B.NSK_NHWC)
        gg, gb = torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda()
        rm0 = torch.zeros(shape[1], device="cuda")
        rv0 = torch.ones(shape[1], device="cuda")
        rm1, rv1 = rm0.clone(), rv0.clone()
        out0, mean0, inv0 = B.bn_relu_add_fwd(gx, gg, gb, gr, 1e-5, True, ws=ws, running_mean=rm0, running_var=rv0)
        # outputs created before the call: the call itself must not need the allocator
        out1, mean1, inv1 = torch.full_like(gx, float("nan")), torch.empty_like(mean0), torch.empty_like(inv0)
        torch.cuda.synchronize()
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        B.bn_relu_add_fwd_static(gx, gg, gb, gr, 1e-5, True, running_mean=rm1, running_var=rv1, out=out1,
                                 save_mean=mean1, save_invstd=inv1)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
        assert torch.equal(out0, out1) and torch.equal(mean0, mean1) and torch.equal(inv0, inv1)
        assert torch.equal(rm0, rm1) and torch.equal(rv0, rv1)
        want_out, want_mean, want_inv = oracle.bn_relu_add_fwd(x, g, b, r, 1e-5, True)
        assert max_rel_err(to_host(out1, B.NSK_NHWC), want_out) <= TOL[dtype]
        assert max_rel_err(mean1.cpu().numpy(), want_mean) <= 1e-5
        assert max_rel_err(inv1.cpu().numpy(), want_inv) <= 1e-5


def test_static_scratch_call_rejects_what_does_not_fit():
    """A descriptor whose partial sums exceed the static array is refused with NSK_ERR_WORKSPACE (host check)."""
    L = B.lib()
    d = B.nsk_bn_desc_t(128, 2048, 14, 14, B.NSK_BF16, B.NSK_NHWC, 1e-5, 0.1, 1)
    assert L.nsk_bn_workspace_bytes(ctypes.byref(d), B.NSK_BN_FWD) > L.nsk_static_scratch_bytes()
    one = ctypes.c_void_p(256)       # never dereferenced: the size check comes first
    rc = L.nsk_bn_relu_add_fwd_static(ctypes.byref(d), one, None, one, one, one, one, one, None, None, None)
    assert rc == B.NSK_ERR_WORKSPACE
