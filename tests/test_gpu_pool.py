"""The memory pool on the device: libnsk calls run on buffers it hands out, with no PyTorch allocation in the loop,
and nothing is allocated after the first iteration (section "Caching and Pooling")."""
import ctypes

import numpy as np
import pytest
import torch

import nsk_inputs as gen
import oracle
from paper_2409_11600_amd import binding as B
from parity import TOL, max_rel_err

pytestmark = pytest.mark.gpu


def test_convolutions_on_pooled_device_buffers_match_the_oracle_and_stop_allocating():
    L = B.lib()
    N, C, H, W, K = 4, 16, 12, 12, 32
    x = gen.normal(2100, 0, (N, C, H, W)).astype(np.float32)
    w = gen.he_normal(2100, 1, (K, C, 3, 3)).astype(np.float32)
    want = oracle.conv2d_fwd(x, w, 1, 1, 1)
    xh = torch.from_numpy(np.ascontiguousarray(x.transpose(0, 2, 3, 1))).pin_memory()
    wh = torch.from_numpy(np.ascontiguousarray(w.transpose(0, 2, 3, 1))).pin_memory()
    yh = torch.empty((N, H, W, K), dtype=torch.float32).pin_memory()
    d = B.conv_desc((N, C, H, W), (K, 3, 3), 1, 1, 1, B.NSK_F32, B.NSK_NHWC)
    pool = B.Pool(B.NSK_POOL_DEVICE)
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
    hip.hipDeviceSynchronize.argtypes = []
    try:
        for it in range(3):
            dx, dw, dy = pool.get(xh.numel() * 4), pool.get(wh.numel() * 4), pool.get(yh.numel() * 4)
            assert hip.hipMemcpy(dx, xh.data_ptr(), xh.numel() * 4, 1) == 0          # host to device
            assert hip.hipMemcpy(dw, wh.data_ptr(), wh.numel() * 4, 1) == 0
            rc = L.nsk_conv2d_fwd(ctypes.byref(d), ctypes.c_void_p(dx), ctypes.c_void_p(dw), ctypes.c_void_p(dy), None, 0, None)
            assert rc == B.NSK_OK
            assert hip.hipDeviceSynchronize() == 0
            assert hip.hipMemcpy(yh.data_ptr(), dy, yh.numel() * 4, 2) == 0          # device to host
            got = yh.numpy().transpose(0, 3, 1, 2).astype(np.float64)
            assert max_rel_err(got, want) <= TOL["f32"]
            for p in (dx, dw, dy):
                pool.put(p)
            assert pool.stats()["allocations"] == 3                                  # all from the first iteration
        g, created = pool.cached("w.grad", wh.numel() * 4)
        assert created and pool.cached("w.grad", wh.numel() * 4) == (g, False)
    finally:
        pool.destroy()
