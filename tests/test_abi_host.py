"""Host-only checks of the C ABI: the library loads, exports every symbol include/nsk.h declares,
and rejects bad arguments with the documented status codes before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2409_11600_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x10000)          # non-NULL, 16-byte aligned, never dereferenced on these paths
ODD = ctypes.c_void_p(0x10004)


def _declared():
    text = open(os.path.join(ROOT, "include", "nsk.h")).read()
    return sorted(set(re.findall(r"\b(nsk_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert set(names) == set(B.EXPORTS)
    L = B.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_status_strings():
    L = B.lib()
    assert L.nsk_version() >= 100
    seen = {L.nsk_status_string(s) for s in range(0, 7)}
    assert len(seen) == 7 and all(seen)
    assert L.nsk_status_string(99) == b"unknown status"
    assert L.nsk_last_hip_error() == 0


def test_out_dims_and_descriptor_validation():
    L = B.lib()
    d = B.conv_desc((64, 3, 224, 224), (64, 7, 7), 2, 3, 1, B.NSK_BF16, B.NSK_NHWC)
    assert B.conv2d_out_dims(d) == (112, 112)
    P, Q = ctypes.c_int(-7), ctypes.c_int(-7)
    assert L.nsk_conv2d_out_dims(None, ctypes.byref(P), ctypes.byref(Q)) == B.NSK_ERR_NULL
    for field, bad in (("N", 0), ("C", -1), ("stride_h", 0), ("dil_w", 0), ("pad_h", -1), ("dtype", 7), ("layout", 2)):
        d2 = B.conv_desc((2, 3, 8, 8), (4, 3, 3), 1, 1, 1, B.NSK_F32, B.NSK_NCHW)
        setattr(d2, field, bad)
        assert L.nsk_conv2d_out_dims(ctypes.byref(d2), ctypes.byref(P), ctypes.byref(Q)) == B.NSK_ERR_BAD_DESC
        assert (P.value, Q.value) == (-7, -7)
        assert L.nsk_conv2d_workspace_bytes(ctypes.byref(d2), B.NSK_PASS_FWD) == 0
    # filter larger than the padded image: extent query says 0, compute calls refuse
    d3 = B.conv_desc((1, 1, 2, 2), (1, 5, 5), 1, 0, 1, B.NSK_F32, B.NSK_NHWC)
    assert B.conv2d_out_dims(d3) == (0, 0)
    assert L.nsk_conv2d_fwd(ctypes.byref(d3), FAKE, FAKE, FAKE, None, 0, None) == B.NSK_ERR_BAD_DESC
    # more taps than the tap table holds
    d4 = B.conv_desc((1, 1, 32, 32), (1, 9, 9), 1, 0, 1, B.NSK_F32, B.NSK_NHWC)
    assert L.nsk_conv2d_fwd(ctypes.byref(d4), FAKE, FAKE, FAKE, None, 0, None) == B.NSK_ERR_UNSUPPORTED


def test_workspace_queries_are_consistent():
    L = B.lib()
    nhwc = B.conv_desc((8, 16, 32, 32), (16, 3, 3), 1, 1, 1, B.NSK_F32, B.NSK_NHWC)
    nchw = B.conv_desc((8, 16, 32, 32), (16, 3, 3), 1, 1, 1, B.NSK_F32, B.NSK_NCHW)
    assert L.nsk_conv2d_workspace_bytes(ctypes.byref(nhwc), B.NSK_PASS_FWD) == 0
    assert L.nsk_conv2d_workspace_bytes(ctypes.byref(nhwc), B.NSK_PASS_DGRAD) >= 16 * 16 * 9 * 4
    assert L.nsk_conv2d_workspace_bytes(ctypes.byref(nhwc), B.NSK_PASS_WGRAD) >= 16 * 16 * 9 * 4
    act = 8 * 16 * 32 * 32 * 4
    assert L.nsk_conv2d_workspace_bytes(ctypes.byref(nchw), B.NSK_PASS_FWD) >= 2 * act
    assert L.nsk_conv2d_workspace_bytes(ctypes.byref(nchw), 3) == 0
    bd = B.nsk_bn_desc_t(8, 16, 32, 32, B.NSK_F32, B.NSK_NHWC, 1e-5, 0.1, 1)
    assert L.nsk_bn_workspace_bytes(ctypes.byref(bd), B.NSK_BN_FWD) > 0
    assert L.nsk_bn_workspace_bytes(ctypes.byref(bd), 5) == 0


def test_compute_calls_reject_bad_arguments_without_a_gpu():
    L = B.lib()
    d = B.conv_desc((2, 8, 8, 8), (8, 3, 3), 1, 1, 1, B.NSK_F32, B.NSK_NCHW)
    need = L.nsk_conv2d_workspace_bytes(ctypes.byref(d), B.NSK_PASS_FWD)
    assert need > 0
    dp = ctypes.byref(d)
    assert L.nsk_conv2d_fwd(dp, None, FAKE, FAKE, FAKE, need, None) == B.NSK_ERR_NULL
    assert L.nsk_conv2d_fwd(dp, FAKE, ODD, FAKE, FAKE, need, None) == B.NSK_ERR_ALIGNMENT
    assert L.nsk_conv2d_fwd(dp, FAKE, FAKE, FAKE, None, 0, None) == B.NSK_ERR_WORKSPACE
    assert L.nsk_conv2d_fwd(dp, FAKE, FAKE, FAKE, FAKE, need - 1, None) == B.NSK_ERR_WORKSPACE
    assert L.nsk_conv2d_dgrad(dp, FAKE, FAKE, FAKE, 2, FAKE, 1 << 30, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_conv2d_dgrad(dp, FAKE, FAKE, None, 0, FAKE, 1 << 30, None) == B.NSK_ERR_NULL
    assert L.nsk_conv2d_wgrad(dp, FAKE, FAKE, FAKE, 0, None, 0, None) == B.NSK_ERR_WORKSPACE
    assert L.nsk_conv2d_wgrad(dp, FAKE, FAKE, ODD, 0, FAKE, 1 << 30, None) == B.NSK_ERR_ALIGNMENT
    bd = B.nsk_bn_desc_t(2, 8, 4, 4, B.NSK_F32, B.NSK_NHWC, 1e-5, 0.1, 1)
    bp = ctypes.byref(bd)
    args = [FAKE] * 9                        # x, residual, gamma, beta, out, mean, invstd, run_mean, run_var
    assert L.nsk_bn_relu_add_fwd(bp, *args, None, 0, None) == B.NSK_ERR_WORKSPACE
    args[0] = None
    assert L.nsk_bn_relu_add_fwd(bp, *args, FAKE, 1 << 20, None) == B.NSK_ERR_NULL
    args = [FAKE] * 9
    args[8] = None                           # running_mean without running_var
    assert L.nsk_bn_relu_add_fwd(bp, *args, FAKE, 1 << 20, None) == B.NSK_ERR_NULL
    bad = B.nsk_bn_desc_t(2, 8, 4, 4, B.NSK_F32, B.NSK_NHWC, -1.0, 0.1, 1)
    assert L.nsk_bn_relu_add_fwd(ctypes.byref(bad), *([FAKE] * 9), FAKE, 1 << 20, None) == B.NSK_ERR_BAD_DESC
    bargs = [FAKE] * 10
    bargs[1] = None                          # `out` is required when relu = 1
    assert L.nsk_bn_relu_add_bwd(bp, *bargs, FAKE, 1 << 20, None) == B.NSK_ERR_NULL
    pd = B.nsk_pool_desc_t(1, 4, 8, 8, 3, 3, 2, 2, 1, 1, B.NSK_F32, B.NSK_NHWC)
    assert L.nsk_maxpool2d_fwd(ctypes.byref(pd), FAKE, None, FAKE, None) == B.NSK_ERR_NULL
    pd.R = 12
    pd.S = 12
    assert L.nsk_maxpool2d_fwd(ctypes.byref(pd), FAKE, FAKE, FAKE, None) == B.NSK_ERR_UNSUPPORTED


def test_grouped_convolution_validation_without_a_gpu():
    L = B.lib()
    d = B.conv_desc((2, 12, 8, 8), (8, 3, 3), 1, 1, 1, B.NSK_F32, B.NSK_NHWC)
    dp = ctypes.byref(d)
    big = 1 << 30
    # groups must be positive and divide both channel counts (12 and 8): 1, 2, 4 do, 0, 3, 8 do not
    for groups in (0, -1, 3, 8, 12):
        for p in (B.NSK_PASS_FWD, B.NSK_PASS_DGRAD, B.NSK_PASS_WGRAD):
            assert L.nsk_conv2d_grouped_workspace_bytes(dp, groups, p) == 0
        assert L.nsk_conv2d_grouped_fwd(dp, groups, FAKE, FAKE, FAKE, FAKE, big, None) == B.NSK_ERR_BAD_DESC
        assert L.nsk_conv2d_grouped_dgrad(dp, groups, FAKE, FAKE, FAKE, 0, FAKE, big, None) == B.NSK_ERR_BAD_DESC
        assert L.nsk_conv2d_grouped_wgrad(dp, groups, FAKE, FAKE, FAKE, 0, FAKE, big, None) == B.NSK_ERR_BAD_DESC
    # one group: the same workspace as the plain call; more groups: the filter-sized parts shrink with the filter
    for p in (B.NSK_PASS_FWD, B.NSK_PASS_DGRAD, B.NSK_PASS_WGRAD):
        assert L.nsk_conv2d_grouped_workspace_bytes(dp, 1, p) == L.nsk_conv2d_workspace_bytes(dp, p)
    assert 0 < L.nsk_conv2d_grouped_workspace_bytes(dp, 4, B.NSK_PASS_DGRAD) <= L.nsk_conv2d_workspace_bytes(dp, B.NSK_PASS_DGRAD)
    assert L.nsk_conv2d_grouped_workspace_bytes(dp, 4, B.NSK_PASS_WGRAD) >= 8 * 3 * 9 * 4
    assert L.nsk_conv2d_grouped_workspace_bytes(dp, 4, 3) == 0
    # the other checks come in the same order as in the plain calls
    assert L.nsk_conv2d_grouped_fwd(dp, 4, None, FAKE, FAKE, None, 0, None) == B.NSK_ERR_NULL
    assert L.nsk_conv2d_grouped_fwd(dp, 4, FAKE, ODD, FAKE, None, 0, None) == B.NSK_ERR_ALIGNMENT
    assert L.nsk_conv2d_grouped_dgrad(dp, 4, FAKE, FAKE, FAKE, 2, FAKE, big, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_conv2d_grouped_dgrad(dp, 4, FAKE, FAKE, FAKE, 0, None, 0, None) == B.NSK_ERR_WORKSPACE
    assert L.nsk_conv2d_grouped_wgrad(dp, 4, FAKE, FAKE, FAKE, 0, FAKE, 16, None) == B.NSK_ERR_WORKSPACE
    assert L.nsk_conv2d_grouped_wgrad(dp, 4, FAKE, FAKE, ODD, 0, FAKE, big, None) == B.NSK_ERR_ALIGNMENT


def test_tail_entry_points_reject_bad_arguments_without_a_gpu():
    L = B.lib()
    # global average pool
    assert L.nsk_global_avgpool_fwd(B.NSK_F32, B.NSK_NHWC, 0, 4, 2, 2, FAKE, FAKE, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_global_avgpool_fwd(B.NSK_F32, 5, 1, 4, 2, 2, FAKE, FAKE, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_global_avgpool_fwd(B.NSK_F32, B.NSK_NHWC, 1, 4, 2, 2, None, FAKE, None) == B.NSK_ERR_NULL
    assert L.nsk_global_avgpool_bwd(B.NSK_BF16, B.NSK_NCHW, 1, 4, 2, 2, FAKE, ODD, 0, None) == B.NSK_ERR_ALIGNMENT
    assert L.nsk_global_avgpool_bwd(B.NSK_BF16, B.NSK_NCHW, 1, 4, 2, 2, FAKE, FAKE, 3, None) == B.NSK_ERR_BAD_DESC
    # fully connected layer: same workspace rules as the convolution it runs on
    ld = B.nsk_linear_desc_t(128, 512, 10, B.NSK_BF16)
    assert L.nsk_linear_workspace_bytes(ctypes.byref(ld), B.NSK_PASS_WGRAD) > 0
    assert L.nsk_linear_workspace_bytes(ctypes.byref(B.nsk_linear_desc_t(0, 512, 10, B.NSK_BF16)), B.NSK_PASS_FWD) == 0
    assert L.nsk_linear_fwd(None, FAKE, FAKE, None, FAKE, None, 0, None) == B.NSK_ERR_NULL
    assert L.nsk_linear_fwd(ctypes.byref(B.nsk_linear_desc_t(4, 4, 4, 9)), FAKE, FAKE, None, FAKE, None, 0, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_linear_fwd(ctypes.byref(ld), FAKE, FAKE, ODD, FAKE, None, 0, None) == B.NSK_ERR_ALIGNMENT
    assert L.nsk_linear_wgrad(ctypes.byref(ld), FAKE, FAKE, FAKE, FAKE, 0, None, 0, None) == B.NSK_ERR_WORKSPACE
    assert L.nsk_linear_dgrad(ctypes.byref(ld), FAKE, FAKE, None, 0, FAKE, 1 << 30, None) == B.NSK_ERR_NULL
    # loss
    assert L.nsk_softmax_xent_fwd(B.NSK_F32, 0, 10, FAKE, FAKE, FAKE, FAKE, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_softmax_xent_fwd(B.NSK_F32, 4, 10, FAKE, None, FAKE, FAKE, None) == B.NSK_ERR_NULL
    assert L.nsk_softmax_xent_bwd(B.NSK_F32, 4, 10, FAKE, FAKE, 1.0, ODD, None) == B.NSK_ERR_ALIGNMENT
    # optimizers
    assert L.nsk_sgd_momentum_step(0, FAKE, FAKE, FAKE, None, 0.1, 0.9, 0.0, None, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_sgd_momentum_step(4, FAKE, None, FAKE, None, 0.1, 0.9, 0.0, None, None) == B.NSK_ERR_NULL
    assert L.nsk_sgd_momentum_step(4, FAKE, FAKE, ODD, None, 0.1, 0.9, 0.0, None, None) == B.NSK_ERR_ALIGNMENT
    assert L.nsk_adamw_step(4, FAKE, FAKE, FAKE, FAKE, None, 0, 0.1, 0.9, 0.999, 1e-8, 0.0, None, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_adamw_step(4, FAKE, FAKE, FAKE, FAKE, None, 1, 0.1, 1.0, 0.999, 1e-8, 0.0, None, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_adamw_step(4, FAKE, FAKE, FAKE, None, None, 1, 0.1, 0.9, 0.999, 1e-8, 0.0, None, None) == B.NSK_ERR_NULL
    tab = (B.nsk_param_t * 2)(B.nsk_param_t(0x10000, 0x10000, 0x10000, None, None, 8, 0.0),
                              B.nsk_param_t(0x10000, 0x10004, 0x10000, None, None, 8, 0.0))
    assert L.nsk_sgd_momentum_step_multi(2, tab, 0.1, 0.9, None, None) == B.NSK_ERR_ALIGNMENT   # nothing launched
    assert L.nsk_sgd_momentum_step_multi(0, tab, 0.1, 0.9, None, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_adamw_step_multi(1, tab, 1, 0.1, 0.9, 0.999, 1e-8, None, None) == B.NSK_ERR_NULL     # AdamW needs state2
    assert L.nsk_sumsq_accumulate(0, FAKE, FAKE, FAKE, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_clip_scale(FAKE, 0.0, FAKE, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_clip_scale(None, 5.0, FAKE, None) == B.NSK_ERR_NULL


def test_recurrent_entry_points_reject_bad_arguments_without_a_gpu():
    L = B.lib()
    assert L.nsk_embedding_fwd(B.NSK_F32, 0, 8, 16, FAKE, FAKE, FAKE, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_embedding_fwd(B.NSK_F32, 4, 8, 16, None, FAKE, FAKE, None) == B.NSK_ERR_NULL
    assert L.nsk_embedding_fwd(B.NSK_BF16, 4, 8, 16, FAKE, ODD, FAKE, None) == B.NSK_ERR_ALIGNMENT
    assert L.nsk_embedding_bwd(B.NSK_F32, 4, 8, 16, FAKE, FAKE, FAKE, 2, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_embedding_bwd(B.NSK_F32, 4, 8, 16, FAKE, FAKE, None, 0, None) == B.NSK_ERR_NULL
    assert L.nsk_gru_gates_fwd(B.NSK_F32, 4, 0, *([FAKE] * 7), None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_gru_gates_fwd(B.NSK_F32, 4, 8, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, None) == B.NSK_ERR_NULL
    assert L.nsk_gru_gates_bwd(9, 4, 8, *([FAKE] * 8), None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_gru_gates_bwd(B.NSK_F32, 4, 8, FAKE, FAKE, None, None, None, FAKE, FAKE, FAKE, None) == B.NSK_ERR_NULL     # dh_a is required
    assert L.nsk_gru_gates_bwd(B.NSK_F32, 4, 8, FAKE, FAKE, FAKE, ODD, None, FAKE, FAKE, FAKE, None) == B.NSK_ERR_ALIGNMENT
    assert L.nsk_gru_step_supported(50, 256) == 1 and L.nsk_gru_step_supported(50, 254) == 0 and L.nsk_gru_step_supported(257, 256) == 0
    assert L.nsk_gru_step_fwd(B.NSK_F32, 0, 8, *([FAKE] * 7), None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_gru_step_fwd(B.NSK_F32, 4, 8, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, None) == B.NSK_ERR_NULL
    assert L.nsk_gru_step_fwd(B.NSK_F32, 4, 8, FAKE, FAKE, FAKE, FAKE, ODD, FAKE, FAKE, None) == B.NSK_ERR_ALIGNMENT
    assert L.nsk_gru_step_fwd(B.NSK_F32, 5000, 256, *([FAKE] * 7), None) == B.NSK_ERR_UNSUPPORTED
    assert L.nsk_gru_step_bwd(B.NSK_F32, 4, 8, FAKE, FAKE, None, None, None, FAKE, FAKE, FAKE, FAKE, None) == B.NSK_ERR_NULL   # no gradient source
    assert L.nsk_gru_step_bwd(B.NSK_F32, 4, 8, FAKE, FAKE, FAKE, None, ODD, FAKE, FAKE, FAKE, FAKE, None) == B.NSK_ERR_ALIGNMENT
    assert L.nsk_gru_step_bwd(B.NSK_BF16, 4, 6, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, FAKE, FAKE, None) == B.NSK_ERR_UNSUPPORTED
    assert L.nsk_transpose2d(B.NSK_F32, 0, 4, FAKE, FAKE, None) == B.NSK_ERR_BAD_DESC
    assert L.nsk_transpose2d(B.NSK_F32, 4, 4, FAKE, None, None) == B.NSK_ERR_NULL
    # few rows: the per-element product kernels validate like the rest
    small = B.nsk_linear_desc_t(50, 256, 768, B.NSK_F32)
    assert L.nsk_linear_fwd(ctypes.byref(small), FAKE, None, None, FAKE, None, 0, None) == B.NSK_ERR_NULL
    assert L.nsk_linear_dgrad(ctypes.byref(small), FAKE, FAKE, ODD, 0, None, 0, None) == B.NSK_ERR_ALIGNMENT
    assert L.nsk_linear_dgrad(ctypes.byref(small), FAKE, FAKE, FAKE, 5, None, 0, None) == B.NSK_ERR_BAD_DESC


def test_binding_raises_loudly_when_library_is_missing(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libnsk.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        B.lib()
