"""Helpers shared by the GPU parity tests (no arithmetic of the method)."""
import numpy as np
import torch

import nsk_inputs as gen
from paper_2409_11600_amd import binding as B

TOL = {"f32": 1e-4, "bf16": 2e-2}      # max-relative-error bars stated for this path


def max_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max_i |got_i - want_i| / max(|want_i|, rms(want)): element-wise relative error, floored at the
    tensor's RMS so exact or near zeros (post-ReLU, cells no tap reaches) do not divide by ~0."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(want * want)))
    floor = max(rms, 1e-30)
    return float(np.max(np.abs(got - want) / np.maximum(np.abs(want), floor)))


def torch_dtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def on_grid(a: np.ndarray, dtype: str) -> np.ndarray:
    return gen.to_bf16_grid(a) if dtype == "bf16" else np.ascontiguousarray(a, dtype=np.float32)


def to_gpu(a: np.ndarray, dtype: str, layout: int) -> torch.Tensor:
    """Host NCHW / KCRS float array -> device tensor in the physical layout."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if layout == B.NSK_NHWC and t.dim() == 4:
        t = t.permute(0, 2, 3, 1)
    return t.contiguous().to("cuda:0", dtype=torch_dtype(dtype))


def to_host(t: torch.Tensor, layout: int) -> np.ndarray:
    """Device tensor in the physical layout -> host NCHW / KCRS float64."""
    a = t.detach().to(torch.float32).cpu()
    if layout == B.NSK_NHWC and a.dim() == 4:
        a = a.permute(0, 3, 1, 2)
    return a.contiguous().numpy().astype(np.float64)


def guarded(shape, dtype, fill=float("nan"), guard=512):
    """A tensor view with NaN canaries on both sides; returns (view, check) where check() asserts the
    canaries are intact."""
    n = int(np.prod(shape))
    guard_elems = guard
    raw = torch.full((n + 2 * guard_elems,), fill, dtype=dtype, device="cuda:0")
    view = raw[guard_elems:guard_elems + n].view(*shape)

    def check():
        lo, hi = raw[:guard_elems], raw[guard_elems + n:]
        assert bool(torch.isnan(lo).all()) and bool(torch.isnan(hi).all()), "kernel wrote outside its output"

    return view, check
