#!/usr/bin/env python3
"""Benchmark of the residual-CNN training hot path on one MI355X.

A step is one forward + backward pass of the workload (every libnsk call of the unit list) on
seeded synthetic tensors that are already resident in HBM.  Default workload: the fp32 basic
residual block (N=128, C=K=64, 32x32), NHWC.  Prints ONE JSON line:

  value        images/s of the whole step (batch * steps / wall time between two device syncs)
  roofline     the dominant kernel (largest share of step time): algorithmic FLOPs (or bytes) per
               launch / its average launch duration, measured with HIP events recorded on the
               launching stream around that kernel's launches INSIDE the timed steps
  cpu_baseline the CPU oracle (tests' reference, never tuned) timed on the host cores on the same
               workload, bounded to about 10-30 s of CPU work

Other workloads: --config {1,2,3,4,5} [--stage A|B] [--batch N].  --breakdown prints a per-call
table to stderr.  Runs on one GPU only.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"mfma_f32": 157.3e12, "mfma_bf16": 2516.6e12, "hbm": 8.0e12}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--stage", default="A")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--layout", default="nhwc", choices=["nhwc", "nchw"])
    ap.add_argument("--no-graph", action="store_true", help="issue every call from Python instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--breakdown", action="store_true")
    return ap.parse_args()


def call_cost(net, f, args):
    """(kind, flops, algorithmic bytes) of one libnsk call, from its descriptor (integer bookkeeping)."""
    from paper_2409_11600_amd import binding as B
    name = f.__name__
    d = args[0]._obj
    es = 2 if d.dtype == B.NSK_BF16 else 4
    if name.startswith("nsk_conv2d"):
        P, Q = B.conv2d_out_dims(d)
        flops = 2.0 * d.N * P * Q * d.K * d.C * d.R * d.S
        x, y, w = d.N * d.H * d.W * d.C, d.N * P * Q * d.K, d.K * d.C * d.R * d.S
        if name.endswith("wgrad"):
            byts = (x + y) * es + w * 4
        else:
            byts = (x + y + w) * es
        # forward and backward-data of one layer run the same kernel on the same GEMM shape
        kind = "conv2d_wgrad" if name.endswith("wgrad") else "conv2d_fwd/dgrad"
        return kind, flops, byts
    if name.startswith("nsk_bn"):
        e = d.N * d.C * d.H * d.W
        res = (args[2] if name.endswith("fwd") else args[8]) is not None
        if name.endswith("fwd"):
            byts = (2 + res + 1) * e * es          # stats read + apply read (+ residual) + write
        else:
            byts = (6 if d.relu else 4) * e * es + (1 + res) * e * es   # two passes over x,(out),dout + writes
        return name[len("nsk_"):], 0.0, byts
    if name.startswith("nsk_maxpool"):
        e_in = d.N * d.C * d.H * d.W
        e_out = e_in // 4
        return name[len("nsk_"):], 0.0, (e_in + e_out) * es + e_out
    return name, 0.0, 0.0


def stored_traffic(workload, kind):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary
    (profiles/traffic.txt: `<workload> <kernel kind> <bytes>`), or None if no line covers it."""
    path = os.path.join(ROOT, "profiles", "traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 3 and not line.startswith("#") and f[0] == workload and f[1] == kind:
                return float(f[2])
    except OSError:
        pass
    return None


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import nsk_inputs as gen
    from paper_2409_11600_amd import binding as B
    from paper_2409_11600_amd.network import GpuNetwork

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.lib()  # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    wl = gen.workload(a.config, batch=a.batch, stage=a.stage)
    tensors = gen.workload_tensors(wl)
    layout = B.NSK_NHWC if a.layout == "nhwc" else B.NSK_NCHW
    net = GpuNetwork(wl, tensors, layout=layout)
    batch = wl["input"][0]
    calls = net.fwd_calls + net.bwd_calls
    costs = [call_cost(net, f, args) for f, args in calls]
    stream = torch.cuda.Stream()
    st = ctypes.c_void_p(stream.cuda_stream)

    def issue(record=None):
        for i, (f, args) in enumerate(calls):
            if record is not None and i in record:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                rc = f(*args, st)
                e1.record(stream)
                record[i].append((e0, e1))
            else:
                rc = f(*args, st)
            if rc != B.NSK_OK:
                raise B.NskError(rc, f.__name__)

    with torch.cuda.stream(stream):
        # ---- warm-up, with every call bracketed by events: finds the dominant kernel
        probe = {i: [] for i in range(len(calls))}
        for w in range(max(a.warmup, 2)):
            issue(probe if w >= 1 else None)
        stream.synchronize()
        per_call_ms = [float(np.mean([e0.elapsed_time(e1) for e0, e1 in probe[i]])) for i in range(len(calls))]
        # group by (kind, cost): the same kernel on the same shape
        groups = {}
        for i, c in enumerate(costs):
            groups.setdefault(c, []).append(i)
        dominant = max(groups, key=lambda c: sum(per_call_ms[i] for i in groups[c]))
        dom_idx = groups[dominant]

        # ---- optional HIP graph of the whole step (removes the Python/ctypes launch gaps)
        graph = None
        if not a.no_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                gst = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
                for f, args in calls:
                    rc = f(*args, gst)
                    if rc != B.NSK_OK:
                        raise B.NskError(rc, f.__name__)
            graph.replay()
            stream.synchronize()

        # ---- timed region A: the step, back to back
        stream.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            if graph is not None:
                graph.replay()
            else:
                issue()
        stream.synchronize()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        # ---- timed region B: same steps issued call by call with events around the dominant kernel.
        # A forward call launches exactly that kernel; a backward-data call also packs the filter
        # first, so when both are in the group only the forward launches are bracketed.
        fwd_only = [i for i in dom_idx if calls[i][0].__name__ == "nsk_conv2d_fwd"]
        timed_idx = fwd_only or dom_idx
        rec = {i: [] for i in timed_idx}
        for _ in range(a.steps):
            issue(rec)
        stream.synchronize()
    dom_ms = float(np.mean([e0.elapsed_time(e1) for i in timed_idx for e0, e1 in rec[i]]))
    ms_per_step = (t1 - t0) * 1e3 / a.steps
    value = batch * a.steps / (t1 - t0)

    kind, flops, byts = dominant
    if flops > 0 and flops / byts > (PEAK["mfma_bf16" if wl["dtype"] == "bf16" else "mfma_f32"] / PEAK["hbm"]):
        peak = PEAK["mfma_bf16" if wl["dtype"] == "bf16" else "mfma_f32"]
        roof = dict(bound="mfma", achieved=flops / (dom_ms * 1e-3) / 1e12, peak=peak / 1e12, unit="TFLOP/s")
    else:
        roof = dict(bound="hbm", achieved=byts / (dom_ms * 1e-3) / 1e9, peak=PEAK["hbm"] / 1e9, unit="GB/s")
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = stored_traffic(wl["name"], kind)
    roof["kernel"] = kind
    roof["launch_ms"] = dom_ms
    roof["launches_per_step"] = len(dom_idx)
    roof["algorithmic_per_launch"] = flops if roof["bound"] == "mfma" else byts

    conv_flops = sum(c[1] for c in costs)
    conv_ms = sum(per_call_ms[i] for i, c in enumerate(costs) if c[1] > 0)
    if a.breakdown:
        print(f"{'call':<22}{'ms':>9}{'TFLOP/s':>10}{'GB/s':>9}", file=sys.stderr)
        for i, c in enumerate(costs):
            ms = per_call_ms[i]
            print(f"{c[0]:<22}{ms:9.4f}{c[1] / ms / 1e9:10.1f}{c[2] / ms / 1e6:9.0f}", file=sys.stderr)
        print(f"sum of calls {sum(per_call_ms):.3f} ms; step {ms_per_step:.3f} ms", file=sys.stderr)

    out = {
        "metric": "conv fwd+dgrad+wgrad TFLOP/s & % MFMA peak; residual-block images/s at 1 GPU",
        "value": value, "unit": "images/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl["dtype"] == "f32" else "bf16", "data": "synthetic",
        "config": {"workload": f"{wl['name']}: {len(wl['units'])} units, input {list(wl['input'])}, "
                               f"{a.layout}, forward+backward", "batch": batch, "hip_graph": graph is not None},
        "conv_tflops": conv_flops / (conv_ms * 1e-3) / 1e12,
        "conv_frac_of_mfma_peak": conv_flops / (conv_ms * 1e-3) / PEAK["mfma_bf16" if wl["dtype"] == "bf16" else "mfma_f32"],
        "roofline": roof,
    }

    if not a.no_cpu_baseline:
        import oracle
        from oracle import network as onet
        # bounded sample: the oracle runs about 9 GFLOP/s on 8 cores, so cap the work at ~100 GFLOP
        total_gflop = conv_flops / 1e9
        sample_batch = batch if total_gflop <= 100 else max(1, int(batch * 100 / total_gflop))
        swl = gen.workload(a.config, batch=sample_batch, stage=a.stage)
        stens = gen.workload_tensors(swl)
        c0 = time.perf_counter()
        f = onet.forward(swl, stens["x"], stens["params"])
        onet.backward(swl, f, stens["params"], stens["dout"])
        c1 = time.perf_counter()
        out["cpu_baseline"] = {"value": sample_batch / (c1 - c0), "unit": "images/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": f"{sample_batch} of {batch} images, one forward+backward of the same workload "
                                         f"({c1 - c0:.1f} s)"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
