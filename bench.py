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
  bf16_...     (default run only) the figures the target is quoted on: FLOP-weighted TFLOP/s and fraction of the
               bf16 MFMA peak over the 3x3 layers of configurations 4 and 5 (forward + backward-data +
               backward-weight, cold buffers), and the step time of the bf16 workloads 3, 4, 5A, 5B

Other workloads: --config {1,2,3,4,5} [--stage A|B] [--batch N].  --breakdown prints a per-call
table to stderr.  --train-step adds a "train_step" object: the same workload followed by the head of the network,
the loss, their backward passes and the SGD update of every parameter, timed as one HIP graph.  --no-fusion /
--no-stats switch the fused batch-norm statistics and the ReLU-mask hand-over off (A/B runs).  Runs on one GPU only.

--layers prints, instead, one line per distinct convolution layer of configurations 2-5 at its full
size: microseconds and TFLOP/s of forward, backward-data and backward-weight, the fraction of the
MFMA peak and the fraction of the layer's own roofline cap min(MFMA peak, intensity x 8 TB/s), and
the FLOP-weighted total over the bf16 3x3 layers of configurations 4 and 5.  Every call of a layer
runs on its own buffer set, rotated so that the sets together exceed the 256 MB last-level cache; the calls of a
pass are replayed from one HIP graph, so the cost of issuing them from Python is not in the figures.

--grouped prints the same kind of table for grouped convolution layers (the grouped entry points; not a workload of
the paper): depthwise layers are bound by memory bandwidth, so the table gives GB/s of algorithmic traffic
(x + y + w once) against the 8 TB/s peak next to TFLOP/s.
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
    ap.add_argument("--no-extras", action="store_true",
                    help="leave out the bf16 figures the default run appends (3x3 layer TFLOP/s of configurations 4 and 5, "
                         "step times of the bf16 workloads)")
    ap.add_argument("--no-stats", action="store_true",
                    help="keep the ReLU-mask hand-over but let every batch-norm compute its own statistics")
    ap.add_argument("--no-fusion", action="store_true",
                    help="plain entry points only: no statistics hand-over from convolution to batch-norm, no ReLU mask")
    ap.add_argument("--fused-act", action="store_true",
                    help="a conv + batch-norm + ReLU that feeds one convolution does not store its normalised activation: that "
                         "convolution applies it on load (measured: no gain on configuration 2, whose kernels have the fused "
                         "load, 3-5%% slower where the activation is applied into the workspace instead; off by default)")
    ap.add_argument("--overlap", action="store_true",
                    help="issue the backward-weight calls on a second stream (measured: no gain on MI355X, the "
                         "convolution kernels already hold every CU)")
    ap.add_argument("--train-step", action="store_true",
                    help="also time the whole training step: the workload followed by average pool, fully connected "
                         "layer, loss, their backward passes and the SGD update of every parameter")
    ap.add_argument("--gru", action="store_true",
                    help="time the recurrent workload instead: embedding + GRU(256) + output layer, batch 50, sequence "
                         "length 200, vocabulary 32768, 2 classes, forward + backward through time + clipped AdamW")
    ap.add_argument("--layers", action="store_true", help="per-layer convolution table instead of the step benchmark")
    ap.add_argument("--grouped", action="store_true", help="table of grouped / depthwise convolution layers")
    return ap.parse_args()


def _time_calls(torch, fn, sets, repeats):
    """Milliseconds per call of fn over `repeats` calls on rotating buffer sets.  The calls are captured into one HIP
    graph and the replay is timed, so the Python and ctypes cost of issuing a call (10-20 us) does not show in layers
    that run shorter than that."""
    nset = len(sets)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for i in range(3):
            fn(sets[i % nset])
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(repeats):
                fn(sets[i % nset])
        graph.replay()
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        graph.replay()
        e1.record(stream)
        stream.synchronize()
    return e0.elapsed_time(e1) / repeats


def distinct_layers(configs=((2, "A"), (3, "A"), (4, "A"), (5, "A"), (5, "B"))):
    """(tag, (dtype, N, C, H, W, K, R, stride, pad)) of every distinct convolution layer of the given workloads."""
    import nsk_inputs as gen
    seen, layers = set(), []
    for config, stage in configs:
        wl = gen.workload(config, stage=stage)
        shapes = gen.tensor_shapes(wl)
        for u in wl["units"]:
            if u["kind"] == "pool":
                continue
            key = (wl["dtype"],) + tuple(shapes[u["src"]]) + (u["K"], u["R"], u["stride"], u["pad"])
            if key not in seen:
                seen.add(key)
                layers.append((f"C{config}{stage if config == 5 else ''}", key))
    return layers


def time_layers(layers, repeats=20):
    """Times forward, backward-data and backward-weight of each layer at full size on cold buffers (see the module
    docstring) and yields one row per pass."""
    import torch
    from paper_2409_11600_amd import binding as B

    ws = B.Workspace()
    gen_t = torch.Generator(device="cuda").manual_seed(7)
    for cfg, (dtype, N, C, H, W, K, R, stride, pad) in layers:
        dt = torch.bfloat16 if dtype == "bf16" else torch.float32
        es = 2 if dtype == "bf16" else 4
        peak = PEAK["mfma_bf16" if dtype == "bf16" else "mfma_f32"]
        P = (H + 2 * pad - R) // stride + 1
        flops = 2.0 * N * P * P * K * C * R * R
        xb, yb, wb = N * H * W * C * es, N * P * P * K * es, K * R * R * C
        # a filter narrower than the stride reads only the pixels it touches (a 1x1 stride-2 layer: a quarter of x);
        # backward-data still writes all of dx (zeros where nothing arrives)
        touched = min(1.0, R / stride) ** 2
        nset = max(2, int(300e6 // (xb + yb)) + 1)          # buffer sets that together exceed the last-level cache
        sets = []
        for _ in range(nset):
            x = torch.randn(N, H, W, C, device="cuda", generator=gen_t).to(dt)
            dy = torch.randn(N, P, P, K, device="cuda", generator=gen_t).to(dt)
            sets.append((x, dy, torch.empty_like(dy), torch.empty_like(x)))
        w = (torch.randn(K, R, R, C, device="cuda", generator=gen_t) * (2.0 / (C * R * R)) ** 0.5).to(dt)
        dw = torch.empty(K, R, R, C, device="cuda")
        passes = {
            "fwd": (lambda s: B.conv2d_fwd(s[0], w, stride, pad, 1, out=s[2], ws=ws), (xb * touched + yb + wb * es)),
            "dgrad": (lambda s: B.conv2d_dgrad(s[1], w, (N, C, H, W), stride, pad, 1, out=s[3], ws=ws), (xb + yb + wb * es)),
            "wgrad": (lambda s: B.conv2d_wgrad(s[0], s[1], (K, C, R, R), stride, pad, 1, out=dw, ws=ws), (xb * touched + yb + wb * 4)),
        }
        name = f"{R}x{R} s{stride} {C}->{K} @{H}x{W} N={N} {dtype}"
        for pname, (fn, byts) in passes.items():
            ms = _time_calls(torch, fn, sets, repeats)
            cap = min(peak, flops / byts * PEAK["hbm"])
            tf = flops / ms / 1e9
            yield {"config": cfg, "layer": name, "pass": pname, "us": ms * 1e3, "tflops": tf, "flops": flops,
                   "frac_of_mfma_peak": tf * 1e12 / peak, "roofline_cap_tflops": cap / 1e12, "frac_of_cap": tf * 1e12 / cap,
                   "is_bf16_3x3": dtype == "bf16" and R == 3 and cfg in ("C4", "C5A", "C5B")}
        del sets


def head_figure(rows):
    """FLOP-weighted TFLOP/s over the bf16 3x3 layers of configurations 4 and 5, all passes: total FLOPs / total time."""
    fl = sum(r["flops"] for r in rows if r["is_bf16_3x3"])
    us = sum(r["us"] for r in rows if r["is_bf16_3x3"])
    return fl / us / 1e6 if us else 0.0


def layer_table(repeats=20):
    """Per-layer convolution timings at full size (see the module docstring)."""
    print(f"{'cfg':<5}{'layer':<38}{'pass':<7}{'us':>9}{'TFLOP/s':>9}{'%peak':>7}{'cap TF':>8}{'%cap':>6}")
    rows = []
    for r in time_layers(distinct_layers(), repeats):
        print(f"{r['config']:<5}{r['layer']:<38}{r['pass']:<7}{r['us']:9.1f}{r['tflops']:9.1f}{100 * r['frac_of_mfma_peak']:7.1f}"
              f"{r['roofline_cap_tflops']:8.0f}{100 * r['frac_of_cap']:6.1f}", flush=True)
        rows.append(r)
    head = head_figure(rows)
    print(f"bf16 3x3 layers of configurations 4 and 5, all passes: {head:.1f} TFLOP/s = {100 * head * 1e12 / PEAK['mfma_bf16']:.1f}% of the bf16 MFMA peak")
    print(json.dumps({"metric": "bf16 3x3 conv TFLOP/s over configs 4 and 5 (fwd+dgrad+wgrad, FLOP-weighted)", "value": head,
                      "unit": "TFLOP/s", "frac_of_mfma_peak": head * 1e12 / PEAK["mfma_bf16"], "layers": rows}))


def bf16_target_figures(replays=10):
    """What the target is quoted on, for the default run's JSON line: the bf16 3x3 layers of configurations 4 and 5
    (each pass on cold buffers, 20 calls from one HIP graph) and the step time of the bf16 workloads (forward +
    backward, fused call sequence, `replays` replays of one HIP graph each)."""
    import torch
    import nsk_inputs as gen
    from paper_2409_11600_amd.network import GpuNetwork

    layers = [l for l in distinct_layers(((4, "A"), (5, "A"), (5, "B"))) if l[1][0] == "bf16" and l[1][6] == 3]
    rows = list(time_layers(layers))
    head = head_figure(rows)
    out = {"bf16_3x3_conv_tflops": head, "bf16_3x3_conv_frac_of_mfma_peak": head * 1e12 / PEAK["mfma_bf16"],
           "bf16_3x3_layers": [{k: (round(r[k], 4) if isinstance(r[k], float) else r[k])
                                for k in ("config", "layer", "pass", "us", "tflops", "frac_of_mfma_peak")} for r in rows],
           "bf16_step_ms": {}}
    for config, stage in ((3, "A"), (4, "A"), (5, "A"), (5, "B")):
        wl = gen.workload(config, stage=stage)
        net = GpuNetwork(wl, gen.workload_tensors(wl))
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            for _ in range(2):
                net.step()
            stream.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                net.step()
            graph.replay()
            stream.synchronize()
            t0 = time.perf_counter()
            for _ in range(replays):
                graph.replay()
            stream.synchronize()
            t1 = time.perf_counter()
        ms = (t1 - t0) * 1e3 / replays
        out["bf16_step_ms"][wl["name"]] = {"ms_per_step": ms, "images_per_s": wl["input"][0] / ms * 1e3, "batch": wl["input"][0]}
        del net, graph
        torch.cuda.empty_cache()
    return out


# N, C, H, K, R, stride, pad, groups: depthwise layers at the sizes of the bottleneck stages, and two 32-group layers
GROUPED_LAYERS = [
    (128, 128, 56, 128, 3, 1, 1, 128),
    (128, 128, 56, 128, 3, 2, 1, 128),
    (128, 256, 28, 256, 3, 1, 1, 256),
    (128, 512, 14, 512, 3, 1, 1, 512),
    (128, 256, 28, 256, 3, 1, 1, 32),
    (128, 128, 56, 128, 3, 1, 1, 32),
]


def grouped_table(repeats=10):
    """Grouped convolution layers at full size (see the module docstring)."""
    import torch
    from paper_2409_11600_amd import binding as B

    ws = B.Workspace()
    gen_t = torch.Generator(device="cuda").manual_seed(11)
    dt, es = torch.bfloat16, 2
    print(f"{'layer':<46}{'pass':<7}{'us':>9}{'GB/s':>8}{'%hbm':>6}{'TFLOP/s':>9}")
    rows = []
    for N, C, H, K, R, stride, pad, G in GROUPED_LAYERS:
        P = (H + 2 * pad - R) // stride + 1
        cg = C // G
        flops = 2.0 * N * P * P * K * cg * R * R
        xb, yb = N * H * H * C * es, N * P * P * K * es
        nset = max(2, int(300e6 // (xb + yb)) + 1)
        sets = []
        for _ in range(nset):
            x = torch.randn(N, H, H, C, device="cuda", generator=gen_t).to(dt)
            dy = torch.randn(N, P, P, K, device="cuda", generator=gen_t).to(dt)
            sets.append((x, dy, torch.empty_like(dy), torch.empty_like(x)))
        w = (torch.randn(K, R, R, cg, device="cuda", generator=gen_t) * (2.0 / (cg * R * R)) ** 0.5).to(dt)
        dw = torch.empty(K, R, R, cg, device="cuda")
        wbytes = K * R * R * cg
        passes = {
            "fwd": (lambda s: B.conv2d_grouped_fwd(s[0], w, G, stride, pad, 1, out=s[2], ws=ws), xb + yb + wbytes * es),
            "dgrad": (lambda s: B.conv2d_grouped_dgrad(s[1], w, (N, C, H, H), G, stride, pad, 1, out=s[3], ws=ws), xb + yb + wbytes * es),
            "wgrad": (lambda s: B.conv2d_grouped_wgrad(s[0], s[1], (K, cg, R, R), G, stride, pad, 1, out=dw, ws=ws), xb + yb + wbytes * 4),
        }
        name = f"{R}x{R} s{stride} {C}->{K} groups={G} @{H}x{H} N={N} bf16"
        for pname, (fn, byts) in passes.items():
            ms = _time_calls(torch, fn, sets, repeats)
            gbs, tf = byts / ms / 1e6, flops / ms / 1e9
            print(f"{name:<46}{pname:<7}{ms * 1e3:9.1f}{gbs:8.0f}{100 * gbs * 1e9 / PEAK['hbm']:6.1f}{tf:9.1f}", flush=True)
            rows.append({"layer": name, "pass": pname, "us": ms * 1e3, "gbytes_per_s": gbs,
                         "frac_of_hbm_peak": gbs * 1e9 / PEAK["hbm"], "tflops": tf})
        del sets
    print(json.dumps({"metric": "grouped convolution layers (fwd, dgrad, wgrad)", "unit": "us", "layers": rows}))


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
        fwd = "_fwd" in name                         # nsk_bn_relu_add_fwd[_mask] / nsk_bn_relu_add_bwd[_mask]
        res = (args[2] if fwd else args[8]) is not None
        if fwd:
            byts = (2 + res + 1) * e * es          # stats read + apply read (+ residual) + write
        else:
            byts = (6 if d.relu else 4) * e * es + (1 + res) * e * es   # two passes over x,(out),dout + writes
        return name[len("nsk_"):].replace("_mask", "").replace("_stats", ""), 0.0, byts
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


def gru_bench(a):
    """The recurrent workload of the paper's section "Experiments and Discussion" at its stated sizes (the embedding
    width is not stated: 256, the hidden size).  A step is forward, backward through time, gradient clip and AdamW
    over one batch of seeded random tokens; fp32 as in the paper.  Prints one JSON line."""
    import numpy as np
    import torch
    import nsk_inputs as gen
    from paper_2409_11600_amd.recurrent import GpuGruClassifier

    T, N, E, H, V, K = 200, 50, 256, 256, 32768, 2
    tokens = ((gen.uniform(77, 0, (T, N)) * V).astype(np.int32)) % V
    labels = ((gen.uniform(77, 1, (N,)) * K).astype(np.int32)) % K
    p = dict(table=gen.normal(77, 2, (V, E)), w_ih=gen.normal(77, 3, (3 * H, E)) / np.sqrt(E),
             w_hh=gen.normal(77, 4, (3 * H, H)) / np.sqrt(H), b_ih=np.zeros(3 * H), b_hh=np.zeros(3 * H),
             w_out=gen.normal(77, 7, (K, H)) / np.sqrt(H), b_out=np.zeros(K))
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        m = GpuGruClassifier(tokens, labels, **p, dtype="f32", lr=1e-3, weight_decay=1e-4, clip=5.0)
        for _ in range(max(a.warmup, 2)):
            m.step()
        stream.synchronize()
        graph = None
        if not a.no_graph:
            # forward and backward through time as one HIP graph (about 1000 launches); the optimizer call carries the
            # step number as a host argument and is issued after each replay
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                m.forward()
                m.backward()
        steps = min(a.steps, 20)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            if graph is not None:
                graph.replay()
                m.update()
            else:
                m.step()
        stream.synchronize()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    ms = (t1 - t0) * 1e3 / steps
    print(json.dumps({"metric": "GRU sentiment classifier training step (embedding + GRU 256 + output layer, clipped AdamW)",
                      "value": N * steps / (t1 - t0), "unit": "sequences/s", "n_gpus": 1, "steps": steps, "warmup": a.warmup,
                      "ms_per_step": ms, "higher_is_better": True, "dtype": "f32", "data": "synthetic",
                      "config": {"workload": f"tokens [{T}, {N}], vocabulary {V}, embedding {E}, hidden {H}, {K} classes",
                                 "hip_graph": graph is not None}, "loss": float(m.loss.item())}))


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
    if a.layers:
        layer_table()
        return
    if a.gru:
        gru_bench(a)
        return
    if a.grouped:
        grouped_table()
        return
    wl = gen.workload(a.config, batch=a.batch, stage=a.stage)
    tensors = gen.workload_tensors(wl)
    layout = B.NSK_NHWC if a.layout == "nhwc" else B.NSK_NCHW
    fused_act = a.fused_act and not (a.no_fusion or a.no_stats) and a.layout == "nhwc"
    net = GpuNetwork(wl, tensors, layout=layout, use_relu_mask=not a.no_fusion, use_fused_stats=not (a.no_fusion or a.no_stats),
                     use_fused_act=fused_act)
    batch = wl["input"][0]
    calls = net.fwd_calls + net.bwd_calls
    costs = [call_cost(net, f, args) for f, args in calls]
    stream = torch.cuda.Stream()
    side = torch.cuda.Stream() if a.overlap else None
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
                net.step(side_stream=side)     # backward-weight calls fork to the side stream and join at the end
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
                net.step(side_stream=side)
        stream.synchronize()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        # ---- timed region B: same steps issued call by call with events around EVERY launch of the dominant group
        # (a backward-data call also packs its filter first: that small launch is inside its bracket).
        timed_idx = dom_idx
        rec = {i: [] for i in timed_idx}
        for _ in range(a.steps):
            issue(rec)
        stream.synchronize()
    dom_all = np.array([e0.elapsed_time(e1) for i in timed_idx for e0, e1 in rec[i]], dtype=np.float64)
    dom_ms, dom_mean, dom_min = float(np.median(dom_all)), float(np.mean(dom_all)), float(np.min(dom_all))
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
    roof["launch_ms"] = dom_ms      # median over all launches of the group inside the timed steps: what `achieved` uses
    roof["launch_ms_mean"] = dom_mean
    roof["launch_ms_min"] = dom_min
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
                               f"{a.layout}, forward+backward", "batch": batch, "hip_graph": graph is not None, "fused_bn_statistics": not (a.no_fusion or a.no_stats), "relu_mask": not a.no_fusion,
                   "activations_applied_on_load": sorted(net.fused_away),
                   "streams": 1 if side is None else 2},
        "conv_tflops": conv_flops / (conv_ms * 1e-3) / 1e12,
        "conv_frac_of_mfma_peak": conv_flops / (conv_ms * 1e-3) / PEAK["mfma_bf16" if wl["dtype"] == "bf16" else "mfma_f32"],
        "roofline": roof,
    }

    if a.train_step:
        from paper_2409_11600_amd.trainer import GpuTrainer
        classes = 10 if a.config <= 3 else 1000
        Cout = gen.tensor_shapes(wl)[wl["output"]][1]
        fc_w = (gen.normal(wl["seed"], 2000, (classes, Cout)) / np.sqrt(Cout)).astype(np.float32)
        fc_b = np.zeros((classes,), np.float32)
        labels = (gen.uniform(wl["seed"], 2002, (batch,)) * classes).astype(np.int32) % classes
        with torch.cuda.stream(stream):
            tr = GpuTrainer(net, fc_w, fc_b, labels, lr=0.1, momentum=0.9, weight_decay=1e-4)
            for _ in range(2):
                tr.step()
            stream.synchronize()
            tgraph = None
            if not a.no_graph:
                tgraph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(tgraph, stream=stream):
                    tr.step()
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            for _ in range(a.steps):
                tgraph.replay() if tgraph is not None else tr.step()
            stream.synchronize()
            torch.cuda.synchronize()
            c1 = time.perf_counter()
        n_params = sum(p[0].numel() for g in tr.groups.values() for p in g)
        out["train_step"] = {"ms_per_step": (c1 - c0) * 1e3 / a.steps, "images_per_s": batch * a.steps / (c1 - c0),
                             "tail": f"avgpool + fc({Cout}->{classes}) + softmax-xent + backward + SGD-momentum over "
                                     f"{n_params} parameters", "loss": float(tr.loss.item())}

    if a.config == 2 and a.batch is None and not a.no_extras:
        out.update(bf16_target_figures())

    if not a.no_cpu_baseline:
        import oracle
        from oracle import network as onet
        # bounded sample: the oracle runs about 9 GFLOP/s on 8 cores, so cap the work at ~100 GFLOP
        total_gflop = conv_flops / 1e9
        sample_batch = batch if total_gflop <= 100 else max(1, int(batch * 100 / total_gflop))
        swl = gen.workload(a.config, batch=sample_batch, stage=a.stage)
        stens = gen.workload_tensors(swl)
        # repeat the same pass until about 10 s of CPU work have been timed (at least once)
        reps, c0 = 0, time.perf_counter()
        while True:
            f = onet.forward(swl, stens["x"], stens["params"])
            onet.backward(swl, f, stens["params"], stens["dout"])
            reps += 1
            c1 = time.perf_counter()
            if c1 - c0 >= 10.0:
                break
        out["cpu_baseline"] = {"value": reps * sample_batch / (c1 - c0), "unit": "images/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": f"{sample_batch} of {batch} images, forward+backward of the same workload, "
                                         f"{reps} time(s) ({c1 - c0:.1f} s)"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
