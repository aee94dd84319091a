#!/usr/bin/env python3
"""Benchmark of the ukst hot path on one MI355X.

One "step" is one call of ukst_conv_transpose2d on the headline workload (cfg2a: 16 images of
224x224x3, n = 3, P = 0, odd 445x445 output -- the paper's dataset shape), with inputs resident
in HBM.  Steps rotate over enough distinct (x, y) buffer sets to exceed the 256 MB last-level
cache, so every launch reads its input from, and writes its output to, HBM.

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      for the headline kernel (algorithmic bytes / average launch duration from HIP
                events on the launch stream, against the 8 TB/s HBM peak),
  cpu_baseline  the fp64 CPU oracle timed on this machine's host cores on the same workload,
  per_config    the same measurements for every other benchmark configuration (each against the
                roofline that bounds it), for the four cfg3 generator layers chained on one
                stream (cfg3_stack), and for the two gradients of the backward pass.
"""
from __future__ import annotations

import argparse
import functools
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PEAK_TFLOPS = {"mfma_bf16": 2500.0, "mfma_f32": 157.3, "alu_f32": 78.6, "alu_f32_published": 157.3}
LLC_BYTES = 256 << 20

HEADLINE = "cfg2a"
# which roofline bounds each configuration (algorithmic intensity vs. the ridge)
BOUND = {"cfg1": "hbm", "cfg2a": "hbm", "cfg2b": "hbm", "cfg3_L4": "hbm",
         "cfg3_L1": "mfma_f32", "cfg3_L2": "mfma_f32", "cfg3_L3": "mfma_f32",
         "cfg4a": "mfma_f32", "cfg4b": "mfma_f32", "cfg5a": "mfma_bf16", "cfg5b": "mfma_bf16"}


def _device_tensors(w, data):
    import numpy as np
    import torch
    if w.dtype == "bf16":
        x = torch.from_numpy(data["x_bits"].view(np.int16)).view(torch.bfloat16).cuda()
        k = torch.from_numpy(data["w_bits"].view(np.int16)).view(torch.bfloat16).cuda()
    else:
        x, k = torch.from_numpy(data["x"]).cuda(), torch.from_numpy(data["w"]).cuda()
    return x, k


def algorithmic_bytes(w, OH, OW, out_bytes=4):
    es = 2 if w.dtype == "bf16" else 4
    return (w.B * w.Cin * w.H * w.W * es + w.Cout * w.Cin * w.n * w.n * es
            + w.B * w.Cout * OH * OW * out_bytes)


def measure(w, steps, warmup, rotate_bytes=LLC_BYTES + (64 << 20), warm_seconds=0.0, fused=False,
            out_bf16=False):
    """Time `steps` launches of workload w.  Returns a dict of rates.  fused: the same launches
    through ukst_conv_transpose2d_bias_act with a bias vector and ReLU in the store.
    out_bf16 (bf16 workloads): the output is bf16 too (UKST_BF16_BF16)."""
    import torch
    from paper_2502_20493_amd import binding as ukst
    from paper_2502_20493_amd import workloads as wl

    data = wl.generate(w)
    x0, k = _device_tensors(w, data)
    OH, OW = ukst.ukst_output_shape(w.H, w.W, w.n, w.P)
    nbytes = algorithmic_bytes(w, OH, OW, 2 if out_bf16 else 4)
    nsets = max(1, min(16, -(-rotate_bytes // nbytes)))
    xs = [x0] + [x0.clone() for _ in range(nsets - 1)]
    ys = [torch.empty((w.B, w.Cout, OH, OW), dtype=torch.bfloat16 if out_bf16 else torch.float32,
                      device="cuda") for _ in range(nsets)]
    dt = (ukst.UKST_BF16_BF16 if out_bf16 else ukst.UKST_BF16_F32) if w.dtype == "bf16" else ukst.UKST_F32
    stream = torch.cuda.current_stream()

    # arguments are marshalled once (the binding's checks and pointer lookups stay outside the
    # timed loop, which then is one C call per step); the first call goes through the checking
    # binding so that a bad shape fails loudly
    sp = stream.cuda_stream
    if fused:
        bias = torch.randn(w.Cout, dtype=torch.float32, device="cuda")
        ukst.ukst_conv_transpose2d_bias_act(xs[0], k, w.P, bias=bias, act=ukst.UKST_ACT_RELU,
                                            y=ys[0], stream=stream)
        fn = ukst.lib().ukst_conv_transpose2d_bias_act
        calls = [functools.partial(fn, xs[j].data_ptr(), k.data_ptr(), bias.data_ptr(),
                                   ys[j].data_ptr(), w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, dt,
                                   ukst.UKST_ACT_RELU, ukst.UKST_PATH_AUTO, sp) for j in range(nsets)]
    else:
        ukst.ukst_conv_transpose2d(xs[0], k, w.P, y=ys[0], stream=stream)
        fn = ukst.lib().ukst_conv_transpose2d
        calls = [functools.partial(fn, xs[j].data_ptr(), k.data_ptr(), ys[j].data_ptr(), w.B, w.Cin,
                                   w.Cout, w.H, w.W, w.n, w.P, dt, sp) for j in range(nsets)]

    def step(i):
        if calls[i % nsets]() != 0:
            raise RuntimeError("ukst_conv_transpose2d failed")

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    # extra configs: keep launching until the clocks have settled (the first ~100 ms after idle
    # run at a much lower core clock, which matters for the matrix-core kernels)
    t_w = time.perf_counter()
    while warm_seconds > 0 and time.perf_counter() - t_w < warm_seconds:
        for i in range(20):
            step(i)
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for i in range(steps):
        step(i)
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = e0.elapsed_time(e1)

    exact = 2 * ukst.ukst_mac_count(w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, 0)
    nominal = 2 * ukst.ukst_mac_count(w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, 1)
    per_launch_s = ev_ms / 1e3 / steps
    bound = BOUND.get(w.name, "hbm")
    gflops = exact / per_launch_s / 1e9
    gbs = nbytes / per_launch_s / 1e9
    if bound == "hbm":
        roof = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None}
    else:
        peak = PEAK_TFLOPS[bound]
        roof = {"bound": "mfma", "achieved": round(gflops / 1e3, 2), "peak": peak,
                "unit": "TFLOP/s", "frac": round(gflops / 1e3 / peak, 4), "traffic": None}
    roof["traffic"] = None if (fused or out_bf16) else measured_traffic(w.name)
    roof["kernel"] = ukst.ukst_kernel_name(w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, dt)
    roof["us_per_launch"] = round(per_launch_s * 1e6, 2)
    roof["algorithmic_bytes"] = nbytes
    return {
        "workload": w.name + ("+bias+relu" if fused else "") + ("+bf16out" if out_bf16 else ""),
        "shape": f"B{w.B} {w.Cin}->{w.Cout} {w.H}x{w.W} n{w.n} P{w.P} {w.dtype}"
                 + (", bias and ReLU fused into the store" if fused else "")
                 + (", bf16 output" if out_bf16 else ""),
        "out": f"{OH}x{OW}", "useful_gflops": round(gflops, 1),
        "nominal_gflops": round(nominal / per_launch_s / 1e9, 1),
        "out_gpixels": round(w.B * w.Cout * OH * OW / per_launch_s / 1e9, 3),
        "gbs": round(gbs, 1), "us": round(per_launch_s * 1e6, 2),
        "wall_ms_per_step": wall_ms / steps, "buffer_sets": nsets, "roofline": roof,
        "_data": data, "_exact_flop": exact,
    }


def measure_backward(w, which, steps, warm_seconds=0.2, rotate_bytes=LLC_BYTES + (64 << 20)):
    """Time `steps` launches of one gradient of workload w (which = "grad_input" | "grad_weight").
    The kernels are vector-ALU kernels: the narrow image layers are reported against the HBM peak,
    everything else against the fp32 vector peak.  Useful flops = 2 x the exact in-range
    multiply-adds, the same count as the forward pass (every (pixel, tap, output) triple appears
    once in each of the three products)."""
    import numpy as np
    import torch
    from paper_2502_20493_amd import binding as ukst
    from paper_2502_20493_amd import workloads as wl

    data = wl.generate(w)
    OH, OW = ukst.ukst_output_shape(w.H, w.W, w.n, w.P)
    dyd = wl.generate_dy(w, (OH, OW))
    x, k = _device_tensors(w, data)
    if w.dtype == "bf16":
        dy = torch.from_numpy(dyd["dy_bits"].view(np.int16)).view(torch.bfloat16).cuda()
    else:
        dy = torch.from_numpy(dyd["dy"]).cuda()
    del data, dyd
    es = 2 if w.dtype == "bf16" else 4
    nx, nw, ny = w.B * w.Cin * w.H * w.W, w.Cout * w.Cin * w.n * w.n, w.B * w.Cout * OH * OW
    dt = ukst.UKST_BF16_F32 if w.dtype == "bf16" else ukst.UKST_F32
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    if which == "grad_input":
        nbytes = ny * es + nw * es + nx * 4
        nsets = max(1, min(8, -(-rotate_bytes // nbytes)))
        ins = [dy] + [dy.clone() for _ in range(nsets - 1)]
        outs = [torch.empty((w.B, w.Cin, w.H, w.W), dtype=torch.float32, device="cuda") for _ in range(nsets)]
        ukst.ukst_conv_transpose2d_grad_input(ins[0], k, w.H, w.W, w.P, dx=outs[0], stream=stream)
        fn = ukst.lib().ukst_conv_transpose2d_grad_input
        calls = [functools.partial(fn, ins[j].data_ptr(), k.data_ptr(), outs[j].data_ptr(), w.B, w.Cin,
                                   w.Cout, w.H, w.W, w.n, w.P, dt, sp) for j in range(nsets)]
        kernel = ukst.ukst_grad_kernel_name(0, w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, dt)
    else:
        nbytes = nx * es + ny * es + nw * 4
        nsets = max(1, min(8, -(-rotate_bytes // nbytes)))
        ins = [(x, dy)] + [(x.clone(), dy.clone()) for _ in range(nsets - 1)]
        outs = [torch.empty((w.Cout, w.Cin, w.n, w.n), dtype=torch.float32, device="cuda") for _ in range(nsets)]
        ukst.ukst_conv_transpose2d_grad_weight(x, dy, w.n, w.P, dw=outs[0], stream=stream)
        fn = ukst.lib().ukst_conv_transpose2d_grad_weight
        calls = [functools.partial(fn, ins[j][0].data_ptr(), ins[j][1].data_ptr(), outs[j].data_ptr(), w.B,
                                   w.Cin, w.Cout, w.H, w.W, w.n, w.P, dt, sp) for j in range(nsets)]
        kernel = ukst.ukst_grad_kernel_name(1, w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, dt)

    def step(i):
        if calls[i % nsets]() != 0:
            raise RuntimeError(which + " failed")

    t_w = time.perf_counter()
    step(0)
    torch.cuda.synchronize()
    while time.perf_counter() - t_w < warm_seconds:
        for i in range(4):
            step(i)
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for i in range(steps):
        step(i)
    e1.record(stream)
    torch.cuda.synchronize()
    per_launch_s = e0.elapsed_time(e1) / 1e3 / steps
    exact = 2 * ukst.ukst_mac_count(w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, 0)
    gflops, gbs = exact / per_launch_s / 1e9, nbytes / per_launch_s / 1e9
    if BOUND.get(w.name, "hbm") == "hbm":
        roof = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None}
    else:
        # fp32 vector peak and fp32 MFMA peak are the same published number on this chip; the bf16
        # input gradient multiplies on the bf16 matrix pipe
        peak = PEAK_TFLOPS["mfma_bf16" if "mfma_bf16" in kernel else "alu_f32_published"]
        roof = {"bound": "mfma" if "mfma" in kernel else "alu", "achieved": round(gflops / 1e3, 2),
                "peak": peak, "unit": "TFLOP/s", "frac": round(gflops / 1e3 / peak, 4), "traffic": None}
    roof.update(kernel=kernel, us_per_launch=round(per_launch_s * 1e6, 2), algorithmic_bytes=nbytes,
                traffic=measured_traffic(f"{w.name} {which}"))
    return {"workload": f"{w.name} {which}",
            "shape": f"B{w.B} {w.Cin}->{w.Cout} {w.H}x{w.W} n{w.n} P{w.P} {w.dtype}, backward pass",
            "out": f"{w.H}x{w.W}" if which == "grad_input" else f"{w.n}x{w.n}",
            "useful_gflops": round(gflops, 1), "gbs": round(gbs, 1), "us": round(per_launch_s * 1e6, 2),
            "buffer_sets": nsets, "roofline": roof}


def measure_stack(steps, warm_seconds=0.3, nsets=8):
    """The four generator layers of cfg3 chained on one stream: the output of layer k is the input
    of layer k+1 (Table 4 reports such a stack as one total).  One step = four launches; steps
    rotate over `nsets` complete sets of activations and weights (about 45 MB each)."""
    import torch
    from paper_2502_20493_amd import binding as ukst
    from paper_2502_20493_amd import workloads as wl

    names = ["cfg3_L1", "cfg3_L2", "cfg3_L3", "cfg3_L4"]
    layers = [wl.WORKLOADS[n] for n in names]
    for a, b in zip(layers, layers[1:]):
        oh, ow = ukst.ukst_output_shape(a.H, a.W, a.n, a.P)
        assert (a.B, a.Cout, oh, ow) == (b.B, b.Cin, b.H, b.W), "layers do not chain"
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    fn = ukst.lib().ukst_conv_transpose2d
    sets, flop, nbytes = [], 0, 0
    for j in range(nsets):
        x = torch.from_numpy(wl.generate(layers[0])["x"]).cuda()
        calls, keep = [], [x]
        for w in layers:
            k = torch.from_numpy(wl.generate(w)["w"]).cuda()
            oh, ow = ukst.ukst_output_shape(w.H, w.W, w.n, w.P)
            y = torch.empty((w.B, w.Cout, oh, ow), dtype=torch.float32, device="cuda")
            if j == 0:
                ukst.ukst_conv_transpose2d(x, k, w.P, y=y, stream=stream)  # checked call
                flop += 2 * ukst.ukst_mac_count(w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, 0)
                nbytes += algorithmic_bytes(w, oh, ow)
            calls.append(functools.partial(fn, x.data_ptr(), k.data_ptr(), y.data_ptr(), w.B, w.Cin,
                                           w.Cout, w.H, w.W, w.n, w.P, ukst.UKST_F32, sp))
            keep += [k, y]
            x = y
        sets.append((calls, keep))

    def step(i):
        for c in sets[i % nsets][0]:
            if c() != 0:
                raise RuntimeError("ukst_conv_transpose2d failed")

    t_w = time.perf_counter()
    while time.perf_counter() - t_w < warm_seconds:
        for i in range(10):
            step(i)
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for i in range(steps):
        step(i)
    e1.record(stream)
    torch.cuda.synchronize()
    per_s = e0.elapsed_time(e1) / 1e3 / steps
    tf = flop / per_s / 1e12
    return {"workload": "cfg3_stack", "shape": "B64 512->256->128->64->3, 4x4 -> 64x64, n4 P2 f32, "
            "four chained launches on one stream", "out": "64x64",
            "useful_gflops": round(flop / per_s / 1e9, 1), "us": round(per_s * 1e6, 2),
            "buffer_sets": nsets,
            "roofline": {"bound": "mfma", "achieved": round(tf, 2), "peak": PEAK_TFLOPS["mfma_f32"],
                         "unit": "TFLOP/s", "frac": round(tf / PEAK_TFLOPS["mfma_f32"], 4),
                         "traffic": None, "kernel": "ukst_mfma_f32_kernel x3 + ukst_thin_mfma_kernel",
                         "us_per_launch": round(per_s * 1e6 / 4, 2), "algorithmic_bytes": nbytes}}


def cpu_baseline(w, data, budget_s=2.0):
    """Time the CPU oracle (as it stands) on the headline workload, all host cores.

    The whole batch is one oracle call; calls are repeated until about `budget_s` seconds of
    wall-clock (times the core count in CPU work) have been spent, and the mean is reported."""
    import oracle
    from paper_2502_20493_amd import binding as ukst
    oracle.naive(data["x"][:1], data["w"], w.P)  # build / page in
    reps, t0 = 0, time.perf_counter()
    while True:
        oracle.naive(data["x"], data["w"], w.P)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or reps >= 200:
            break
    exact = 2 * ukst.ukst_mac_count(w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, 0)
    return {"value": round(exact * reps / dt / 1e9, 3), "unit": "GFLOP/s",
            "cores": oracle.threads(), "kind": "oracle", "seconds": round(dt, 3),
            "sample": f"{reps} passes over the full {w.name} batch ({w.B} images each): naive "
                      f"fp64 Algorithm 1 incl. fp32->fp64 conversion; useful (zero-free) FLOPs "
                      f"counted exactly as for the GPU"}


def copy_ceiling(nbytes, steps=200):
    """Measured ceiling shown next to the published peak: a plain device-to-device copy (torch's
    copy kernel) of buffers of the workload's size, rotated beyond the last-level cache; bytes
    read plus bytes written per second."""
    import torch
    n = max(1 << 20, nbytes // 2 // 4)
    nsets = max(2, min(16, -(-(LLC_BYTES + (64 << 20)) // (8 * n))))
    src = [torch.empty(n, dtype=torch.float32, device="cuda").normal_() for _ in range(nsets)]
    dst = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(nsets)]
    for i in range(20):
        dst[i % nsets].copy_(src[i % nsets])
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        dst[i % nsets].copy_(src[i % nsets])
    e1.record()
    torch.cuda.synchronize()
    s = e0.elapsed_time(e1) / 1e3 / steps
    return {"d2d_copy_GBps": round(8 * n / s / 1e9, 1), "d2d_copy_bytes": 8 * n,
            "d2d_copy_us": round(s * 1e6, 2)}


def mfma_ceiling(dtype_name, seconds=0.3):
    """Measured ceiling shown next to the published MFMA peak: a register-resident loop of
    independent MFMAs (no memory traffic), launched until the clocks have settled and then timed
    with events on the launch stream."""
    import torch
    from paper_2502_20493_amd import binding as ukst
    dt = ukst.UKST_BF16_F32 if dtype_name == "mfma_bf16" else ukst.UKST_F32
    iters = 20000 if dt == ukst.UKST_BF16_F32 else 10000
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    t_w = time.perf_counter()
    while time.perf_counter() - t_w < seconds:
        ukst.ukst_bench_mfma_ceiling(dt, iters, sink, stream)
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps, flop = 5, 0.0
    e0.record(stream)
    for _ in range(reps):
        flop += ukst.ukst_bench_mfma_ceiling(dt, iters, sink, stream)
    e1.record(stream)
    torch.cuda.synchronize()
    if flop <= 0:
        return None
    return {"mfma_loop_TFLOPs": round(flop / (e0.elapsed_time(e1) / 1e3) / 1e12, 1),
            "what": "register-resident loop of independent MFMAs, 8 waves per compute unit"}


def measured_traffic(kernel_workload):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE / WRITE_SIZE,
    each scaled by what the counter reads for a plain copy of known size), or None."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    try:
        with open(path) as f:
            t = json.load(f).get(kernel_workload)
        return None if t is None else int(t["fetch_bytes"] + t["write_bytes"])
    except (OSError, ValueError, KeyError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=500)
    ap.add_argument("--configs", default="all",
                    help="'all', 'none' or comma-separated extra configs for per_config")
    ap.add_argument("--only", default=None, help="time just this workload as the headline")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--grad", default=None, choices=["grad_input", "grad_weight"],
                    help="with --only: time this gradient of the workload instead of the forward "
                         "pass (used for the per-kernel counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards by batch with no "
              "exchange; no multi-GPU figure is produced). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2502_20493_amd import build as b
    from paper_2502_20493_amd import workloads as wl
    if not os.path.exists(b.LIB):
        b.build_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    head = wl.WORKLOADS[args.only or HEADLINE]
    if args.grad:
        if not args.only:
            ap.error("--grad needs --only <workload>")
        r = measure_backward(head, args.grad, args.steps, warm_seconds=0.0)
        print(json.dumps({"metric": "useful (zero-free) GFLOP/s", "value": r["useful_gflops"],
                          "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": r["us"] / 1e3, "higher_is_better": True, "scaling": "weak",
                          "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                          "config": {"workload": r["workload"] + ": " + r["shape"]},
                          "roofline": r["roofline"], "cpu_baseline": None}))
        return
    m = measure(head, args.steps, args.warmup)
    data = m.pop("_data")
    m.pop("_exact_flop")
    cpu = None if args.no_cpu else cpu_baseline(head, data)
    del data
    m["roofline"]["measured_ceiling"] = copy_ceiling(m["roofline"]["algorithmic_bytes"])

    per = []
    ceilings = {}
    if args.configs != "none" and not args.only:
        names = [n for n in wl.WORKLOADS if n not in (HEADLINE, "cfg1_int")] \
            if args.configs == "all" else args.configs.split(",")
        for name in names:
            w = wl.WORKLOADS[name]
            r = measure(w, max(5, min(args.steps, 50)), max(2, min(args.warmup, 5)), warm_seconds=0.3)
            r.pop("_data"); r.pop("_exact_flop")
            b = BOUND.get(name, "hbm")
            if b != "hbm":
                if b not in ceilings:
                    ceilings[b] = mfma_ceiling(b)
                r["roofline"]["measured_ceiling"] = ceilings[b]
            per.append(r)
            torch.cuda.empty_cache()
        if args.configs == "all":
            per.append(measure_stack(max(5, min(args.steps, 50))))
            torch.cuda.empty_cache()
            # the fused epilogue on the two ends of the range: HBM-bound images, MFMA-bound layer
            # and bf16 output for the bf16 layers, without and with the epilogue
            for name, kw in (("cfg2a", dict(fused=True)), ("cfg5a", dict(fused=True)),
                             ("cfg5a", dict(out_bf16=True)), ("cfg5b", dict(out_bf16=True)),
                             ("cfg5a", dict(out_bf16=True, fused=True))):
                r = measure(wl.WORKLOADS[name], max(5, min(args.steps, 50)), max(2, min(args.warmup, 5)),
                            warm_seconds=0.3, **kw)
                r.pop("_data"); r.pop("_exact_flop")
                if BOUND.get(name, "hbm") != "hbm":
                    r["roofline"]["measured_ceiling"] = ceilings.get(BOUND[name])
                per.append(r)
                torch.cuda.empty_cache()
            # backward pass: both gradients of every configuration
            for name in names:
                if name == "cfg1":
                    continue
                for which in ("grad_input", "grad_weight"):
                    per.append(measure_backward(wl.WORKLOADS[name], which, max(5, min(args.steps, 20))))
                    torch.cuda.empty_cache()
            for which in ("grad_input", "grad_weight"):
                per.append(measure_backward(wl.WORKLOADS[HEADLINE], which, max(5, min(args.steps, 200))))
                torch.cuda.empty_cache()

    line = {
        "metric": "useful (zero-free) GFLOP/s", "value": m["useful_gflops"], "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(m["wall_ms_per_step"], 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32" if head.dtype == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": f"{head.name}: {m['shape']} -> {m['out']}",
                   "buffer_sets_rotated": m["buffer_sets"],
                   "out_gpixels_per_s": m["out_gpixels"], "nominal_gflops": m["nominal_gflops"]},
        "roofline": m["roofline"], "cpu_baseline": cpu,
        "per_config": [{k: v for k, v in r.items() if k != "wall_ms_per_step"} for r in per],
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
