#!/usr/bin/env python3
"""Benchmark of the ukst hot path on one MI355X.

One "step" is one call of ukst_conv_transpose2d on the headline workload -- cfg4a, the largest
single-GPU configuration at the paper's fp32: 32 images of 64x64x128, n = 5, P = 0, odd 123x123
output with unequal parity classes and sub-kernels (9/6/6/4 taps) -- with inputs resident in HBM.
Steps rotate over enough distinct (x, y) buffer sets to exceed the 256 MB last-level cache.

Timing: after `warmup` launches and at least 0.3 s of further warm-up launches (the core clock
ramps for the first ~100 ms after idle), 5 windows of `steps` launches each are timed with HIP
events on the launch stream; the MEDIAN window is reported (the spread is in `roofline.windows_us`).

Prints ONE compact JSON line on stdout (detail rows go to stderr).  Besides the contract fields:
  roofline      for the headline kernel (useful flops / launch duration against the fp32 MFMA
                peak), with
    roofline.per_config   every benchmark configuration, forward and backward, each against the
                          roofline that bounds it: {us, frac, bound, peak, traffic_ratio}
    roofline.ceilings     what the chip sustains with nothing else going on (matrix pipes,
                          streaming kernels with each HBM-bound layer's read/write mix)
  cpu_baseline  the fp64 CPU oracle timed on this machine's host cores on a sample of complete
                (image, output channel) planes of the headline workload.
"""
from __future__ import annotations

import argparse
import functools
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PEAK_TFLOPS = {"mfma_bf16": 2500.0, "mfma_f32": 157.3}
LLC_BYTES = 256 << 20
WINDOWS = 5
MIN_WARM_SECONDS = 0.3

HEADLINE = "cfg4a"
# which roofline bounds each configuration (algorithmic intensity vs. the ridge)
BOUND = {"cfg1": "hbm", "cfg2a": "hbm", "cfg2b": "hbm", "cfg3_L4": "hbm",
         "cfg3_L1": "mfma_f32", "cfg3_L2": "mfma_f32", "cfg3_L3": "mfma_f32",
         "cfg4a": "mfma_f32", "cfg4b": "mfma_f32", "cfg5a": "mfma_bf16", "cfg5b": "mfma_bf16",
         "cfg5a_n3": "mfma_bf16", "cfg5a_n5": "mfma_bf16"}
FORWARD = ["cfg1", "cfg2a", "cfg2b", "cfg3_L1", "cfg3_L2", "cfg3_L3", "cfg3_L4", "cfg4a", "cfg4b",
           "cfg5a", "cfg5b"]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


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


def time_windows(step, steps, warmup, warm_seconds=MIN_WARM_SECONDS, windows=WINDOWS, stream=None):
    """Seconds per launch: median, min and the list over `windows` windows of `steps` launches,
    each bracketed by two HIP events recorded on the launch stream."""
    import torch
    stream = stream or torch.cuda.current_stream()
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t_w, i = time.perf_counter(), warmup
    while time.perf_counter() - t_w < warm_seconds:
        for _ in range(10):
            step(i)
            i += 1
        torch.cuda.synchronize()
    per = []
    for _ in range(windows):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            step(i)
            i += 1
        e1.record(stream)
        torch.cuda.synchronize()
        per.append(e0.elapsed_time(e1) / 1e3 / steps)
    return statistics.median(per), min(per), per


def measured_traffic(kernel_workload):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE / WRITE_SIZE,
    each scaled by what the counter reads for a plain copy of known size), or None.  Not measured
    in this run: `traffic_source` in the JSON line says so."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    try:
        with open(path) as f:
            t = json.load(f).get(kernel_workload)
        return None if t is None else int(t["fetch_bytes"] + t["write_bytes"])
    except (OSError, ValueError, KeyError):
        return None


def _roof(bound, exact_flop, nbytes, per_s, kernel, traffic):
    gflops, gbs = exact_flop / per_s / 1e9, nbytes / per_s / 1e9
    if bound == "hbm":
        r = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
             "frac": round(gbs / HBM_PEAK_GBS, 4)}
    else:
        peak = PEAK_TFLOPS[bound]
        r = {"bound": "mfma", "achieved": round(gflops / 1e3, 2), "peak": peak, "unit": "TFLOP/s",
             "frac": round(gflops / 1e3 / peak, 4)}
    r.update(traffic=traffic, kernel=kernel, us_per_launch=round(per_s * 1e6, 2),
             algorithmic_bytes=nbytes)
    return r


def measure(w, steps, warmup, rotate_bytes=LLC_BYTES + (64 << 20), fused=False, out_bf16=False,
            workspace=True, keep_data=False):
    """Time launches of workload w.  workspace=True: ukst_conv_transpose2d_ws with a workspace of
    ukst_workspace_bytes allocated once, outside the timed region (no benchmark shape asks for one
    any more: the figure is zero and the call equals the plain one);
    False: ukst_conv_transpose2d, the entry point that takes none."""
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
    shape = (w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P)
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    wants = ukst.ukst_workspace_bytes(ukst.UKST_OP_FORWARD, *shape, dt)
    need = wants if workspace else 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
    bias = torch.randn(w.Cout, dtype=torch.float32, device="cuda") if fused else None
    act = ukst.UKST_ACT_RELU if fused else ukst.UKST_ACT_NONE
    # the first call goes through the checking binding so that a bad shape fails loudly; the timed
    # loop is one C call per step with arguments marshalled once
    ukst.ukst_conv_transpose2d_bias_act(xs[0], k, w.P, bias=bias, act=act, y=ys[0], stream=stream,
                                        workspace=ws if need else False)
    if need or fused:
        fn = ukst.lib().ukst_conv_transpose2d_ws
        calls = [functools.partial(fn, xs[j].data_ptr(), k.data_ptr(),
                                   None if bias is None else bias.data_ptr(), ys[j].data_ptr(), *shape,
                                   dt, act, ukst.UKST_PATH_AUTO, ws.data_ptr() if need else None, need, sp)
                 for j in range(nsets)]
    else:
        fn = ukst.lib().ukst_conv_transpose2d
        calls = [functools.partial(fn, xs[j].data_ptr(), k.data_ptr(), ys[j].data_ptr(), *shape, dt, sp)
                 for j in range(nsets)]

    def step(i):
        if calls[i % nsets]() != 0:
            raise RuntimeError("ukst_conv_transpose2d failed")

    t0 = time.perf_counter()
    med, best, per = time_windows(step, steps, warmup, stream=stream)
    wall = time.perf_counter() - t0
    exact = 2 * ukst.ukst_mac_count(*shape, 0)
    nominal = 2 * ukst.ukst_mac_count(*shape, 1)
    base = w.name.split("+")[0]
    roof = _roof(BOUND.get(base, "hbm"), exact, nbytes, med, ukst.ukst_kernel_name(*shape, dt),
                 None if (fused or out_bf16) else measured_traffic(base))
    roof["windows_us"] = [round(p * 1e6, 2) for p in per]
    name = w.name + ("+bias+relu" if fused else "") + ("+bf16out" if out_bf16 else "") \
        + ("_nows" if wants and not workspace else "")
    return {
        "workload": name,
        "shape": f"B{w.B} {w.Cin}->{w.Cout} {w.H}x{w.W} n{w.n} P{w.P} {w.dtype}",
        "out": f"{OH}x{OW}", "useful_gflops": round(exact / med / 1e9, 1),
        "nominal_gflops": round(nominal / med / 1e9, 1),
        "out_gpixels": round(w.B * w.Cout * OH * OW / med / 1e9, 3),
        "us": round(med * 1e6, 2), "us_min": round(best * 1e6, 2), "buffer_sets": nsets,
        "workspace_bytes": need, "roofline": roof, "wall_s": wall,
        "_data": data if keep_data else None,
    }


def measure_backward(w, which, steps, rotate_bytes=LLC_BYTES + (64 << 20)):
    """Time launches of one gradient of workload w (which = "grad_input" | "grad_weight") with a
    caller-owned workspace allocated once.  Useful flops = 2 x the exact in-range multiply-adds,
    the same count as the forward pass.  Compute-bound shapes are reported against the MFMA peak
    of their operand type (bf16 operands: 2500 TFLOP/s, also where the kernel widens them and
    multiplies on the fp32 pipe), the narrow image layers against HBM."""
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
    shape = (w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P)
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    op = ukst.UKST_OP_GRAD_INPUT if which == "grad_input" else ukst.UKST_OP_GRAD_WEIGHT
    need = ukst.ukst_workspace_bytes(op, *shape, dt)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    wsp = ws.data_ptr() if need else None
    if which == "grad_input":
        nbytes = ny * es + nw * es + nx * 4
        nsets = max(1, min(8, -(-rotate_bytes // nbytes)))
        ins = [dy] + [dy.clone() for _ in range(nsets - 1)]
        outs = [torch.empty((w.B, w.Cin, w.H, w.W), dtype=torch.float32, device="cuda") for _ in range(nsets)]
        ukst.ukst_conv_transpose2d_grad_input(ins[0], k, w.H, w.W, w.P, dx=outs[0], stream=stream,
                                              workspace=ws if need else False)
        fn = ukst.lib().ukst_conv_transpose2d_grad_input
        calls = [functools.partial(fn, ins[j].data_ptr(), k.data_ptr(), outs[j].data_ptr(), *shape, dt,
                                   wsp, need, sp) for j in range(nsets)]
        kernel = ukst.ukst_grad_kernel_name(0, *shape, dt)
    else:
        nbytes = nx * es + ny * es + nw * 4
        nsets = max(1, min(8, -(-rotate_bytes // nbytes)))
        ins = [(x, dy)] + [(x.clone(), dy.clone()) for _ in range(nsets - 1)]
        outs = [torch.empty((w.Cout, w.Cin, w.n, w.n), dtype=torch.float32, device="cuda") for _ in range(nsets)]
        ukst.ukst_conv_transpose2d_grad_weight(x, dy, w.n, w.P, dw=outs[0], stream=stream,
                                               workspace=ws if need else False)
        fn = ukst.lib().ukst_conv_transpose2d_grad_weight
        calls = [functools.partial(fn, ins[j][0].data_ptr(), ins[j][1].data_ptr(), outs[j].data_ptr(),
                                   *shape, dt, wsp, need, sp) for j in range(nsets)]
        kernel = ukst.ukst_grad_kernel_name(1, *shape, dt)

    def step(i):
        if calls[i % nsets]() != 0:
            raise RuntimeError(which + " failed")

    med, best, per = time_windows(step, steps, 1, warm_seconds=0.2, windows=3, stream=stream)
    exact = 2 * ukst.ukst_mac_count(*shape, 0)
    bound = BOUND.get(w.name, "hbm")
    roof = _roof(bound, exact, nbytes, med, kernel, measured_traffic(f"{w.name} {which}"))
    if bound != "hbm" and "mfma" not in kernel:
        roof["bound"] = "alu"  # fp32 vector peak = fp32 MFMA peak on this chip (157.3 TFLOP/s)
    return {"workload": f"{w.name} {which}",
            "shape": f"B{w.B} {w.Cin}->{w.Cout} {w.H}x{w.W} n{w.n} P{w.P} {w.dtype}, backward pass",
            "useful_gflops": round(exact / med / 1e9, 1), "us": round(med * 1e6, 2),
            "us_min": round(best * 1e6, 2), "buffer_sets": nsets, "workspace_bytes": need,
            "roofline": roof}


def measure_stack(steps, nsets=8):
    """The four generator layers of cfg3 chained on one stream: the output of layer k is the input
    of layer k+1 (Table 4 reports such a stack as one total).  One step = four calls of
    ukst_conv_transpose2d_ws (workspaces allocated once); steps rotate over `nsets` complete sets
    of activations and weights (about 45 MB each)."""
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
    fn = ukst.lib().ukst_conv_transpose2d_ws
    spaces = []
    for w in layers:
        need = ukst.ukst_workspace_bytes(ukst.UKST_OP_FORWARD, w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P,
                                         ukst.UKST_F32)
        spaces.append((torch.empty(max(need, 256), dtype=torch.uint8, device="cuda"), need))
    sets, flop, nbytes = [], 0, 0
    for j in range(nsets):
        x = torch.from_numpy(wl.generate(layers[0])["x"]).cuda()
        calls, keep = [], [x]
        for w, (ws, need) in zip(layers, spaces):
            k = torch.from_numpy(wl.generate(w)["w"]).cuda()
            oh, ow = ukst.ukst_output_shape(w.H, w.W, w.n, w.P)
            y = torch.empty((w.B, w.Cout, oh, ow), dtype=torch.float32, device="cuda")
            if j == 0:
                ukst.ukst_conv_transpose2d_ws(x, k, w.P, y=y, stream=stream, workspace=ws if need else False)
                flop += 2 * ukst.ukst_mac_count(w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, 0)
                nbytes += algorithmic_bytes(w, oh, ow)
            calls.append(functools.partial(fn, x.data_ptr(), k.data_ptr(), None, y.data_ptr(), w.B, w.Cin,
                                           w.Cout, w.H, w.W, w.n, w.P, ukst.UKST_F32, ukst.UKST_ACT_NONE,
                                           ukst.UKST_PATH_AUTO, ws.data_ptr() if need else None, need, sp))
            keep += [k, y]
            x = y
        sets.append((calls, keep))

    def step(i):
        for c in sets[i % nsets][0]:
            if c() != 0:
                raise RuntimeError("ukst_conv_transpose2d_ws failed")

    med, best, per = time_windows(step, steps, 2, stream=stream)
    roof = _roof("mfma_f32", flop, nbytes, med, "ukst_mfma_f32_kernel x3 + ukst_thin_mfma_kernel", None)
    roof["windows_us"] = [round(p * 1e6, 2) for p in per]
    return {"workload": "cfg3_stack", "shape": "B64 512->256->128->64->3, 4x4 -> 64x64, n4 P2 f32, "
            "four chained launches on one stream", "useful_gflops": round(flop / med / 1e9, 1),
            "us": round(med * 1e6, 2), "us_min": round(best * 1e6, 2), "buffer_sets": nsets,
            "roofline": roof}


def measure_general(op, k, shape, steps):
    """Time one of the generalised operations of Sec. 5 (op = "strided": stride-k transpose
    convolution, "dilated": dilation-k convolution) on a synthetic fp32 layer; reported against the
    fp32 vector peak (the kernel runs on the vector ALUs)."""
    import torch
    from paper_2502_20493_amd import binding as ukst
    B, Cin, Cout, H, W, n, P = shape
    g = torch.Generator(device="cuda").manual_seed(20493)
    x = torch.randn((B, Cin, H, W), generator=g, device="cuda")
    wt = torch.randn((Cout, Cin, n, n), generator=g, device="cuda") * 0.05
    if op == "strided":
        OH, OW = ukst.ukst_output_shape_strided(H, W, n, P, k)
        fn, macs = ukst.lib().ukst_conv_transpose2d_strided, ukst.ukst_mac_count_strided(*shape, k, 0)
        ukst.ukst_conv_transpose2d_strided(x, wt, P, k)
    else:
        OH, OW = ukst.ukst_output_shape_dilated(H, W, n, P, k)
        fn, macs = ukst.lib().ukst_dilated_conv2d, ukst.ukst_mac_count_dilated(*shape, k, 0)
        ukst.ukst_dilated_conv2d(x, wt, P, k)
    nbytes = 4 * (x.numel() + wt.numel() + B * Cout * OH * OW)
    nsets = max(1, min(8, -(-(LLC_BYTES + (64 << 20)) // nbytes)))
    xs = [x] + [x.clone() for _ in range(nsets - 1)]
    ys = [torch.empty((B, Cout, OH, OW), dtype=torch.float32, device="cuda") for _ in range(nsets)]
    stream = torch.cuda.current_stream()
    calls = [functools.partial(fn, xs[j].data_ptr(), wt.data_ptr(), ys[j].data_ptr(), *shape, k,
                               ukst.UKST_F32, stream.cuda_stream) for j in range(nsets)]

    def step(i):
        if calls[i % nsets]() != 0:
            raise RuntimeError(op + " failed")

    med, best, per = time_windows(step, steps, 2, warm_seconds=0.2, windows=3, stream=stream)
    roof = _roof("mfma_f32", 2 * macs, nbytes, med, "ukst_general_kernel", None)
    roof["bound"] = "alu"  # fp32 vector peak: the same published 157.3 TFLOP/s
    return {"workload": f"{op}{k}", "shape": f"B{B} {Cin}->{Cout} {H}x{W} n{n} P{P} f32, "
            + (f"stride {k} transpose convolution" if op == "strided" else f"dilation {k} convolution"),
            "out": f"{OH}x{OW}", "useful_gflops": round(2 * macs / med / 1e9, 1), "us": round(med * 1e6, 2),
            "us_min": round(best * 1e6, 2), "buffer_sets": nsets, "roofline": roof}


def cpu_baseline(w, data, budget_s=1.5, chunk=32):
    """Time the CPU oracle (as it stands) on complete (image, output channel) planes of the
    headline workload, all host cores: chunks of `chunk` seeded planes until about `budget_s`
    seconds of wall-clock have passed (times the core count in CPU seconds)."""
    import numpy as np
    import oracle
    from paper_2502_20493_amd import binding as ukst
    total = w.B * w.Cout
    rng = np.random.default_rng(w.index)
    order = rng.permutation(total)
    oracle.naive(data["x"], data["w"], w.P, planes=[0])  # build / page in
    done, t0 = 0, time.perf_counter()
    while done < total:
        planes = sorted(order[done:done + chunk].tolist())
        oracle.naive(data["x"], data["w"], w.P, planes=planes)
        done += len(planes)
        dt = time.perf_counter() - t0
        if dt >= budget_s:
            break
    exact = 2 * ukst.ukst_mac_count(w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, 0)
    return {"value": round(exact * done / total / dt / 1e9, 3), "unit": "GFLOP/s",
            "cores": oracle.threads(), "kind": "oracle", "seconds": round(dt, 3),
            "sample": f"{done} of the {total} complete (image, output channel) planes of {w.name} "
                      f"(each sums over all {w.Cin} input channels): naive fp64 Algorithm 1 incl. "
                      f"the fp64 conversion of the inputs; useful (zero-free) FLOPs counted "
                      f"exactly as for the GPU"}


def stream_ceiling(read_bytes, write_bytes, steps=100):
    """Measured ceiling for an HBM-bound layer: a streaming kernel with no arithmetic that reads
    `read_bytes` and writes `write_bytes` (the layer's input and output sizes), buffers rotated
    beyond the last-level cache.  Returns GB/s of bytes read plus bytes written."""
    import torch
    from paper_2502_20493_amd import binding as ukst
    rb, wb = (read_bytes + 15) // 16 * 16, (write_bytes + 15) // 16 * 16
    nsets = max(2, min(16, -(-(LLC_BYTES + (64 << 20)) // (rb + wb))))
    src = [torch.empty(rb, dtype=torch.uint8, device="cuda").random_() for _ in range(nsets)]
    dst = [torch.empty(wb, dtype=torch.uint8, device="cuda") for _ in range(nsets)]

    def step(i):
        ukst.ukst_bench_stream_ceiling(src[i % nsets], dst[i % nsets])

    med, best, _ = time_windows(step, steps, 10, warm_seconds=0.1, windows=3)
    return {"GBps": round((rb + wb) / med / 1e9, 1), "us": round(med * 1e6, 2),
            "read_bytes": rb, "write_bytes": wb}


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
    return round(flop / (e0.elapsed_time(e1) / 1e3) / 1e12, 1) if flop > 0 else None


def compact(r):
    """One per_config entry of the JSON line."""
    ro = r["roofline"]
    out = {"us": r["us"], "frac": ro["frac"],
           "bound": "hbm" if ro["bound"] == "hbm" else ("bf16" if ro["peak"] == 2500.0 else "f32"),
           "peak": ro["peak"]}
    if ro.get("traffic"):
        out["traffic_ratio"] = round(ro["traffic"] / ro["algorithmic_bytes"], 3)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--configs", default="all",
                    help="'all', 'none' or comma-separated extra configs for roofline.per_config")
    ap.add_argument("--only", default=None, help="time just this workload as the headline")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-ws", action="store_true",
                    help="with --only: the entry point without a workspace (cfg3 L1, L2 differ)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="one device-to-device copy of 48 MiB before the timed work: the known-size "
                         "copy kernel that scales the profiler's FETCH_SIZE / WRITE_SIZE counters")
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
    if not (os.path.exists(b.LIB) and os.path.exists(b.BENCH_LIB)):
        b.build_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    if args.calibrate_copy:
        src = torch.empty(12582912, dtype=torch.float32, device="cuda").normal_()
        torch.empty_like(src).copy_(src)
        torch.cuda.synchronize()
    head = wl.WORKLOADS[args.only or HEADLINE]
    if args.grad:
        if not args.only:
            ap.error("--grad needs --only <workload>")
        r = measure_backward(head, args.grad, args.steps)
        print(json.dumps({"metric": "useful (zero-free) GFLOP/s", "value": r["useful_gflops"],
                          "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": r["us"] / 1e3, "higher_is_better": True, "scaling": "weak",
                          "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                          "config": {"workload": r["workload"] + ": " + r["shape"]},
                          "roofline": r["roofline"], "cpu_baseline": None}))
        return
    # a memory-bound headline (--only cfg2a ...) gets many more launches per window
    steps = args.steps if BOUND.get(head.name, "hbm") != "hbm" else max(args.steps, 500)
    m = measure(head, steps, args.warmup, keep_data=True, workspace=not args.no_ws)
    data = m.pop("_data")
    cpu = None if args.no_cpu else cpu_baseline(head, data)
    del data
    roof = m["roofline"]
    roof["traffic_source"] = "profiles/pmc_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of " \
                             "this kernel and workload, scaled by a copy of known size; not measured in this run)"

    per = {head.name: compact(m)}
    ceilings = {}
    if args.configs != "none" and not args.only:
        names = [n for n in FORWARD if n != head.name] if args.configs == "all" else args.configs.split(",")
        rows = []
        for name in names:
            w = wl.WORKLOADS[name]
            hbm = BOUND.get(name, "hbm") == "hbm"
            r = measure(w, 200 if hbm else max(5, min(args.steps, 50)), max(2, min(args.warmup, 5)))
            rows.append(r)
            if r["workspace_bytes"]:  # the same layer through the entry point without a workspace
                rows.append(measure(w, max(5, min(args.steps, 50)), 2, workspace=False))
            torch.cuda.empty_cache()
        if args.configs == "all":
            rows.append(measure_stack(max(5, min(args.steps, 50))))
            torch.cuda.empty_cache()
            # the fused epilogue on the two ends of the range (HBM-bound images, MFMA-bound layer),
            # bf16 output for the bf16 layers, and bf16 layers with the other kernel sides of
            # Tables 2-3
            extra = [("cfg2a", {}, dict(fused=True)), ("cfg5a", {}, dict(fused=True)),
                     ("cfg5a", {}, dict(out_bf16=True)), ("cfg5b", {}, dict(out_bf16=True)),
                     ("cfg5a", {}, dict(out_bf16=True, fused=True)),
                     ("cfg5a", dict(name="cfg5a_n3", n=3, P=1), {}),
                     ("cfg5a", dict(name="cfg5a_n5", n=5, P=2), {})]
            for name, over, kw in extra:
                w = wl.WORKLOADS[name].with_(**over)
                hbm = BOUND.get(w.name, "hbm") == "hbm"
                rows.append(measure(w, 200 if hbm else max(5, min(args.steps, 50)), 2, **kw))
                torch.cuda.empty_cache()
            # the generalised operations (general stride, dilation): generator-sized fp32 layers
            rows.append(measure_general("strided", 3, (16, 128, 64, 32, 32, 5, 2), max(5, min(args.steps, 20))))
            rows.append(measure_general("dilated", 2, (16, 64, 64, 64, 64, 3, 2), max(5, min(args.steps, 20))))
            torch.cuda.empty_cache()
            # backward pass: both gradients of every configuration
            for name in FORWARD[1:]:
                for which in ("grad_input", "grad_weight"):
                    hbm = BOUND.get(name, "hbm") == "hbm"
                    rows.append(measure_backward(wl.WORKLOADS[name], which,
                                                 100 if hbm else max(5, min(args.steps, 20))))
                    torch.cuda.empty_cache()
            # measured ceilings: matrix pipes, and a streaming kernel with each HBM-bound layer's
            # read / write mix
            ceilings["mfma_bf16_TFLOPs"] = mfma_ceiling("mfma_bf16")
            ceilings["mfma_f32_TFLOPs"] = mfma_ceiling("mfma_f32")
            for name in ("cfg2a", "cfg2b", "cfg3_L4"):
                w = wl.WORKLOADS[name]
                oh, ow = 2 * w.H + 2 * w.P - w.n, 2 * w.W + 2 * w.P - w.n
                rd = 4 * (w.B * w.Cin * w.H * w.W + w.Cout * w.Cin * w.n * w.n)
                ceilings["stream_" + name] = stream_ceiling(rd, 4 * w.B * w.Cout * oh * ow)
        for r in rows:
            r.pop("_data", None)
            per[r["workload"]] = compact(r)
            log(json.dumps(r))
    m.pop("wall_s")
    roof["per_config"] = per
    if ceilings:
        roof["ceilings"] = ceilings

    line = {
        "metric": "useful (zero-free) GFLOP/s", "value": m["useful_gflops"], "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(m["us"] / 1e3, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32" if head.dtype == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": f"{m['workload']}: {m['shape']} -> {m['out']}",
                   "timing": f"median of {WINDOWS} windows of {steps} launches after >= "
                             f"{MIN_WARM_SECONDS} s of warm-up launches",
                   "buffer_sets_rotated": m["buffer_sets"], "out_gpixels_per_s": m["out_gpixels"],
                   "nominal_gflops": m["nominal_gflops"]},
        "roofline": roof, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
