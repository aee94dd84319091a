"""GPU parity of the two generalisations Sec. 5 points to -- stride-s transpose convolution and
dilated convolution on segregated inputs -- called through the C ABI, against the fp64 CPU oracle
on the same seeded inputs.  Tolerances as for the stride-2 layer: fp32 1e-5 * sum|x*w| per
output, bf16 operands 1e-2 * sum|x*w|; integer-valued inputs must match exactly."""
import numpy as np
import pytest

import oracle
from paper_2502_20493_amd import binding as ukst
from paper_2502_20493_amd import workloads as wl
from gpu_util import TOL, check_against_oracle, to_device

pytestmark = pytest.mark.gpu


def _run(op, w, k, integer, guard=4096, sentinel=-777.0):
    import torch
    print(f"case {op} k={k} B={w.B} Cin={w.Cin} Cout={w.Cout} H={w.H} W={w.W} n={w.n} P={w.P} {w.dtype} "
          f"integer={integer}", flush=True)
    data = wl.generate(w, integer=integer)
    if op == "strided":
        y_ref, S = oracle.strided_naive(data["x"], data["w"], w.P, k)
        shape_fn, fn = ukst.ukst_output_shape_strided, ukst.ukst_conv_transpose2d_strided
    else:
        y_ref, S = oracle.dilated_naive(data["x"], data["w"], w.P, k)
        shape_fn, fn = ukst.ukst_output_shape_dilated, ukst.ukst_dilated_conv2d
    x, wt = to_device(data, w.dtype)
    OH, OW = shape_fn(w.H, w.W, w.n, w.P, k)
    assert (OH, OW) == y_ref.shape[2:]
    numel = w.B * w.Cout * OH * OW
    buf = torch.full((numel + 2 * guard,), sentinel, dtype=torch.float32, device="cuda")
    y = buf[guard:guard + numel].view(w.B, w.Cout, OH, OW)
    fn(x, wt, w.P, k, y=y)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert (host[:guard] == sentinel).all() and (host[guard + numel:] == sentinel).all()
    check_against_oracle(host[guard:guard + numel].reshape(y_ref.shape), y_ref, S, TOL[w.dtype], exact=integer)


def _mk(idx, B, Cin, Cout, H, W, n, P, dtype="f32"):
    return wl.Workload("general", idx, B, Cin, Cout, H, W, n, P, dtype, "normal", "normal:0.5")


@pytest.mark.parametrize("s", [1, 2, 3, 4, 5])
def test_strided_edge_sweep(s):
    idx = 0
    for n in (1, 2, 3, 4, 5, 7):
        for P in (0, 1, n - 1, n + 1):
            for (B, Cin, Cout, H, W) in [(1, 1, 1, 4, 4), (2, 3, 3, 5, 9), (1, 9, 5, 1, 37), (1, 17, 2, 11, 1),
                                         (2, 2, 11, 33, 40)]:
                if P < 0 or min(oracle.out_shape_strided(H, W, n, P, s)) < 1:
                    continue
                idx += 1
                w = _mk(11000 + 100 * s + idx, B, Cin, Cout, H, W, n, P)
                _run("strided", w, s, integer=True)
                if P == 1:
                    _run("strided", w, s, integer=False)
                    _run("strided", w.with_(dtype="bf16"), s, integer=False)


@pytest.mark.parametrize("d", [1, 2, 3, 4])
def test_dilated_edge_sweep(d):
    idx = 0
    for n in (1, 2, 3, 4, 5):
        for P in (0, 1, d * (n - 1) // 2, d * (n - 1) + 1):
            for (B, Cin, Cout, H, W) in [(1, 1, 1, 9, 9), (2, 3, 3, 15, 19), (1, 9, 5, 17, 37), (1, 17, 2, 21, 13),
                                         (2, 2, 11, 33, 40)]:
                if min(oracle.out_shape_dilated(H, W, n, P, d)) < 1:
                    continue
                idx += 1
                w = _mk(12000 + 100 * d + idx, B, Cin, Cout, H, W, n, P)
                _run("dilated", w, d, integer=True)
                if P == 1:
                    _run("dilated", w, d, integer=False)
                    _run("dilated", w.with_(dtype="bf16"), d, integer=False)


def test_stride2_is_the_papers_layer():
    """s = 2 through the general kernel against the oracle of record of Algorithm 1, and against
    the stride-2 kernels of the library (same tensor)."""
    import torch
    w = wl.WORKLOADS["cfg2a"].with_(B=2)
    data = wl.generate(w)
    x, wt = to_device(data, w.dtype)
    y2 = ukst.ukst_conv_transpose2d(x, wt, w.P)
    ys = ukst.ukst_conv_transpose2d_strided(x, wt, w.P, 2)
    torch.cuda.synchronize()
    y_ref, S = oracle.naive(data["x"], data["w"], w.P)
    check_against_oracle(ys.cpu().numpy(), y_ref, S, TOL["f32"])
    check_against_oracle(y2.cpu().numpy(), y_ref, S, TOL["f32"])


@pytest.mark.parametrize("case", [("strided", 3, (4, 64, 32, 32, 32, 4, 2)), ("strided", 4, (2, 16, 24, 40, 56, 5, 1)),
                                  ("dilated", 2, (4, 32, 32, 64, 64, 3, 2)), ("dilated", 4, (2, 24, 16, 70, 50, 3, 4))])
def test_generator_sized_layers_sampled(case):
    """Layers of a realistic size (several tiles, channel blocks and weight stages, ragged tails):
    every element against the oracle."""
    op, k, shape = case
    w = _mk(13000 + k, *shape)
    _run(op, w, k, integer=True)
    _run(op, w, k, integer=False)
