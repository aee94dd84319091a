"""The entry point that allocates nothing: ukst_conv_transpose2d_grad_weight_static keeps its
partial sums in a static device array of the library.  Checked through the C ABI against
ukst_conv_transpose2d_grad_weight (same kernels, caller-owned workspace) on two calls in a row,
the second with a smaller input, so that whatever the first call left in the array is still there."""
import numpy as np
import pytest

import oracle
from paper_2502_20493_amd import binding as ukst
from paper_2502_20493_amd import workloads as wl
from gpu_util import TOL, check_elements


def test_static_size_and_rejection_need_no_gpu():
    assert ukst.ukst_static_workspace_bytes() == 64 << 20
    X = W = Y = 0x1000
    f = ukst.lib().ukst_conv_transpose2d_grad_weight_static
    # a problem whose partial sums exceed the array is refused on the host, nothing is launched
    big = (64, 2048, 1024, 16, 16, 4, 2)
    assert ukst.ukst_workspace_bytes(ukst.UKST_OP_GRAD_WEIGHT, *big, ukst.UKST_F32) > 64 << 20
    assert f(X, W, Y, *big, ukst.UKST_F32, None) == ukst.UKST_ERR_WORKSPACE
    assert f(None, W, Y, 1, 1, 1, 4, 4, 3, 0, 0, None) == ukst.UKST_ERR_NULL
    assert f(X, W, Y, 1, 1, 1, 4, 1, 3, 0, 0, None) == ukst.UKST_ERR_SHAPE
    # every benchmark configuration fits
    for w in wl.WORKLOADS.values():
        dt = ukst.UKST_BF16_F32 if w.dtype == "bf16" else ukst.UKST_F32
        assert ukst.ukst_workspace_bytes(ukst.UKST_OP_GRAD_WEIGHT, w.B, w.Cin, w.Cout, w.H, w.W, w.n,
                                         w.P, dt) <= 64 << 20, w.name


@pytest.mark.gpu
def test_static_scratch_matches_the_workspace_entry_point():
    import torch
    shapes = [  # first the larger problem (many slices, wide layer: matrix-core kernel), then smaller ones
        wl.Workload("na_big", 9901, 6, 64, 96, 40, 44, 4, 2, "f32", "normal", "normal:0.5"),
        wl.Workload("na_small", 9902, 2, 32, 32, 9, 12, 3, 0, "f32", "normal", "normal:0.5"),
        wl.Workload("na_narrow", 9903, 3, 3, 3, 30, 31, 3, 0, "f32", "normal", "normal:0.5"),
        wl.Workload("na_bf16", 9904, 2, 48, 40, 8, 8, 4, 2, "bf16", "normal", "normal:0.5"),
    ]
    for w in shapes:
        print(f"case {w.name} B={w.B} Cin={w.Cin} Cout={w.Cout} H={w.H} W={w.W} n={w.n} P={w.P} {w.dtype}",
              flush=True)
        data = wl.generate(w)
        OH, OW = oracle.out_shape(w.H, w.W, w.n, w.P)
        dyd = wl.generate_dy(w, (OH, OW))
        if w.dtype == "bf16":
            x = torch.from_numpy(data["x_bits"].view(np.int16)).view(torch.bfloat16).cuda()
            dy = torch.from_numpy(dyd["dy_bits"].view(np.int16)).view(torch.bfloat16).cuda()
        else:
            x, dy = torch.from_numpy(data["x"]).cuda(), torch.from_numpy(dyd["dy"]).cuda()
        want = ukst.ukst_conv_transpose2d_grad_weight(x, dy, w.n, w.P)
        got = torch.full((w.Cout, w.Cin, w.n, w.n), -777.0, dtype=torch.float32, device="cuda")
        ukst.ukst_conv_transpose2d_grad_weight_static(x, dy, w.n, w.P, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), w.name
        ref, S = oracle.grad_weight(data["x"], dyd["dy"], w.n, w.P)
        check_elements(got.cpu().numpy(), ref, S, TOL[w.dtype])
