"""GPU parity of the backward pass: ukst_conv_transpose2d_grad_input / _grad_weight, called through
the C ABI, against the fp64 CPU oracle on the same seeded inputs.  Tolerances as for the forward
pass: fp32 max|err| <= 1e-5 * sum|products| per element, bf16 operands <= 1e-2 * sum|products|;
integer-valued inputs must match exactly."""
import numpy as np
import pytest

import oracle
from paper_2502_20493_amd import binding as ukst
from paper_2502_20493_amd import workloads as wl
from gpu_util import TOL, check_elements, run_gpu_grad_input, run_gpu_grad_weight

pytestmark = pytest.mark.gpu


def _mk(name, idx, B, Cin, Cout, H, W, n, P, dtype="f32"):
    return wl.Workload(name, idx, B, Cin, Cout, H, W, n, P, dtype, "normal", "normal:0.5")


def _both(w, integer=False, guard=4096):
    """Full-tensor parity of both gradients on workload w."""
    print(f"case {w.name} B={w.B} Cin={w.Cin} Cout={w.Cout} H={w.H} W={w.W} n={w.n} P={w.P} "
          f"{w.dtype} integer={integer}", flush=True)
    data = wl.generate(w, integer=integer)
    dyd = wl.generate_dy(w, oracle.out_shape(w.H, w.W, w.n, w.P), integer=integer)
    dx_ref, Sx = oracle.grad_input(dyd["dy"], data["w"], w.H, w.W, w.P)
    dx = run_gpu_grad_input(data, dyd, w.dtype, w.H, w.W, w.P, guard=guard)
    check_elements(dx, dx_ref, Sx, TOL[w.dtype], exact=integer)
    dw_ref, Sw = oracle.grad_weight(data["x"], dyd["dy"], w.n, w.P)
    dw = run_gpu_grad_weight(data, dyd, w.dtype, w.n, w.P, guard=guard)
    check_elements(dw, dw_ref, Sw, TOL[w.dtype], exact=integer)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6, 7])
def test_backward_edge_sweep(n):
    idx = 0
    for P in range(0, n + 2):
        for (B, Cin, Cout, H, W) in [(1, 1, 1, 4, 4), (2, 3, 3, 5, 9), (1, 9, 5, 1, 37),
                                     (1, 17, 2, 11, 1), (2, 2, 4, 33, 70), (3, 5, 3, 2, 3)]:
            if 2 * H + 2 * P - n < 1 or 2 * W + 2 * P - n < 1:
                continue
            idx += 1
            w = _mk(f"bwd_edge_n{n}", 5000 + 100 * n + idx, B, Cin, Cout, H, W, n, P)
            _both(w, integer=True)
            if P in (0, n // 2):
                _both(w, integer=False)
                _both(w.with_(dtype="bf16"), integer=False)


@pytest.mark.parametrize("shape", [
    (3, 20, 18, 37, 45, 5, 1), (2, 33, 65, 19, 70, 3, 0), (5, 16, 8, 8, 8, 4, 2),
    (2, 70, 130, 9, 33, 4, 3), (1, 64, 3, 40, 40, 4, 2), (2, 3, 40, 35, 66, 3, 2),
    (9, 12, 12, 4, 4, 4, 2), (1, 24, 20, 6, 150, 7, 3), (2, 8, 24, 70, 5, 6, 2),
    # wide layers (matrix-core input gradient): narrow maps that share the MFMA columns between
    # rows and images, split sums over the output channels, every kernel side
    (6, 40, 24, 4, 4, 4, 2), (3, 96, 32, 7, 8, 3, 1), (2, 64, 16, 16, 16, 5, 2), (5, 32, 18, 2, 3, 2, 0),
    (1, 32, 16, 9, 40, 7, 3), (2, 48, 17, 12, 20, 6, 1), (37, 130, 16, 1, 1, 1, 0), (2, 200, 40, 3, 70, 5, 4),
    # both channel counts wide (matrix-core kernel gradient): every kernel side it takes, odd widths
    (2, 40, 33, 5, 6, 2, 1), (1, 33, 40, 9, 12, 7, 3), (2, 64, 32, 4, 4, 6, 2), (1, 32, 32, 3, 7, 4, 2),
    (3, 36, 70, 1, 1, 3, 1), (2, 32, 32, 40, 45, 5, 0)])
def test_backward_several_tiles_ragged_tails(shape):
    """Several pixel tiles, channel blocks and reduction slices, with ragged tails in every axis."""
    B, Cin, Cout, H, W, n, P = shape
    w = _mk("bwd_mid", 6000 + sum(shape), B, Cin, Cout, H, W, n, P)
    _both(w, integer=True)
    _both(w, integer=False)
    _both(w.with_(dtype="bf16"), integer=False)


@pytest.mark.parametrize("shape", [
    (2, 32, 32, 4, 16, 4, 2),      # one tile, 16-pixel rows
    (1, 64, 40, 9, 24, 3, 1),      # W = 24 in a 32-wide tile: the second K step of a row is half empty
    (3, 40, 33, 5, 40, 2, 0),      # two column tiles, ragged channel blocks
    (2, 96, 64, 3, 64, 4, 3),      # P > n / 2, two input channel tiles
    (5, 32, 32, 2, 16, 3, 0),      # several images per stage
    (1, 32, 32, 20, 32, 4, 1),     # several row tiles, odd P
    (2, 32, 32, 17, 16, 2, 1),     # ragged row tile
    (4, 64, 32, 16, 16, 4, 2)])    # cfg5b's map
def test_backward_bf16_kernel_gradient_on_the_bf16_matrix_pipe(shape):
    """bf16 layers with both channel counts wide, n <= 4 and rows of 8-element pieces take the
    kernel gradient on the bf16 MFMA pipe (pixels as the K axis, half of the dy fragments read at
    2-byte-aligned LDS addresses): every element, integer-valued data exactly."""
    B, Cin, Cout, H, W, n, P = shape
    assert ukst.ukst_grad_kernel_name(1, B, Cin, Cout, H, W, n, P, ukst.UKST_BF16_F32) == \
        "ukst_grad_weight_mfma_bf16_kernel"
    w = _mk("bwd_b16pipe", 6500 + sum(shape), B, Cin, Cout, H, W, n, P, dtype="bf16")
    _both(w, integer=True)
    _both(w, integer=False)


@pytest.mark.parametrize("shape", [
    (2, 128, 16, 8, 16, 4, 2),     # 16-pixel rows: a tile is 4 images x 8 rows, two of the images absent
    (3, 160, 32, 20, 40, 4, 1),    # one 64-column tile wider than the map; dy rows of 78: the last piece moves
    (1, 136, 48, 9, 70, 4, 0),     # two column tiles, P = 0, eight input channels in the second channel tile
    (2, 96, 16, 16, 32, 4, 3),     # 32-column tiles, P > n / 2, fewer channels than a channel tile
    (2, 72, 32, 5, 17, 4, 2),      # W = 17 in a 32-column tile, rows beyond the map
    (4, 256, 32, 16, 16, 4, 2),    # cfg5b's map: two images per tile, two channel tiles
    (1, 128, 64, 24, 128, 4, 2),   # cfg5a's rows: both column tiles touch one end of the dy rows
    (2, 128, 24, 8, 16, 4, 2),     # three stages of output channels: padded with a stage of zeros
    (1, 72, 8, 5, 40, 4, 1),       # a single stage
    (2, 128, 16, 6, 20, 4, 5),     # P > n - 1: no window begins left of its row, the first dy rows meet nothing
    (2, 128, 16, 8, 16, 3, 1),     # 3 x 3 kernels in the 4 x 4 frame: 16-pixel rows
    (1, 136, 24, 9, 70, 3, 0),     # ... two column tiles, P = 0, three stages
    (3, 160, 32, 20, 40, 3, 2),    # ... P = n - 1
    (2, 128, 16, 8, 16, 2, 0),     # 2 x 2 kernels in the frame: 16-pixel rows
    (1, 136, 24, 9, 70, 2, 1)])    # ... two column tiles, P = n - 1
def test_backward_bf16_input_gradient_with_the_taps_in_the_contraction(shape):
    """bf16 layers with kernels of 2 x 2 to 4 x 4, more than 64 input channels in multiples of 8, output channels
    in multiples of 8 and maps at least 16 wide take the input gradient on the bf16 MFMA pipe with a channel's 16
    taps as the contraction (dy staged as it lies in memory, row-end pieces written at 2-byte-aligned
    LDS addresses): every element, integer-valued data exactly."""
    B, Cin, Cout, H, W, n, P = shape
    assert ukst.ukst_grad_kernel_name(0, B, Cin, Cout, H, W, n, P, ukst.UKST_BF16_F32) == \
        "ukst_grad_input_window_mfma_bf16_kernel"
    w = _mk("bwd_window", 6900 + sum(shape), B, Cin, Cout, H, W, n, P, dtype="bf16")
    _both(w, integer=True)
    _both(w, integer=False)


@pytest.mark.parametrize("shape", [
    (2, 64, 3, 8, 8, 4, 2),        # the last generator layer in small: 3 x 16 (channel, tap) rows, two channel tiles
    (3, 16, 4, 5, 9, 4, 1),        # four output channels fill both row tiles; odd P, rows that are no multiple of 4
    (2, 40, 2, 7, 37, 5, 0),       # n = 5: 2 x 25 rows; two column tiles, ragged row ends
    (1, 100, 3, 33, 6, 3, 3),      # n = 3: one row tile; several row tiles of a narrow map, two channel tiles
    (5, 24, 1, 2, 4, 2, 0),        # a single output channel, rows of exactly four pixels
    (2, 32, 4, 12, 64, 4, 2)])     # several stages per slice
def test_backward_thin_kernel_gradient_on_the_matrix_cores(shape):
    """Few output channels, at least 16 input channels, 2 <= n <= 5, rows of at least four pixels:
    (channel, tap) pairs fill the MFMA rows of the kernel gradient.  Every element, integer data
    exactly, fp32 and bf16 operands."""
    B, Cin, Cout, H, W, n, P = shape
    assert ukst.ukst_grad_kernel_name(1, B, Cin, Cout, H, W, n, P, ukst.UKST_F32) == \
        "ukst_grad_weight_thin_mfma_kernel"
    w = _mk("bwd_thin_gw", 6700 + sum(shape), B, Cin, Cout, H, W, n, P)
    _both(w, integer=True)
    _both(w, integer=False)
    _both(w.with_(dtype="bf16"), integer=False)


@pytest.mark.parametrize("shape", [
    (2, 3, 3, 19, 45, 3, 0),       # the image layer in small: windows begin two columns left of the rows
    (1, 4, 4, 9, 300, 4, 2),       # two 256-column chunks, four channels on both sides
    (2, 1, 2, 7, 33, 2, 1),        # n = 2, one input channel, odd H (a row pair with one row)
    (3, 2, 4, 5, 64, 5, 4),        # n = 5 with P = n - 1: no window begins left of its row
    (2, 3, 3, 8, 40, 3, 3),        # P > n - 1: the first dy rows and columns meet nothing
    (1, 3, 1, 33, 257, 5, 0),      # n = 5, P = 0: windows begin four columns left; one pixel in the second chunk
    (5, 4, 3, 3, 32, 4, 0),        # the narrowest map the kernels take
    (1, 3, 3, 8, 40, 3, 300)])     # padding far beyond the kernel: most of dy meets no input at all
def test_backward_narrow_layers_register_blocked_strips(shape):
    """fp32 layers with at most 4 channels on both sides, 2 <= n <= 5 and maps at least 32 wide:
    both gradients from register-blocked four-column strips with the edges left to the buffer
    addressing hardware.  Every element, integer-valued data exactly."""
    B, Cin, Cout, H, W, n, P = shape
    assert ukst.ukst_grad_kernel_name(0, B, Cin, Cout, H, W, n, P, ukst.UKST_F32) == "ukst_grad_input_narrow_kernel"
    assert ukst.ukst_grad_kernel_name(1, B, Cin, Cout, H, W, n, P, ukst.UKST_F32) == "ukst_grad_weight_narrow_kernel"
    w = _mk("bwd_narrow", 7300 + sum(shape), B, Cin, Cout, H, W, n, P)
    _both(w, integer=True)
    _both(w, integer=False)


def test_backward_cfg2_images_full_size():
    for name in ("cfg2a", "cfg2b"):
        _both(wl.WORKLOADS[name], guard=1 << 16)
        _both(wl.WORKLOADS[name].with_(B=2), integer=True)


def _sampled(w, n_planes=8, n_co=4, n_ci=4, integer=False):
    """Full-size launch; the oracle computes a seeded sample: whole (b, ci) planes of dx (those
    planes only depend on dy[b] and w[:, ci]) and whole (co, ci) kernels of dw (they only depend
    on x[:, ci] and dy[:, co]), first and last always included."""
    print(f"case {w.name} full size, sampled; integer={integer}", flush=True)
    rng = np.random.default_rng(w.index)
    data = wl.generate(w, integer=integer)
    dyd = wl.generate_dy(w, oracle.out_shape(w.H, w.W, w.n, w.P), integer=integer)
    tol = TOL[w.dtype]
    dx = run_gpu_grad_input(data, dyd, w.dtype, w.H, w.W, w.P, guard=1 << 16)
    planes = {(0, 0), (w.B - 1, w.Cin - 1)}
    while len(planes) < min(n_planes, w.B * w.Cin):
        planes.add((int(rng.integers(w.B)), int(rng.integers(w.Cin))))
    for b, ci in sorted(planes):
        ref, S = oracle.grad_input(dyd["dy"][b:b + 1], data["w"][:, ci:ci + 1], w.H, w.W, w.P)
        check_elements(dx[b:b + 1, ci:ci + 1], ref, S, tol, exact=integer)
    del dx
    dw = run_gpu_grad_weight(data, dyd, w.dtype, w.n, w.P, guard=4096)
    cos = sorted({0, w.Cout - 1} | set(rng.choice(w.Cout, size=min(n_co, w.Cout), replace=False).tolist()))
    cis = sorted({0, w.Cin - 1} | set(rng.choice(w.Cin, size=min(n_ci, w.Cin), replace=False).tolist()))
    ref, S = oracle.grad_weight(np.ascontiguousarray(data["x"][:, cis]),
                                np.ascontiguousarray(dyd["dy"][:, cos]), w.n, w.P)
    check_elements(dw[np.ix_(cos, cis)], ref, S, tol, exact=integer)


@pytest.mark.parametrize("name", ["cfg3_L1", "cfg3_L2", "cfg3_L3", "cfg3_L4"])
def test_backward_cfg3_dcgan_layers_full_size(name):
    _sampled(wl.WORKLOADS[name])
    _sampled(wl.WORKLOADS[name], integer=True)


@pytest.mark.parametrize("name", ["cfg4a", "cfg4b"])
def test_backward_cfg4_odd_output_full_size(name):
    _sampled(wl.WORKLOADS[name])
    if name == "cfg4b":
        _sampled(wl.WORKLOADS[name], n_planes=4, n_co=2, n_ci=2, integer=True)  # exact


@pytest.mark.parametrize("name", ["cfg5a", "cfg5b"])
def test_backward_cfg5_wide_bf16_full_size(name):
    _sampled(wl.WORKLOADS[name], n_planes=6, n_co=3, n_ci=3)
    if name == "cfg5b":
        _sampled(wl.WORKLOADS[name], n_planes=4, n_co=2, n_ci=2, integer=True)  # exact


def test_backward_window_kernel_walks_over_tiles_whose_rows_end_elsewhere():
    """288 tiles of the bf16 window kernel on 256 compute units: blocks take a second tile, and with
    three column tiles per row it lies in another column, so the staging buffers are cleared and
    re-aimed between the two.  Sampled planes (the last image is among the second tiles of their blocks), integer data
    exactly."""
    w = _mk("bwd_window_walk", 6990, 12, 128, 16, 64, 192, 4, 2, dtype="bf16")
    assert ukst.ukst_grad_kernel_name(0, w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, ukst.UKST_BF16_F32) == \
        "ukst_grad_input_window_mfma_bf16_kernel"
    _sampled(w, n_planes=10, n_co=2, n_ci=2, integer=True)
    _sampled(w, n_planes=6, n_co=2, n_ci=2)


def test_backward_on_a_side_stream_is_bit_reproducible():
    """Both gradients on a non-default stream, twice: identical bits (the kernel gradient adds its
    slices in a fixed order)."""
    import torch
    w = _mk("bwd_stream", 7001, 4, 24, 40, 30, 30, 4, 2)
    data = wl.generate(w)
    OH, OW = oracle.out_shape(w.H, w.W, w.n, w.P)
    dyd = wl.generate_dy(w, (OH, OW))
    x, k, dy = (torch.from_numpy(a).cuda() for a in (data["x"], data["w"], dyd["dy"]))
    st = torch.cuda.Stream()
    outs = []
    for _ in range(2):
        with torch.cuda.stream(st):
            dx = ukst.ukst_conv_transpose2d_grad_input(dy, k, w.H, w.W, w.P, stream=st)
            dw = ukst.ukst_conv_transpose2d_grad_weight(x, dy, w.n, w.P, stream=st)
        st.synchronize()
        outs.append((dx.cpu().numpy(), dw.cpu().numpy()))
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])
    dx_ref, Sx = oracle.grad_input(dyd["dy"], data["w"], w.H, w.W, w.P)
    dw_ref, Sw = oracle.grad_weight(data["x"], dyd["dy"], w.n, w.P)
    check_elements(outs[0][0], dx_ref, Sx, TOL["f32"])
    check_elements(outs[0][1], dw_ref, Sw, TOL["f32"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 3, 3, 9, 21, 3, 0), (2, 40, 36, 6, 18, 4, 2), (2, 40, 36, 6, 24, 4, 2),
                                   (2, 128, 32, 6, 24, 4, 2)])  # the last: the bf16 window kernel
def test_backward_operands_with_element_alignment_only(dtype, shape):
    """x, w, dy one element past an aligned address (narrow layer: vector-ALU kernels, wide layer:
    matrix-core kernels): the four-element vector loads of the staging code may assume nothing
    beyond element alignment."""
    import torch
    B, Cin, Cout, H, W, n, P = shape
    w = _mk("bwd_unaligned", 7100 + Cin, B, Cin, Cout, H, W, n, P, dtype=dtype)
    data = wl.generate(w)
    dyd = wl.generate_dy(w, oracle.out_shape(H, W, n, P))

    def shifted(a32, bits):  # same values, storage starting one element after an aligned address
        t = (torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16) if dtype == "bf16"
             else torch.from_numpy(a32))
        buf = torch.empty(t.numel() + 1, dtype=t.dtype, device="cuda")
        v = buf[1:].view(t.shape)
        v.copy_(t)
        assert v.data_ptr() % 16 != 0
        return v

    x = shifted(data["x"], data.get("x_bits"))
    k = shifted(data["w"], data.get("w_bits"))
    dy = shifted(dyd["dy"], dyd.get("dy_bits"))
    dx = ukst.ukst_conv_transpose2d_grad_input(dy, k, H, W, P)
    dw = ukst.ukst_conv_transpose2d_grad_weight(x, dy, n, P)
    torch.cuda.synchronize()
    ref, S = oracle.grad_input(dyd["dy"], data["w"], H, W, P)
    check_elements(dx.cpu().numpy(), ref, S, TOL[dtype])
    ref, S = oracle.grad_weight(data["x"], dyd["dy"], n, P)
    check_elements(dw.cpu().numpy(), ref, S, TOL[dtype])


def test_backward_beyond_32bit_byte_offsets():
    """dy of 4.6 GB: its last planes start past 2^32 bytes.  Integer data, exact comparison of
    sampled dx planes and of all of dw (the oracle sees one image at a time)."""
    import torch
    B, Cin, Cout, H, W, n, P = 2, 2, 3, 6900, 6900, 3, 0
    OH, OW = oracle.out_shape(H, W, n, P)
    assert B * Cout * OH * OW * 4 > 1 << 32
    print(f"case bwd_big B={B} Cin={Cin} Cout={Cout} H={H} W={W} n={n} P={P}", flush=True)
    g = torch.Generator(device="cuda").manual_seed(20493)
    x = torch.randint(-3, 4, (B, Cin, H, W), generator=g, device="cuda").float()
    k = torch.randint(-3, 4, (Cout, Cin, n, n), generator=g, device="cuda").float()
    dy = torch.randint(-3, 4, (B, Cout, OH, OW), generator=g, device="cuda").float()
    dx = ukst.ukst_conv_transpose2d_grad_input(dy, k, H, W, P)
    dw = ukst.ukst_conv_transpose2d_grad_weight(x, dy, n, P)
    torch.cuda.synchronize()
    kh = k.cpu().numpy()
    for b, ci in ((0, 0), (B - 1, Cin - 1)):
        ref, _ = oracle.grad_input(dy[b:b + 1].cpu().numpy(), kh[:, ci:ci + 1], H, W, P)
        assert np.array_equal(dx[b, ci].cpu().numpy().astype(np.float64), ref[0, 0]), (b, ci)
    ref = np.zeros((Cout, Cin, n, n))
    for b in range(B):
        ref += oracle.grad_weight(x[b:b + 1].cpu().numpy(), dy[b:b + 1].cpu().numpy(), n, P)[0]
    # the sums run over up to 2 * 6900^2 terms of magnitude <= 9 and leave the exact range of
    # fp32: compare in the tolerance of the fp32 slices, 1e-5 * sum |x * dy| per element (the
    # oracle's own scale, added up image by image)
    Sw = np.zeros((Cout, Cin, n, n))
    for b in range(B):
        Sw += oracle.grad_weight(x[b:b + 1].cpu().numpy(), dy[b:b + 1].cpu().numpy(), n, P)[1]
    assert (np.abs(dw.cpu().numpy().astype(np.float64) - ref) <= 1e-5 * Sw).all()


def test_backward_window_kernel_beyond_32bit_byte_offsets():
    """bf16 dy of 4.4 GB and dx of 17.7 GB through the window kernel: 67584 tiles, 264 per block, the
    buffer descriptors re-based for every tile.  Integer data, exact comparison of sampled dx planes
    (first and last image, channels of both ends)."""
    import torch
    B, Cin, Cout, H, W, n, P = 33, 128, 16, 1024, 1024, 4, 2
    OH, OW = oracle.out_shape(H, W, n, P)
    assert B * Cout * OH * OW * 2 > 1 << 32
    assert ukst.ukst_grad_kernel_name(0, B, Cin, Cout, H, W, n, P, ukst.UKST_BF16_F32) == \
        "ukst_grad_input_window_mfma_bf16_kernel"
    print(f"case bwd_window_big B={B} Cin={Cin} Cout={Cout} H={H} W={W} n={n} P={P}", flush=True)
    g = torch.Generator(device="cuda").manual_seed(20493)
    k = torch.randint(-3, 4, (Cout, Cin, n, n), generator=g, device="cuda", dtype=torch.int8).to(torch.bfloat16)
    dy = torch.randint(-3, 4, (B, Cout, OH, OW), generator=g, device="cuda", dtype=torch.int8).to(torch.bfloat16)
    dx = ukst.ukst_conv_transpose2d_grad_input(dy, k, H, W, P)
    torch.cuda.synchronize()
    kh = k.float().cpu().numpy()
    for b, ci in ((0, 0), (B - 1, Cin - 1), (B - 1, 5), (17, 64)):
        ref, _ = oracle.grad_input(dy[b:b + 1].float().cpu().numpy(), kh[:, ci:ci + 1], H, W, P)
        assert np.array_equal(dx[b, ci].cpu().numpy().astype(np.float64), ref[0, 0]), (b, ci)
