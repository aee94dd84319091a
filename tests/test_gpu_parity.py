"""GPU parity: the HIP library, called through the C ABI, against the fp64 CPU oracle on the same
seeded inputs.  Tolerances: fp32 max|err| <= 1e-5 * sum|x*w| per output, bf16-in/fp32-accumulate
<= 1e-2 * sum|x*w|; integer-valued inputs must match exactly."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2502_20493_amd import binding as ukst
from paper_2502_20493_amd import workloads as wl
from gpu_util import TOL, check_against_oracle, run_gpu

pytestmark = pytest.mark.gpu

PATHS = {"direct": ukst.UKST_PATH_DIRECT, "mfma": ukst.UKST_PATH_MFMA, "auto": ukst.UKST_PATH_AUTO}


def _mk(name, idx, B, Cin, Cout, H, W, n, P, dtype="f32"):
    return wl.Workload(name, idx, B, Cin, Cout, H, W, n, P, dtype, "normal", "normal:0.5")


def _supported(w, path):
    if path != ukst.UKST_PATH_MFMA:
        return True
    dt = ukst.UKST_F32 if w.dtype == "f32" else ukst.UKST_BF16_F32
    return bool(ukst.ukst_kernel_name(w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, dt, path))


def _parity(w, path, integer=False, guard=4096, planes=None, workspace=False):
    print(f"case {w.name} B={w.B} Cin={w.Cin} Cout={w.Cout} H={w.H} W={w.W} n={w.n} P={w.P} "
          f"{w.dtype} path={path} integer={integer} workspace={workspace}", flush=True)
    data = wl.generate(w, integer=integer)
    y_ref, S = oracle.naive(data["x"], data["w"], w.P, planes=planes)
    y = run_gpu(data, w.dtype, w.P, path=path, guard=guard, workspace=workspace)
    assert y.shape == y_ref.shape
    return check_against_oracle(y, y_ref, S, TOL[w.dtype], planes=planes, exact=integer)


# ------------------------------------------------------------------ edge sweep, direct path
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6, 7])
def test_direct_edge_sweep(n):
    idx = 0
    for P in range(0, n + 2):
        for (B, Cin, Cout, H, W) in [(1, 1, 1, 4, 4), (2, 3, 3, 5, 9), (1, 9, 5, 1, 37),
                                     (1, 17, 2, 11, 1), (2, 2, 4, 33, 70), (1, 4, 3, 6, 131),
                                     (2, 7, 3, 6, 19), (1, 6, 1, 3, 131)]:
            if 2 * H + 2 * P - n < 1 or 2 * W + 2 * P - n < 1:
                continue
            idx += 1
            w = _mk(f"edge_n{n}", 1000 * n + idx, B, Cin, Cout, H, W, n, P)
            _parity(w, PATHS["direct"], integer=True)
            if P in (0, n // 2):
                _parity(w, PATHS["direct"], integer=False)
                _parity(w.with_(dtype="bf16"), PATHS["direct"], integer=False)


# ------------------------------------------------------------------ the benchmark configs
def test_cfg1_toy_case():
    _parity(wl.WORKLOADS["cfg1"], PATHS["auto"])
    _parity(wl.WORKLOADS["cfg1_int"], PATHS["auto"], integer=True)
    _parity(wl.WORKLOADS["cfg1"], PATHS["auto"], integer=True)


@pytest.mark.parametrize("name", ["cfg2a", "cfg2b"])
def test_cfg2_images_full_size(name):
    w = wl.WORKLOADS[name]
    _parity(w, PATHS["auto"], guard=1 << 16)
    _parity(w.with_(B=2), PATHS["auto"], integer=True)


def _sample_planes(w, k=16):
    rng = np.random.default_rng(w.index)
    total = w.B * w.Cout
    extra = rng.choice(total, size=min(k, total) - 2, replace=False).tolist() if total > 2 else []
    return sorted(set([0, total - 1] + extra))


@pytest.mark.parametrize("name", ["cfg3_L1", "cfg3_L2", "cfg3_L3", "cfg3_L4"])
def test_cfg3_dcgan_layers_full_size(name):
    # through the entry point that takes no workspace and through ukst_conv_transpose2d_ws (the
    # tiny layers L1, L2 share the K loop of a 32 x 32 tile among the waves of a block: no
    # workspace either way)
    w = wl.WORKLOADS[name]
    planes = _sample_planes(w, 64)
    dt = ukst.UKST_F32
    need = ukst.ukst_workspace_bytes(ukst.UKST_OP_FORWARD, w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, dt)
    assert need == 0
    for workspace in (False, None):
        _parity(w, PATHS["auto"], planes=planes, workspace=workspace)
        _parity(w, PATHS["auto"], planes=planes, integer=True, workspace=workspace)


def test_cfg3_generator_stack_chained():
    # the four generator layers back to back on one stream, each fed the previous layer's fp32
    # output (Table 4 reports such a stack as one total): every layer is checked against the
    # oracle applied to the very input the GPU consumed, so the per-layer tolerance holds
    import torch
    layers = [wl.WORKLOADS[n] for n in ("cfg3_L1", "cfg3_L2", "cfg3_L3", "cfg3_L4")]
    x = torch.from_numpy(wl.generate(layers[0])["x"]).cuda()
    ks = [torch.from_numpy(wl.generate(w)["w"]).cuda() for w in layers]
    outs = []
    spaces = [torch.empty(ukst.ukst_workspace_bytes(ukst.UKST_OP_FORWARD, w.B, w.Cin, w.Cout, w.H, w.W,
                                                    w.n, w.P, ukst.UKST_F32), dtype=torch.uint8,
                          device="cuda") for w in layers]
    for w, k, ws in zip(layers, ks, spaces):  # all four enqueued before anything is read back
        assert tuple(x.shape) == (w.B, w.Cin, w.H, w.W)
        x = ukst.ukst_conv_transpose2d_ws(x, k, w.P, workspace=ws)
        outs.append(x)
    torch.cuda.synchronize()
    xin = wl.generate(layers[0])["x"]
    for w, k, y in zip(layers, ks, outs):
        print(f"stack layer {w.name}", flush=True)
        planes = _sample_planes(w, 24)
        y_ref, S = oracle.naive(xin, k.cpu().numpy(), w.P, planes=planes)
        check_against_oracle(y.cpu().numpy(), y_ref, S, TOL["f32"], planes=planes)
        xin = y.cpu().numpy()


def _stratified_planes(w, block=64):
    """One seeded (b, co) plane per (image, block of 64 output channels), plus the first and the
    last plane: every (image, channel block) tile group of the matrix-core kernels meets the
    oracle, whatever the tile walk."""
    rng = np.random.default_rng(w.index + 77)
    planes = {0, w.B * w.Cout - 1}
    for b in range(w.B):
        for c0 in range(0, w.Cout, block):
            planes.add(b * w.Cout + c0 + int(rng.integers(min(block, w.Cout - c0))))
    return sorted(planes)


@pytest.mark.parametrize("name", ["cfg4a", "cfg4b", "cfg5a", "cfg5b"])
def test_cfg45_full_size_sampled_planes(name):
    # the naive oracle is too slow for every plane at these sizes: it computes complete (b, co)
    # planes, one per (image, 64-channel block) -- 64 to 512 planes; each still reduces over all
    # Cin and holds every parity class and edge
    w = wl.WORKLOADS[name]
    planes = _stratified_planes(w)
    assert len(planes) >= w.B * ((w.Cout + 63) // 64)
    _parity(w, PATHS["auto"], planes=planes, guard=1 << 16)
    _parity(w, PATHS["auto"], planes=_sample_planes(w, 16), integer=True)


def test_cfg5a_shape_with_kernel_side_3_full_size_sampled_planes():
    """The benchmark row cfg5a_n3 (cfg5a's shape with n = 3, P = 1) in the launch configuration
    bench.py times: one plane per (image, 64-channel block) against the oracle, integer data
    exactly, and three launches bit-identical."""
    import torch
    from gpu_util import to_device
    w = wl.WORKLOADS["cfg5a"].with_(n=3, P=1)
    assert ukst.ukst_kernel_name(w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, ukst.UKST_BF16_F32) == \
        "ukst_mfma_bf16_kernel"
    _parity(w, PATHS["auto"], planes=_stratified_planes(w), guard=1 << 16)
    _parity(w, PATHS["auto"], planes=_sample_planes(w, 16), integer=True)
    x, wt = to_device(wl.generate(w), w.dtype)
    ys = [ukst.ukst_conv_transpose2d_ws(x, wt, w.P) for _ in range(3)]
    torch.cuda.synchronize()
    assert torch.equal(ys[0], ys[1]) and torch.equal(ys[0], ys[2])


@pytest.mark.parametrize("name", ["cfg3_L2", "cfg4a", "cfg4b", "cfg5b"])
def test_reduced_configs_every_element_both_paths(name):
    # same layer shapes with fewer images / channels so that the oracle covers every element
    w = wl.WORKLOADS[name]
    small = w.with_(B=2, Cin=min(w.Cin, 48), Cout=min(w.Cout, 40), H=min(w.H, 23), W=min(w.W, 31))
    for pname in ("direct", "mfma"):
        if _supported(small, PATHS[pname]):
            _parity(small, PATHS[pname])
            _parity(small, PATHS[pname], integer=True)


MFMA_BF16_SHAPES = [
    # B, Cin, Cout, H, W, P        (n = 4; Cin % 16 == 0, Cout % 8 == 0, W % 8 == 0)
    (1, 16, 64, 4, 8, 2),      # one partial tile
    (3, 32, 64, 5, 8, 2),      # tiles span images, ragged last tile
    (2, 48, 128, 9, 16, 2),    # two channel blocks, several K stages
    (2, 16, 64, 7, 24, 0),     # P = 0: output 2H-4, no halo on the left
    (2, 16, 64, 6, 16, 1),     # odd P: class order flips (Sec. 3.4)
    (1, 32, 64, 3, 40, 3),     # odd P > 1
    (5, 16, 64, 2, 8, 2),      # many tiny images inside one tile
    (1, 16, 64, 33, 64, 2),    # several row tiles of one image
    (1, 16, 64, 1, 8, 2),      # single input row
    # odd P stays with the shifted quads (even P goes to the output-aligned kernel)
    (2, 48, 128, 9, 16, 1),    # two channel blocks, several K stages
    (3, 32, 64, 5, 8, 1),      # tiles span images, ragged last tile
    (5, 16, 64, 2, 8, 3),      # many tiny images inside one tile
    (1, 16, 64, 33, 64, 1),    # several row tiles of one image
    (1, 16, 64, 20, 128, 5),   # cfg5a's row length, P > n - 1
    # more even P
    (2, 48, 128, 9, 16, 2),    # tiles span images
    (3, 16, 64, 7, 24, 0),     # P = 0: no halo, window rows up to H - 1
    (1, 32, 64, 6, 16, 6),     # P > n - 1: border quads meet no input
    (2, 16, 64, 5, 40, 0),
    (1, 16, 64, 3, 8, 18),     # padding far beyond the kernel
    (2, 32, 64, 16, 16, 2),    # cfg5b's map: one image per tile
    (1, 16, 64, 20, 128, 2),   # cfg5a's row length: two quad rows per tile
    (2, 16, 64, 9, 136, 2),    # wide rows: three quad rows and an image boundary in one tile
    # channel counts that are no multiple of 64: the last channel block is partial
    (2, 32, 96, 9, 16, 2),     # one and a half blocks
    (1, 16, 40, 5, 8, 1),      # odd P (shifted quads), 40 channels: 5 groups of 8
    (2, 16, 8, 6, 16, 2),      # a single group of 8
    (3, 32, 72, 4, 8, 0),      # P = 0, one block and one group
]


@pytest.mark.parametrize("shape", MFMA_BF16_SHAPES)
def test_mfma_bf16_small_shapes_every_element(shape):
    B, Cin, Cout, H, W, P = shape
    w = _mk("mfma_bf16", 7000 + sum(shape), B, Cin, Cout, H, W, 4, P, dtype="bf16")
    assert _supported(w, PATHS["mfma"]), "shape should be runnable by the MFMA path"
    _parity(w, PATHS["mfma"], integer=True)
    _parity(w, PATHS["mfma"], integer=False)
    # the direct path must agree with the oracle on the same data too
    _parity(w, PATHS["direct"], integer=False)


MFMA_BF16_N3_SHAPES = [
    # B, Cin, Cout, H, W, P        (n = 3: 4 / 2 / 2 / 1 taps per class, 18-byte weight rows)
    (1, 16, 64, 4, 8, 0),      # one partial tile, odd output 5 x 13
    (3, 32, 64, 5, 8, 1),      # P = 1: even output, tiles span images
    (2, 48, 128, 9, 16, 0),    # two channel blocks, several K stages (three: an odd count)
    (2, 16, 64, 7, 24, 2),     # P = 2
    (1, 32, 64, 3, 40, 3),     # P > n - 1: the outer ring meets no input
    (5, 16, 64, 2, 8, 1),      # many tiny images inside one tile
    (1, 16, 64, 33, 64, 0),    # several row tiles of one image
    (1, 16, 64, 20, 128, 1),   # cfg5a's row length
    (2, 64, 64, 16, 16, 1),    # cfg5b's map
    (2, 32, 72, 7, 16, 0),     # 72 channels: a partial second channel block
    (1, 16, 24, 5, 8, 1),      # less than half a block
]


@pytest.mark.parametrize("shape", MFMA_BF16_N3_SHAPES)
def test_mfma_bf16_kernel_side_3_every_element(shape):
    """n = 3 on the bf16 matrix pipe: the classes have unequal sub-kernels (Sec. 3.2), so a K step
    has 9 MFMA groups instead of 16; the weight rows are 18 bytes and are fetched with 16-byte
    loads at 2-byte alignment."""
    B, Cin, Cout, H, W, P = shape
    w = _mk("mfma_bf16_n3", 7300 + sum(shape), B, Cin, Cout, H, W, 3, P, dtype="bf16")
    assert ukst.ukst_kernel_name(B, Cin, Cout, H, W, 3, P, ukst.UKST_BF16_F32, PATHS["mfma"]) == \
        "ukst_mfma_bf16_kernel"
    _parity(w, PATHS["mfma"], integer=True)
    _parity(w, PATHS["mfma"], integer=False)


MFMA_F32_SHAPES = [
    # B, Cin, Cout, H, W, n, P   (Cout % 8 == 0, Cin % 8 == 0 for n = 4, 5 and % 16 for n = 2, 3; any W)
    (1, 8, 64, 4, 8, 4, 2),
    (3, 16, 64, 5, 7, 3, 0),      # odd W, tiles span images
    (2, 24, 40, 9, 13, 5, 0),     # ragged channel block (Cout = 40), n = 5: 9/6/6/4 taps
    (2, 8, 96, 7, 21, 5, 2),
    (2, 16, 64, 6, 16, 4, 1),     # odd P: class order flips (Sec. 3.4)
    (1, 16, 72, 3, 37, 3, 3),      # P > n-1: outer ring meets no input
    (5, 16, 64, 2, 5, 2, 0),       # n = 2, tiny images
    (1, 16, 128, 33, 31, 3, 0),   # several row tiles of one image, two channel blocks
    (1, 8, 64, 1, 9, 4, 2),       # single input row
    (2, 32, 64, 63, 63, 3, 0),    # cfg4b spatial shape: wide tiles (NW = 4)
    (2, 64, 16, 5, 6, 4, 2),      # few tiles, even n and P: 32 x 32 tiles, K pairs dealt to the four waves
    (2, 64, 16, 5, 6, 4, 1),      # few tiles, odd P: the K loop is split over 4 blocks (workspace)
    (1, 96, 8, 3, 5, 3, 1),       # 6 stages of 16: split in 2
    (3, 128, 40, 4, 4, 4, 2),     # 4x4 maps, ragged channel block and ragged last quad tile, 4 stages
    (3, 48, 40, 4, 4, 4, 2),      # same maps, a channel count the small tiles do not take
    (2, 128, 32, 3, 7, 2, 0),     # n = 2 on small tiles (64 input channels per stage: 8 K pairs per wave)
    (5, 64, 72, 2, 3, 4, 4),      # P > n - 1 on tiny maps
]


@pytest.mark.parametrize("shape", MFMA_F32_SHAPES)
def test_mfma_f32_small_shapes_every_element(shape):
    B, Cin, Cout, H, W, n, P = shape
    w = _mk("mfma_f32", 8000 + sum(shape), B, Cin, Cout, H, W, n, P, dtype="f32")
    assert _supported(w, PATHS["mfma"]), "shape should be runnable by the MFMA path"
    _parity(w, PATHS["mfma"], integer=True)
    _parity(w, PATHS["mfma"], integer=False)
    if ukst.ukst_workspace_bytes(ukst.UKST_OP_FORWARD, B, Cin, Cout, H, W, n, P, ukst.UKST_F32):
        _parity(w, PATHS["mfma"], integer=True, workspace=None)   # split K loop
        _parity(w, PATHS["mfma"], integer=False, workspace=None)


@pytest.mark.parametrize("shape", MFMA_F32_SHAPES + [(4, 256, 128, 32, 32, 3, 1), (2, 64, 64, 40, 24, 5, 2)])
def test_bf16_layers_with_other_kernel_sides_run_on_the_fp32_matrix_pipe(shape):
    """bf16 layers whose kernel side the bf16 MFMA kernels do not take (n = 2, 3, 5: the dataset
    kernels of Tables 2-3) are widened on their way into LDS and multiplied by the fp32 MFMA
    kernel instead of falling to the vector ALUs."""
    B, Cin, Cout, H, W, n, P = shape
    w = _mk("mfma_f32_bf16in", 8300 + sum(shape), B, Cin, Cout, H, W, n, P, dtype="bf16")
    name = ukst.ukst_kernel_name(B, Cin, Cout, H, W, n, P, ukst.UKST_BF16_F32, PATHS["mfma"])
    if n == 3 and Cin % 16 == 0 and Cout % 8 == 0 and W % 8 == 0:
        assert name == "ukst_mfma_bf16_kernel"   # 9 taps: the bf16 pipe takes them
    elif n != 4:
        assert name == "ukst_mfma_f32_kernel"
    assert name
    _parity(w, PATHS["mfma"], integer=True)
    _parity(w, PATHS["mfma"], integer=False)
    if ukst.ukst_workspace_bytes(ukst.UKST_OP_FORWARD, B, Cin, Cout, H, W, n, P, ukst.UKST_BF16_F32):
        _parity(w, PATHS["mfma"], integer=False, workspace=None)


THIN_MFMA_SHAPES = [
    # B, Cin, Cout, H, W, n, P      (fp32, Cout <= 4, n in {3, 4}, Cin % 16 == 0, W % 4 == 0)
    (1, 16, 3, 4, 4, 4, 2),      # one partial tile
    (3, 32, 3, 5, 8, 4, 2),      # tiles span images, ragged last tile
    (2, 48, 4, 9, 12, 4, 2),     # four output channels: all 16 MFMA columns in use
    (2, 16, 1, 7, 8, 4, 0),      # P = 0, one output channel
    (2, 16, 2, 6, 16, 4, 1),     # odd P: class order flips (Sec. 3.4)
    (1, 32, 3, 3, 20, 4, 3),     # odd P > 1
    (5, 16, 3, 2, 4, 4, 2),      # many tiny images inside one tile
    (1, 16, 3, 40, 64, 4, 2),    # several tiles per image, wide rows
    (1, 16, 3, 1, 4, 4, 2),      # single input row
    (2, 32, 3, 9, 12, 3, 0),     # n = 3: odd output, classes with fewer taps (Sec. 3.1)
    (2, 16, 4, 6, 8, 3, 1),      # n = 3, odd P
    (1, 16, 2, 5, 8, 3, 2),      # n = 3, P = 2
    (2, 16, 3, 8, 8, 4, 5),      # padding beyond the kernel: zero border
]


@pytest.mark.parametrize("shape", THIN_MFMA_SHAPES)
def test_thin_mfma_small_shapes_every_element(shape):
    B, Cin, Cout, H, W, n, P = shape
    w = _mk("thin_mfma", 8000 + sum(shape), B, Cin, Cout, H, W, n, P)
    assert ukst.ukst_kernel_name(B, Cin, Cout, H, W, n, P, ukst.UKST_F32,
                                 PATHS["mfma"]) == "ukst_thin_mfma_kernel"
    _parity(w, PATHS["mfma"], integer=True)
    _parity(w, PATHS["mfma"], integer=False)


def _parity_sampled_on_device(w, planes, expect_kernel):
    """Large outputs: only the sampled planes (and a guard band on either side of the output)
    travel back to the host."""
    import torch
    from gpu_util import to_device
    print(f"case {w.name} B={w.B} Cin={w.Cin} Cout={w.Cout} H={w.H} W={w.W} n={w.n} P={w.P} "
          f"{w.dtype} planes={planes}", flush=True)
    dt = ukst.UKST_F32 if w.dtype == "f32" else ukst.UKST_BF16_F32
    assert ukst.ukst_kernel_name(w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, dt,
                                 PATHS["auto"]) == expect_kernel
    data = wl.generate(w, integer=True)
    y_ref, S = oracle.naive(data["x"], data["w"], w.P, planes=planes)
    x, wt = to_device(data, w.dtype)
    OH, OW = ukst.ukst_output_shape(w.H, w.W, w.n, w.P)
    numel, guard, sentinel = w.B * w.Cout * OH * OW, 1 << 16, -777.0
    buf = torch.full((numel + 2 * guard,), sentinel, dtype=torch.float32, device="cuda")
    y = buf[guard:guard + numel].view(w.B, w.Cout, OH, OW)
    ukst.ukst_conv_transpose2d(x, wt, w.P, y=y)
    torch.cuda.synchronize()
    assert bool((buf[:guard] == sentinel).all()) and bool((buf[guard + numel:] == sentinel).all())
    yp = y.view(w.B * w.Cout, OH, OW)
    for p in planes:
        got = yp[p].cpu().numpy().astype(np.float64)
        assert np.array_equal(got, y_ref.reshape(w.B * w.Cout, OH, OW)[p]), f"plane {p}"
    return numel


def test_output_beyond_32bit_byte_offsets():
    # 4.7 GB of output: the last plane starts past 2^32 bytes, which only the general kernel
    # (64-bit addressing) may take; integer data, so the comparison is exact
    w = _mk("big_f32", 9101, 2, 2, 3, 7000, 7000, 3, 0)
    numel = _parity_sampled_on_device(w, [0, 3, 5], "ukst_direct_kernel")
    assert numel * 4 > 1 << 32


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_matrix_core_shapes_beyond_their_buffer_limit_fall_back(dtype):
    # a layer the matrix-core kernels would take, but whose output exceeds their single 2 GiB
    # buffer descriptor: automatic selection has to hand it to the general kernel
    w = _mk("big_mfma_shape", 9102, 33, 16, 64, 256, 256, 4, 2, dtype=dtype)
    assert not _supported(w, PATHS["mfma"])
    numel = _parity_sampled_on_device(w, [0, 1000, 33 * 64 - 1], "ukst_direct_kernel")
    assert numel * 4 > (1 << 31)


def test_paths_agree_at_full_size():
    # property that holds at any size: both kernel families compute the same tensor (every
    # element of it, which the sampled planes above cannot show)
    import torch
    from gpu_util import to_device
    ran = 0
    for name in ["cfg5b", "cfg4b", "cfg3_L3", "cfg4a", "cfg5a"]:
        w = wl.WORKLOADS[name]
        if not _supported(w, PATHS["mfma"]):
            continue
        ran += 1
        data = wl.generate(w)
        x, wt = to_device(data, w.dtype)
        ya = ukst.ukst_conv_transpose2d(x, wt, w.P, path=PATHS["direct"])
        yb = ukst.ukst_conv_transpose2d(x, wt, w.P, path=PATHS["mfma"])
        scale = ukst.ukst_conv_transpose2d(x.abs(), wt.abs(), w.P, path=PATHS["direct"])
        torch.cuda.synchronize()
        tol = 2e-5 if w.dtype == "f32" else 2e-2
        assert bool(((ya - yb).abs() <= tol * scale).all()), name
        del ya, yb, scale, x, wt
        torch.cuda.empty_cache()
    if not ran:
        pytest.skip("MFMA path not available for these shapes")


def test_repeat_runs_are_bit_identical():
    w = wl.WORKLOADS["cfg2a"].with_(B=2)
    data = wl.generate(w)
    a = run_gpu(data, w.dtype, w.P)
    b = run_gpu(data, w.dtype, w.P)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("name,kernel", [("cfg2a", "ukst_narrow_kernel"), ("cfg2b", "ukst_narrow_kernel"),
                                         ("cfg3_L1", "ukst_mfma_f32_kernel"),
                                         ("cfg3_L4", "ukst_thin_mfma_kernel"),
                                         ("cfg4a", "ukst_mfma_f32_kernel"),
                                         ("cfg5a", "ukst_mfma_bf16_aligned_kernel"),
                                         ("cfg5a_P1", "ukst_mfma_bf16_kernel"),
                                         ("cfg5b", "ukst_mfma_bf16_aligned_kernel"),
                                         ("cfg5b_P1", "ukst_mfma_bf16_kernel")])
def test_repeat_runs_are_bit_identical_at_full_size(name, kernel):
    """Every kernel family at its benchmark shape, three launches into three different buffers:
    the same bits every time (no atomics, fixed summation order, no store that depends on
    timing)."""
    import torch
    from gpu_util import to_device
    w = (wl.WORKLOADS["cfg5b"].with_(P=1) if name == "cfg5b_P1" else
         wl.WORKLOADS["cfg5a"].with_(P=1) if name == "cfg5a_P1" else wl.WORKLOADS[name])
    dt = ukst.UKST_F32 if w.dtype == "f32" else ukst.UKST_BF16_F32
    assert ukst.ukst_kernel_name(w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P, dt) == kernel
    x, wt = to_device(wl.generate(w), w.dtype)
    ys = [ukst.ukst_conv_transpose2d_ws(x, wt, w.P) for _ in range(3)]
    torch.cuda.synchronize()
    assert torch.equal(ys[0], ys[1]) and torch.equal(ys[0], ys[2]), name


@pytest.mark.parametrize("shape,kernel", [
    ((1, 3, 3, 8, 8, 3, 300), "ukst_narrow_kernel"),    # floor(P/2) = 150 > 2 * 64 lanes: waves of
    ((2, 2, 4, 5, 9, 4, 301), "ukst_narrow_kernel"),    # later strips start left of the map too
    ((1, 1, 1, 4, 4, 5, 520), "ukst_narrow_kernel"),
    ((1, 24, 3, 8, 8, 3, 300), "ukst_thin_kernel"),
    ((1, 8, 2, 5, 9, 4, 301), "ukst_thin_kernel"),
    ((1, 32, 3, 6, 8, 4, 300), "ukst_thin_kernel")])  # the class-column MFMA kernel bounds P
def test_padding_far_beyond_the_kernel(shape, kernel):
    """P in the hundreds: most outputs meet no input at all (exact zeros), the map sits in the
    middle of a wide zero border, and lanes whole strips away from the left edge still have
    windows that start left of the map."""
    B, Cin, Cout, H, W, n, P = shape
    w = _mk("far_padding", 9400 + sum(shape), B, Cin, Cout, H, W, n, P)
    assert ukst.ukst_kernel_name(B, Cin, Cout, H, W, n, P, ukst.UKST_F32) == kernel
    _parity(w, PATHS["auto"], integer=True)
    _parity(w, PATHS["auto"], integer=False)


@pytest.mark.parametrize("case", ["narrow", "mfma_f32_split_k", "mfma_bf16"])
def test_non_default_stream(case):
    """Work (including the split-K partial sums in the workspace and their slice sum) follows the
    caller's stream."""
    import torch
    from gpu_util import to_device
    w = {"narrow": wl.WORKLOADS["cfg1"],
         "mfma_f32_split_k": _mk("stream_f32", 8201, 2, 64, 16, 5, 6, 4, 1),
         "mfma_bf16": _mk("stream_bf16", 8202, 2, 32, 64, 6, 16, 4, 2, dtype="bf16")}[case]
    data = wl.generate(w)
    x, wt = to_device(data, w.dtype)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    need = ukst.ukst_workspace_bytes(ukst.UKST_OP_FORWARD, w.B, w.Cin, w.Cout, w.H, w.W, w.n, w.P,
                                     ukst.UKST_F32 if w.dtype == "f32" else ukst.UKST_BF16_F32)
    assert (need > 0) == (case == "mfma_f32_split_k")
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        y1 = ukst.ukst_conv_transpose2d_ws(x, wt, w.P, workspace=ws, stream=s)
        y2 = ukst.ukst_conv_transpose2d_ws(x, wt, w.P, workspace=ws, stream=s)  # back to back, same workspace
    s.synchronize()
    y_ref, S = oracle.naive(data["x"], data["w"], w.P)
    check_against_oracle(y1.cpu().numpy(), y_ref, S, TOL[w.dtype])
    assert torch.equal(y1, y2)


# ------------------------------------------------------------------ bf16 output (UKST_BF16_BF16)
def _bf16_out_case(w, path, integer, planes=None, bias=None, act=None):
    """bf16 in, bf16 out: one rounding (to nearest even) of the fp32 sum at the store.
    Integer data: the fp32 sum is exact, so the stored bits must equal the rounded exact value.
    Otherwise |y - y_oracle| <= 1e-2 * sum|x*w| (the fp32-sum tolerance) + 2^-8 |y_oracle|
    (half an ulp of bf16 is 2^-9 relative)."""
    import torch
    from gpu_util import to_device
    print(f"case {w.name} B={w.B} Cin={w.Cin} Cout={w.Cout} H={w.H} W={w.W} n={w.n} P={w.P} "
          f"bf16->bf16 path={path} integer={integer}", flush=True)
    data = wl.generate(w, integer=integer)
    y_ref, S = oracle.naive(data["x"], data["w"], w.P, planes=planes)
    x, k = to_device(data, "bf16")
    OH, OW = ukst.ukst_output_shape(w.H, w.W, w.n, w.P)
    numel, guard = w.B * w.Cout * OH * OW, 4096
    buf = torch.full((numel + 2 * guard,), -777.0, dtype=torch.bfloat16, device="cuda")
    y = buf[guard:guard + numel].view(w.B, w.Cout, OH, OW)
    if bias is None:
        ukst.ukst_conv_transpose2d(x, k, w.P, y=y, path=path)
    else:
        ukst.ukst_conv_transpose2d_bias_act(x, k, w.P, bias=torch.from_numpy(bias).cuda(), act=act,
                                            y=y, path=path)
        y_ref = np.maximum(y_ref + bias.astype(np.float64)[None, :, None, None], 0.0)
    torch.cuda.synchronize()
    assert bool((buf[:guard] == -777.0).all()) and bool((buf[guard + numel:] == -777.0).all())
    bits = y.view(torch.int16).cpu().numpy().view(np.uint16).reshape(w.B * w.Cout, -1)
    ref = y_ref.reshape(w.B * w.Cout, -1)
    s = S.reshape(w.B * w.Cout, -1)
    if planes is not None:
        bits, ref, s = bits[planes], ref[planes], s[planes]
    if integer and bias is None:
        want = wl.round_to_bf16_bits(ref.astype(np.float32))
        assert np.array_equal(wl.bf16_bits_to_f32(bits), wl.bf16_bits_to_f32(want))
        return
    got = wl.bf16_bits_to_f32(bits).astype(np.float64)
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    assert (err <= TOL["bf16"] * s + 2.0 ** -8 * np.abs(ref) + 1e-30).all()


@pytest.mark.parametrize("shape", MFMA_BF16_SHAPES)
def test_bf16_output_mfma_small_shapes_every_element(shape):
    B, Cin, Cout, H, W, P = shape
    w = _mk("mfma_bf16_out", 7500 + sum(shape), B, Cin, Cout, H, W, 4, P, dtype="bf16")
    assert ukst.ukst_kernel_name(B, Cin, Cout, H, W, 4, P, ukst.UKST_BF16_BF16,
                                 PATHS["mfma"]).startswith("ukst_mfma_bf16_")
    _bf16_out_case(w, PATHS["mfma"], integer=True)
    _bf16_out_case(w, PATHS["mfma"], integer=False)


@pytest.mark.parametrize("shape", [(2, 3, 3, 5, 9, 3, 0), (1, 9, 5, 6, 37, 4, 2), (2, 17, 2, 11, 7, 5, 1),
                                   (1, 4, 3, 6, 131, 2, 0)])
def test_bf16_output_general_kernel_every_element(shape):
    B, Cin, Cout, H, W, n, P = shape
    w = _mk("direct_bf16_out", 7600 + sum(shape), B, Cin, Cout, H, W, n, P, dtype="bf16")
    _bf16_out_case(w, PATHS["direct"], integer=True)
    _bf16_out_case(w, PATHS["direct"], integer=False)


@pytest.mark.parametrize("name", ["cfg5a", "cfg5b"])
def test_bf16_output_full_size_sampled_planes(name):
    w = wl.WORKLOADS[name]
    planes = _sample_planes(w, 12)
    _bf16_out_case(w, PATHS["auto"], integer=False, planes=planes)
    _bf16_out_case(w, PATHS["auto"], integer=True, planes=planes)
    bias = np.random.default_rng(w.index).normal(0.0, 0.5, w.Cout).astype(np.float32)
    _bf16_out_case(w, PATHS["auto"], integer=False, planes=planes, bias=bias, act=ukst.UKST_ACT_RELU)


# ------------------------------------------------------------------ fused bias + activation
EPILOGUE_CASES = [
    # name, (B, Cin, Cout, H, W, n, P), dtype, path, kernel expected
    ("narrow", (2, 3, 3, 19, 45, 3, 0), "f32", "auto", "ukst_narrow_kernel"),
    ("thin", (2, 24, 3, 9, 11, 4, 2), "f32", "auto", "ukst_thin_kernel"),
    ("general", (2, 8, 8, 9, 11, 5, 1), "f32", "auto", "ukst_direct_kernel"),
    ("general_bf16", (2, 8, 8, 9, 11, 4, 2), "bf16", "auto", "ukst_direct_kernel"),
    ("thin_mfma", (2, 32, 3, 9, 12, 4, 2), "f32", "auto", "ukst_thin_mfma_kernel"),
    ("mfma_f32", (2, 16, 40, 23, 31, 3, 0), "f32", "mfma", "ukst_mfma_f32_kernel"),
    ("mfma_f32_split_k", (2, 64, 16, 5, 6, 4, 1), "f32", "mfma", "ukst_mfma_f32_kernel"),
    ("mfma_f32_small_tiles", (2, 64, 24, 5, 6, 4, 2), "f32", "mfma", "ukst_mfma_f32_kernel"),
    ("mfma_bf16", (2, 32, 128, 9, 16, 4, 1), "bf16", "auto", "ukst_mfma_bf16_kernel"),
    ("mfma_bf16_aligned", (2, 32, 128, 9, 16, 4, 2), "bf16", "auto", "ukst_mfma_bf16_aligned_kernel"),
]


@pytest.mark.parametrize("act", ["none", "relu", "tanh"])
@pytest.mark.parametrize("case", EPILOGUE_CASES, ids=[c[0] for c in EPILOGUE_CASES])
def test_fused_bias_activation(case, act):
    """y = act(conv + bias[co]) from the store of every kernel family, against the oracle's fp64
    sums with the same bias and activation applied in fp64.  tanh and ReLU are 1-Lipschitz, so the
    convolution's tolerance carries over; tanh adds its own fp32 evaluation error (2e-6)."""
    import torch
    from gpu_util import to_device
    name, shape, dtype, pname, kernel = case
    B, Cin, Cout, H, W, n, P = shape
    w = _mk("epi_" + name, 9300 + sum(shape), B, Cin, Cout, H, W, n, P, dtype=dtype)
    dt = ukst.UKST_F32 if dtype == "f32" else ukst.UKST_BF16_F32
    assert ukst.ukst_kernel_name(B, Cin, Cout, H, W, n, P, dt, PATHS[pname]) == kernel
    data = wl.generate(w)
    rng = np.random.default_rng(9300 + sum(shape))
    bias = rng.normal(0.0, 1.0, Cout).astype(np.float32)
    y_ref, S = oracle.naive(data["x"], data["w"], P)
    z = y_ref + bias.astype(np.float64)[None, :, None, None]
    code = {"none": ukst.UKST_ACT_NONE, "relu": ukst.UKST_ACT_RELU, "tanh": ukst.UKST_ACT_TANH}[act]
    ref = {"none": z, "relu": np.maximum(z, 0.0), "tanh": np.tanh(z)}[act]
    x, k = to_device(data, dtype)
    # the split-K case needs the workspace entry point (the slice sum applies the epilogue there)
    ws = None if name == "mfma_f32_split_k" else False
    y = ukst.ukst_conv_transpose2d_bias_act(x, k, P, bias=torch.from_numpy(bias).cuda(), act=code,
                                            path=PATHS[pname], workspace=ws)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    # the bias is added in fp32 to an fp32 sum: half an ulp of the biased value on top
    slack = TOL[dtype] * S + 1.2e-7 * np.abs(z) + (2e-6 if act == "tanh" else 0.0)
    err = np.abs(got - ref)
    assert np.isfinite(got).all()
    assert (err <= slack).all(), f"worst excess {np.max(err - slack):.3e}"
    if act == "none":
        # no bias and no activation: bit-identical to the plain entry point
        y0 = ukst.ukst_conv_transpose2d(x, k, P, path=PATHS[pname], workspace=ws)
        y1 = ukst.ukst_conv_transpose2d_bias_act(x, k, P, bias=None, act=ukst.UKST_ACT_NONE,
                                                 path=PATHS[pname], workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(y0, y1)


@pytest.mark.parametrize("name", ["cfg2a", "cfg3_L1", "cfg3_L4", "cfg4b", "cfg5b"])
def test_fused_bias_relu_full_size_sampled_planes(name):
    # the benchmark shapes through the fused entry point (narrow, split-K fp32 MFMA + slice sum,
    # thin MFMA, fp32 MFMA, bf16 MFMA), on a seeded sample of complete (b, co) planes
    import torch
    from gpu_util import to_device
    w = wl.WORKLOADS[name]
    planes = _sample_planes(w, 12)
    data = wl.generate(w)
    bias = np.random.default_rng(w.index).normal(0.0, 0.5, w.Cout).astype(np.float32)
    y_ref, S = oracle.naive(data["x"], data["w"], w.P, planes=planes)
    x, k = to_device(data, w.dtype)
    y = ukst.ukst_conv_transpose2d_bias_act(x, k, w.P, bias=torch.from_numpy(bias).cuda(),
                                            act=ukst.UKST_ACT_RELU, workspace=None)
    torch.cuda.synchronize()
    OH, OW = y.shape[2:]
    got = y.view(w.B * w.Cout, OH, OW)[planes].cpu().numpy().astype(np.float64)
    z = y_ref.reshape(w.B * w.Cout, OH, OW)[planes] + bias.astype(np.float64)[np.array(planes) % w.Cout, None, None]
    ref = np.maximum(z, 0.0)
    slack = TOL[w.dtype] * S.reshape(w.B * w.Cout, OH, OW)[planes] + 1.2e-7 * np.abs(z)
    err = np.abs(got - ref)
    assert (err <= slack).all(), f"worst excess {np.max(err - slack):.3e}"


# ------------------------------------------------------------------ buffers with element alignment only
@pytest.mark.parametrize("dtype,cout", [("f32", 64), ("bf16", 64), ("f32", 3)])
def test_unaligned_buffers_take_the_vector_alu_kernels(dtype, cout):
    """x, w one element past a 16-byte boundary: AUTO must still be right, forced MFMA must refuse."""
    import torch
    w = _mk("unaligned", 8100, 2, 32, cout, 6, 16, 4, 2, dtype=dtype)
    data = wl.generate(w)
    y_ref, S = oracle.naive(data["x"], data["w"], w.P)
    if dtype == "bf16":
        tx = torch.from_numpy(data["x_bits"].view(np.int16)).view(torch.bfloat16)
        tk = torch.from_numpy(data["w_bits"].view(np.int16)).view(torch.bfloat16)
    else:
        tx, tk = torch.from_numpy(data["x"]), torch.from_numpy(data["w"])

    def shifted(t):  # same values, storage starting one element after an aligned address
        buf = torch.empty(t.numel() + 1, dtype=t.dtype, device="cuda")
        v = buf[1:].view(t.shape)
        v.copy_(t)
        assert v.data_ptr() % 16 != 0
        return v

    x, k = shifted(tx), shifted(tk)
    y = ukst.ukst_conv_transpose2d(x, k, w.P)
    torch.cuda.synchronize()
    check_against_oracle(y.cpu().numpy(), y_ref, S, TOL[dtype])
    with pytest.raises(ukst.UkstError):
        ukst.ukst_conv_transpose2d(x, k, w.P, path=PATHS["mfma"])
    torch.cuda.synchronize()
