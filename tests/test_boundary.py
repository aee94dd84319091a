"""Host-side checks of the C-ABI library (no GPU): it loads, exports what include/ukst.h declares,
validates arguments before touching the GPU, and its host arithmetic is right."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2502_20493_amd import binding as ukst
from paper_2502_20493_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "ukst.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ukst_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(ukst.LIB_PATH)
    declared = _declared_symbols()
    assert len(declared) >= 8
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(ukst.EXPORTS) == declared


def test_bench_library_exports_every_declared_symbol():
    # the measured ceilings live in a library of their own: the product ABI has no benchmark kernel
    text = open(os.path.join(ROOT, "include", "ukst_bench.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = sorted(set(re.findall(r"\b(ukst_[a-z0-9_]+)\s*\(", text)))
    lib = ctypes.CDLL(ukst.BENCH_LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(ukst.BENCH_EXPORTS) == declared
    product = ctypes.CDLL(ukst.LIB_PATH)
    for name in declared:
        assert not hasattr(product, name), name


def test_version_and_status_strings():
    assert ukst.ukst_version() >= 100
    seen = {ukst.ukst_status_string(s) for s in range(7)}
    assert len(seen) == 7 and ukst.ukst_status_string(0) == "ok"
    assert ukst.ukst_status_string(99) == "unknown status"


def test_output_shape():
    assert ukst.ukst_output_shape(4, 4, 3, 0) == (5, 5)      # Sec. 1
    assert ukst.ukst_output_shape(4, 4, 3, 2) == (9, 9)      # Fig. 2
    assert ukst.ukst_output_shape(4, 4, 5, 2) == (7, 7)      # Figs. 5-6
    assert ukst.ukst_output_shape(224, 200, 3, 0) == (445, 397)
    for bad in [(1, 4, 3, 0), (4, 1, 3, 0), (0, 4, 3, 2), (4, 4, 0, 0), (4, 4, 3, -1)]:
        with pytest.raises(ukst.UkstError) as e:
            ukst.ukst_output_shape(*bad)
        assert e.value.status == ukst.UKST_ERR_SHAPE
    oh = ctypes.c_int(0)
    assert ukst.lib().ukst_output_shape(4, 4, 3, 0, None, ctypes.byref(oh)) == ukst.UKST_ERR_NULL


def test_validation_happens_on_the_host():
    # fake non-null addresses: validation must reject before any launch
    X = W = Y = 0x1000
    call = ukst.ukst_conv_transpose2d_raw
    ok_shape = (1, 1, 1, 4, 4, 3, 0)
    assert call(None, W, Y, *ok_shape, 0) == ukst.UKST_ERR_NULL
    assert call(X, None, Y, *ok_shape, 0) == ukst.UKST_ERR_NULL
    assert call(X, W, None, *ok_shape, 0) == ukst.UKST_ERR_NULL
    for bad in [(0, 1, 1, 4, 4, 3, 0), (1, 0, 1, 4, 4, 3, 0), (1, 1, 0, 4, 4, 3, 0),
                (1, 1, 1, 0, 4, 3, 0), (1, 1, 1, 4, 0, 3, 0), (1, 1, 1, 4, 4, 0, 0),
                (1, 1, 1, 4, 4, 3, -1), (1, 1, 1, 1, 4, 3, 0), (1, 1, 1, 4, 1, 3, 0)]:
        assert call(X, W, Y, *bad, 0) == ukst.UKST_ERR_SHAPE, bad
    assert call(X, W, Y, *ok_shape, 3) == ukst.UKST_ERR_DTYPE
    assert call(X, W, Y, *ok_shape, -1) == ukst.UKST_ERR_DTYPE
    assert call(X, W, Y, 1, 1, 1, 8, 8, ukst.UKST_MAX_N + 1, 0, 0) == ukst.UKST_ERR_UNSUPPORTED
    assert call(X, W, Y, *ok_shape, 0, path=7) == ukst.UKST_ERR_UNSUPPORTED
    # MFMA path cannot run a 1-channel problem
    assert call(X, W, Y, *ok_shape, 0, path=ukst.UKST_PATH_MFMA) == ukst.UKST_ERR_UNSUPPORTED
    # element alignment: fp32 buffers at 4 bytes, a bf16 output at 2
    assert call(X + 2, W, Y, *ok_shape, 0) == ukst.UKST_ERR_UNSUPPORTED
    assert call(X, W, Y + 2, *ok_shape, ukst.UKST_BF16_F32) == ukst.UKST_ERR_UNSUPPORTED
    assert call(X, W, Y + 1, *ok_shape, ukst.UKST_BF16_BF16) == ukst.UKST_ERR_UNSUPPORTED
    # the fused entry point validates the same way, plus the activation code
    fused = ukst.lib().ukst_conv_transpose2d_bias_act
    assert fused(X, W, None, None, *ok_shape, 0, 0, 0, None) == ukst.UKST_ERR_NULL
    assert fused(X, W, None, Y, 1, 1, 1, 0, 4, 3, 0, 0, 0, 0, None) == ukst.UKST_ERR_SHAPE
    assert fused(X, W, None, Y, *ok_shape, 0, 9, 0, None) == ukst.UKST_ERR_UNSUPPORTED
    assert fused(X, W, X + 2, Y, *ok_shape, 0, 1, 0, None) == ukst.UKST_ERR_UNSUPPORTED
    # the backward entry points validate the same way; gradients are fp32 only
    for back in (ukst.lib().ukst_conv_transpose2d_grad_input, ukst.lib().ukst_conv_transpose2d_grad_weight):
        assert back(None, W, Y, *ok_shape, 0, None, 0, None) == ukst.UKST_ERR_NULL
        assert back(X, None, Y, *ok_shape, 0, None, 0, None) == ukst.UKST_ERR_NULL
        assert back(X, W, None, *ok_shape, 0, None, 0, None) == ukst.UKST_ERR_NULL
        assert back(X, W, Y, 1, 1, 1, 4, 1, 3, 0, 0, None, 0, None) == ukst.UKST_ERR_SHAPE
        assert back(X, W, Y, *ok_shape, 5, None, 0, None) == ukst.UKST_ERR_DTYPE
        assert back(X, W, Y, *ok_shape, ukst.UKST_BF16_BF16, None, 0, None) == ukst.UKST_ERR_UNSUPPORTED
        assert back(X, W, Y, 1, 1, 1, 8, 8, ukst.UKST_MAX_N + 1, 0, 0, None, 0, None) == ukst.UKST_ERR_UNSUPPORTED
        assert back(X + 2, W, Y, *ok_shape, 0, None, 0, None) == ukst.UKST_ERR_UNSUPPORTED
        assert back(X, W, Y + 2, *ok_shape, ukst.UKST_BF16_F32, None, 0, None) == ukst.UKST_ERR_UNSUPPORTED
        # workspace: NULL with a size, or misaligned, is refused before anything else happens
        assert back(X, W, Y, *ok_shape, 0, None, 64, None) == ukst.UKST_ERR_WORKSPACE
        assert back(X, W, Y, *ok_shape, 0, 0x1010, 1 << 20, None) == ukst.UKST_ERR_WORKSPACE


def test_workspace_sizes_are_host_arithmetic():
    """ukst_workspace_bytes needs no GPU, and a call whose workspace is too small is refused on the
    host (fake addresses: nothing may be launched)."""
    wsb = ukst.ukst_workspace_bytes
    F, GI, GW = ukst.UKST_OP_FORWARD, ukst.UKST_OP_GRAD_INPUT, ukst.UKST_OP_GRAD_WEIGHT
    w = wl.WORKLOADS

    def shape(k):
        return (w[k].B, w[k].Cin, w[k].Cout, w[k].H, w[k].W, w[k].n, w[k].P)

    # forward: only layers whose K loop is split want one (a whole number of copies of y)
    for k in ("cfg1", "cfg2a", "cfg2b", "cfg3_L4", "cfg4a", "cfg4b"):
        assert wsb(F, *shape(k), ukst.UKST_F32) == 0, k
    for k in ("cfg5a", "cfg5b"):
        assert wsb(F, *shape(k), ukst.UKST_BF16_F32) == 0, k
    # kernel gradient: always a whole number of copies of dw, at least one
    for k in ("cfg2a", "cfg3_L1", "cfg3_L4", "cfg4a"):
        n_dw = w[k].Cout * w[k].Cin * w[k].n ** 2 * 4
        got = wsb(GW, *shape(k), ukst.UKST_F32)
        assert got >= n_dw and got % n_dw == 0, k
    # input gradient: the vector-ALU kernels need none, the matrix-core kernels at least the
    # packed weights
    assert wsb(GI, *shape("cfg2a"), ukst.UKST_F32) == 0
    assert wsb(GI, *shape("cfg4a"), ukst.UKST_F32) >= 128 * 128 * 25 * 4
    assert wsb(GI, *shape("cfg5a"), ukst.UKST_BF16_F32) >= 128 * 256 * 16 * 2
    # invalid arguments give 0
    assert wsb(7, *shape("cfg4a"), ukst.UKST_F32) == 0
    assert wsb(GW, 1, 1, 1, 1, 4, 3, 0, ukst.UKST_F32) == 0
    assert wsb(GW, *shape("cfg4a"), ukst.UKST_BF16_BF16) == 0
    # too small a workspace is a host-side error
    X = W = Y = 0x1000
    WS = 0x10000
    need = wsb(GW, *shape("cfg4a"), ukst.UKST_F32)
    gw = ukst.lib().ukst_conv_transpose2d_grad_weight
    assert gw(X, W, Y, *shape("cfg4a"), ukst.UKST_F32, WS, need - 1, None) == ukst.UKST_ERR_WORKSPACE
    assert gw(X, W, Y, *shape("cfg4a"), ukst.UKST_F32, None, 0, None) == ukst.UKST_ERR_WORKSPACE
    gi = ukst.lib().ukst_conv_transpose2d_grad_input
    need = wsb(GI, *shape("cfg4a"), ukst.UKST_F32)
    assert gi(X, W, Y, *shape("cfg4a"), ukst.UKST_F32, WS, need - 1, None) == ukst.UKST_ERR_WORKSPACE
    fw = ukst.lib().ukst_conv_transpose2d_ws
    ok_shape = (1, 1, 1, 4, 4, 3, 0)
    assert fw(X, W, None, Y, *ok_shape, 0, 0, 0, None, 16, None) == ukst.UKST_ERR_WORKSPACE
    assert fw(X, W, None, Y, *ok_shape, 0, 0, 0, WS + 8, 1 << 20, None) == ukst.UKST_ERR_WORKSPACE
    assert fw(None, W, None, Y, *ok_shape, 0, 0, 0, None, 0, None) == ukst.UKST_ERR_NULL


def _brute_macs(H, W, n, P):
    """Count products by walking the padded upsampled map of Algorithm 1."""
    OH, OW = 2 * H + 2 * P - n, 2 * W + 2 * P - n
    U = np.zeros((2 * H - 1 + 2 * P, 2 * W - 1 + 2 * P), dtype=np.int64)
    U[P:P + 2 * H - 1:2, P:P + 2 * W - 1:2] = 1
    exact = sum(int(U[oy:oy + n, ox:ox + n].sum()) for oy in range(OH) for ox in range(OW))
    hi, lo = (n + 1) // 2, n // 2
    nominal = sum((hi if (oy + P) % 2 == 0 else lo) * (hi if (ox + P) % 2 == 0 else lo)
                  for oy in range(OH) for ox in range(OW))
    return exact, nominal, OH * OW * n * n


def test_mac_counts():
    for (H, W, n, P) in [(4, 4, 3, 0), (4, 4, 4, 2), (5, 3, 5, 0), (5, 3, 5, 3), (3, 6, 2, 1),
                         (4, 4, 7, 6), (2, 2, 1, 0), (2, 3, 2, 4)]:
        e, nom, nv = _brute_macs(H, W, n, P)
        for kind, want in ((0, e), (1, nom), (2, nv)):
            assert ukst.ukst_mac_count(2, 3, 5, H, W, n, P, kind) == 2 * 3 * 5 * want
        assert e <= nom <= nv
    # Sec. 3.1: 25 multiplications per four outputs for n = 5 instead of 100
    assert ukst.ukst_mac_count(1, 1, 1, 8, 8, 5, 0, 1) * 4 < ukst.ukst_mac_count(1, 1, 1, 8, 8, 5, 0, 2) * 1.1
    assert ukst.ukst_mac_count(1, 1, 1, 1, 8, 5, 0, 0) == 0  # invalid shape
    # figures used by the benchmark (GFLOP = 2 * MAC / 1e9)
    assert ukst.ukst_mac_count(16, 3, 3, 224, 224, 3, 0, 0) == 16 * 9 * 668 * 668  # rows: 223 even outputs x 2 taps + 222 odd x 1
    assert abs(2 * ukst.ukst_mac_count(32, 128, 128, 64, 64, 5, 0, 0) / 1e9 - 99.47) < 0.01


def test_select_path():
    assert ukst.ukst_select_path(16, 3, 3, 224, 224, 3, 0, ukst.UKST_F32) == ukst.UKST_PATH_DIRECT
    # few output channels: the parity classes fill the MFMA columns when Cin % 16 == 0, W % 4 == 0
    assert ukst.ukst_select_path(64, 64, 3, 32, 32, 4, 2, ukst.UKST_F32) == ukst.UKST_PATH_MFMA
    assert ukst.ukst_kernel_name(64, 64, 3, 32, 32, 4, 2, 0) == "ukst_thin_mfma_kernel"
    assert ukst.ukst_select_path(64, 24, 3, 32, 31, 4, 2, ukst.UKST_F32) == ukst.UKST_PATH_DIRECT
    assert ukst.ukst_kernel_name(64, 24, 3, 32, 31, 4, 2, 0) == "ukst_thin_kernel"
    assert ukst.ukst_select_path(32, 256, 128, 128, 128, 4, 2, ukst.UKST_BF16_F32) == ukst.UKST_PATH_MFMA
    with pytest.raises(ukst.UkstError):
        ukst.ukst_select_path(16, 3, 3, 1, 224, 3, 0, ukst.UKST_F32)
    assert "narrow" in ukst.ukst_kernel_name(16, 3, 3, 224, 224, 3, 0, 0)
    assert "direct" in ukst.ukst_kernel_name(16, 8, 8, 224, 224, 3, 0, 0)
    assert ukst.ukst_kernel_name(16, 3, 3, 1, 224, 3, 0, 0) == ""


def test_workloads_are_seeded_and_shaped():
    from paper_2502_20493_amd import workloads as wl
    a = wl.generate(wl.WORKLOADS["cfg1"])
    b = wl.generate(wl.WORKLOADS["cfg1"])
    assert a["x"].shape == (1, 1, 32, 32) and a["w"].shape == (1, 1, 3, 3)
    assert np.array_equal(a["x"], b["x"]) and np.array_equal(a["w"], b["w"])
    i = wl.generate(wl.WORKLOADS["cfg1_int"])
    assert set(np.unique(i["x"])).issubset(set(range(-3, 4)))
    small = wl.WORKLOADS["cfg5b"].with_(B=1, Cin=8, Cout=4)
    d = wl.generate(small)
    assert d["x_bits"].dtype == np.uint16
    # bf16 values survive a second rounding unchanged, and rounding is to nearest even
    assert np.array_equal(wl.round_to_bf16_bits(d["x"]), d["x_bits"])
    t = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7], dtype=np.float32)
    assert wl.bf16_bits_to_f32(wl.round_to_bf16_bits(t)).tolist() == [1.0, 1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7]


def test_backward_kernel_selection_is_host_arithmetic():
    """ukst_grad_kernel_name needs no GPU: wide layers go to the matrix cores (bf16 operands to the
    bf16 pipe for the input gradient), narrow ones to the vector ALUs."""
    name = ukst.ukst_grad_kernel_name
    w = wl.WORKLOADS
    def shape(k):
        return (w[k].B, w[k].Cin, w[k].Cout, w[k].H, w[k].W, w[k].n, w[k].P)
    for k in ("cfg2a", "cfg2b"):  # narrow fp32 image layers: register-blocked strips
        assert name(0, *shape(k), ukst.UKST_F32) == "ukst_grad_input_narrow_kernel"
        assert name(1, *shape(k), ukst.UKST_F32) == "ukst_grad_weight_narrow_kernel"
    # narrow layers those kernels do not take: bf16 operands, maps narrower than 32, n = 1 or n > 5
    assert name(0, *shape("cfg2a"), ukst.UKST_BF16_F32) == "ukst_grad_input_kernel"
    assert name(1, *shape("cfg2a"), ukst.UKST_BF16_F32) == "ukst_grad_weight_kernel"
    assert name(0, 2, 3, 3, 40, 24, 3, 0, ukst.UKST_F32) == "ukst_grad_input_kernel"
    assert name(1, 2, 3, 3, 40, 40, 6, 0, ukst.UKST_F32) == "ukst_grad_weight_kernel"
    assert name(1, 2, 3, 3, 40, 40, 1, 0, ukst.UKST_F32) == "ukst_grad_weight_kernel"
    assert name(0, *shape("cfg3_L4"), ukst.UKST_F32) == "ukst_grad_input_kernel"      # Cout = 3
    assert name(1, *shape("cfg3_L4"), ukst.UKST_F32) == "ukst_grad_weight_thin_mfma_kernel"  # 3 x 16 rows
    assert name(1, 2, 16, 5, 16, 16, 4, 2, ukst.UKST_F32) == "ukst_grad_weight_kernel"   # 5 x 16 rows: too many
    assert name(1, 2, 16, 3, 16, 2, 3, 0, ukst.UKST_F32) == "ukst_grad_weight_kernel"    # rows of two pixels
    assert name(1, 2, 16, 3, 16, 16, 3, 0, ukst.UKST_F32) == "ukst_grad_weight_thin_mfma_kernel"
    for k in ("cfg3_L1", "cfg3_L2", "cfg3_L3", "cfg4a", "cfg4b"):
        assert name(0, *shape(k), ukst.UKST_F32) == "ukst_grad_input_mfma_kernel", k
        assert name(1, *shape(k), ukst.UKST_F32) == "ukst_grad_weight_mfma_kernel", k
    for k in ("cfg5a", "cfg5b"):
        assert name(0, *shape(k), ukst.UKST_BF16_F32) == "ukst_grad_input_window_mfma_bf16_kernel", k
        assert name(1, *shape(k), ukst.UKST_BF16_F32) == "ukst_grad_weight_mfma_bf16_kernel", k
    # bf16 layers the bf16-pipe kernel gradient does not take (n = 5, rows that are no multiple of 8)
    assert name(1, 2, 64, 64, 16, 16, 5, 2, ukst.UKST_BF16_F32) == "ukst_grad_weight_mfma_kernel"
    assert name(1, 2, 64, 64, 16, 20, 4, 2, ukst.UKST_BF16_F32) == "ukst_grad_weight_mfma_kernel"
    # bf16 layers the window kernel does not take: n other than 2, 3 or 4, at most 64 input channels or no multiple of
    # 8, output channels that are no multiple of 8, maps narrower than 16
    assert name(0, 2, 132, 32, 16, 16, 4, 2, ukst.UKST_BF16_F32) == "ukst_grad_input_mfma_bf16_kernel"
    assert name(0, 2, 128, 32, 16, 16, 2, 0, ukst.UKST_BF16_F32) == "ukst_grad_input_window_mfma_bf16_kernel"
    assert name(0, 2, 128, 32, 16, 16, 1, 0, ukst.UKST_BF16_F32) != "ukst_grad_input_window_mfma_bf16_kernel"
    assert name(0, 2, 128, 32, 16, 16, 5, 2, ukst.UKST_BF16_F32) == "ukst_grad_input_mfma_bf16_kernel"
    assert name(0, 2, 128, 32, 16, 16, 3, 1, ukst.UKST_BF16_F32) == "ukst_grad_input_window_mfma_bf16_kernel"
    assert name(0, 2, 64, 32, 16, 16, 4, 2, ukst.UKST_BF16_F32) == "ukst_grad_input_mfma_bf16_kernel"
    assert name(0, 2, 128, 36, 16, 16, 4, 2, ukst.UKST_BF16_F32) == "ukst_grad_input_mfma_bf16_kernel"
    assert name(0, 2, 128, 40, 16, 16, 4, 2, ukst.UKST_BF16_F32) == "ukst_grad_input_window_mfma_bf16_kernel"
    assert name(0, 2, 128, 32, 16, 8, 4, 2, ukst.UKST_BF16_F32) == "ukst_grad_input_mfma_bf16_kernel"
    assert name(0, 2, 128, 32, 16, 16, 4, 2, ukst.UKST_BF16_F32) == "ukst_grad_input_window_mfma_bf16_kernel"
    # kernel sides whose tile does not fit the bf16 kernel's LDS budget fall back to the fp32 pipe
    assert name(0, 2, 64, 32, 40, 40, 7, 3, ukst.UKST_BF16_F32) == "ukst_grad_input_mfma_kernel"
    assert name(0, 1, 1, 1, 4, 4, 3, 0, ukst.UKST_BF16_BF16) == ""
    assert name(2, 1, 1, 1, 4, 4, 3, 0, ukst.UKST_F32) == ""
    assert name(0, 1, 1, 1, 1, 4, 3, 0, ukst.UKST_F32) == ""


def test_generalised_operations_host_side():
    """Stride-s transpose convolution and dilated convolution: shapes, multiply-add counts and
    argument validation are host arithmetic (fake addresses: nothing may be launched)."""
    assert ukst.ukst_output_shape_strided(4, 4, 3, 0, 2) == ukst.ukst_output_shape(4, 4, 3, 0)
    assert ukst.ukst_output_shape_strided(2, 2, 2, 1, 3) == (5, 5)     # tests/golden/worked_stride3_2x2_k2.txt
    assert ukst.ukst_output_shape_dilated(4, 4, 2, 0, 2) == (2, 2)     # tests/golden/worked_dilated2_4x4_k2.txt
    assert ukst.ukst_output_shape_dilated(9, 7, 3, 2, 3) == (7, 5)
    for bad in [(0, 4, 3, 0, 2), (4, 4, 0, 0, 2), (4, 4, 3, -1, 2), (4, 4, 3, 0, 0), (1, 1, 3, 0, 2)]:
        with pytest.raises(ukst.UkstError) as e:
            ukst.ukst_output_shape_strided(*bad)
        assert e.value.status == ukst.UKST_ERR_SHAPE
    with pytest.raises(ukst.UkstError):
        ukst.ukst_output_shape_dilated(4, 4, 3, 0, 2)  # 4 - 2*2 = 0: empty output

    def brute_strided(H, W, n, P, s):
        OH, OW = s * (H - 1) + 2 * P - n + 2, s * (W - 1) + 2 * P - n + 2
        U = np.zeros((s * (H - 1) + 1 + 2 * P, s * (W - 1) + 1 + 2 * P), dtype=np.int64)
        U[P:P + s * (H - 1) + 1:s, P:P + s * (W - 1) + 1:s] = 1
        return sum(int(U[oy:oy + n, ox:ox + n].sum()) for oy in range(OH) for ox in range(OW)), OH * OW * n * n

    def brute_dilated(H, W, n, P, d):
        OH, OW = H + 2 * P - d * (n - 1), W + 2 * P - d * (n - 1)
        X = np.pad(np.ones((H, W), dtype=np.int64), P)
        nd = d * (n - 1) + 1
        return sum(int(X[oy:oy + nd:d, ox:ox + nd:d].sum()) for oy in range(OH) for ox in range(OW)), OH * OW * nd * nd

    for (H, W, n, P, k) in [(4, 4, 3, 0, 2), (3, 5, 4, 2, 3), (5, 3, 5, 3, 4), (2, 2, 2, 1, 3), (6, 4, 3, 2, 1)]:
        e, nv = brute_strided(H, W, n, P, k)
        assert ukst.ukst_mac_count_strided(2, 3, 5, H, W, n, P, k, 0) == 30 * e
        assert ukst.ukst_mac_count_strided(2, 3, 5, H, W, n, P, k, 2) == 30 * nv
        assert e <= ukst.ukst_mac_count_strided(1, 1, 1, H, W, n, P, k, 1) <= nv
    assert ukst.ukst_mac_count_strided(2, 3, 5, 4, 4, 3, 1, 2, 0) == ukst.ukst_mac_count(2, 3, 5, 4, 4, 3, 1, 0)
    assert ukst.ukst_mac_count_strided(2, 3, 5, 4, 4, 3, 1, 2, 1) == ukst.ukst_mac_count(2, 3, 5, 4, 4, 3, 1, 1)
    for (H, W, n, P, k) in [(9, 8, 3, 0, 2), (7, 7, 3, 3, 3), (6, 9, 2, 2, 4), (5, 5, 4, 1, 1)]:
        e, nv = brute_dilated(H, W, n, P, k)
        assert ukst.ukst_mac_count_dilated(2, 3, 5, H, W, n, P, k, 0) == 30 * e
        assert ukst.ukst_mac_count_dilated(2, 3, 5, H, W, n, P, k, 2) == 30 * nv
    X = W_ = Y = 0x1000
    for f in (ukst.lib().ukst_conv_transpose2d_strided, ukst.lib().ukst_dilated_conv2d):
        ok = (1, 1, 1, 8, 8, 3, 1, 2)
        assert f(None, W_, Y, *ok, 0, None) == ukst.UKST_ERR_NULL
        assert f(X, W_, None, *ok, 0, None) == ukst.UKST_ERR_NULL
        assert f(X, W_, Y, 1, 1, 1, 8, 8, 3, 1, 0, 0, None) == ukst.UKST_ERR_SHAPE
        assert f(X, W_, Y, 0, 1, 1, 8, 8, 3, 1, 2, 0, None) == ukst.UKST_ERR_SHAPE
        assert f(X, W_, Y, *ok, 7, None) == ukst.UKST_ERR_DTYPE
        assert f(X, W_, Y, *ok, ukst.UKST_BF16_BF16, None) == ukst.UKST_ERR_UNSUPPORTED
        assert f(X, W_, Y, 1, 1, 1, 8, 8, 3, 1, 9, 0, None) == ukst.UKST_ERR_UNSUPPORTED
        assert f(X + 2, W_, Y, *ok, 0, None) == ukst.UKST_ERR_UNSUPPORTED
    assert ukst.lib().ukst_dilated_conv2d(X, W_, Y, 1, 1, 1, 4, 4, 3, 0, 2, 0, None) == ukst.UKST_ERR_SHAPE
