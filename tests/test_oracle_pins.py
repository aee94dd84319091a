"""Pins for the CPU oracle (no GPU).  Each test checks ``oracle.naive`` -- and the two check
formulations -- against something other than itself: hand-worked values for the paper's example
shapes, closed forms, invariants, library routines, and exact three-way agreement on tiny
integer inputs."""
import itertools
import os

import numpy as np
import pytest

import oracle

FORMS = [oracle.naive, oracle.scatter, oracle.segregated]


def _read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, vals = line.split(":")
            out.setdefault(key.strip(), []).append([int(v) for v in vals.split()])
    return out


# ---------------------------------------------------------------- hand-worked fixtures
@pytest.mark.parametrize("form", FORMS)
def test_worked_4x4_k3(golden_dir, form):
    g = _read_golden(os.path.join(golden_dir, "worked_4x4_k3.txt"))
    H, W, n = g["H"][0][0], g["W"][0][0], g["n"][0][0]
    x = np.array(g["x"][0], dtype=np.float64).reshape(1, 1, H, W)
    w = np.array(g["w"][0], dtype=np.float64).reshape(1, 1, n, n)
    y0, _ = form(x, w, 0)
    assert y0.shape == (1, 1, 5, 5)
    assert np.array_equal(y0.ravel(), np.array(g["y_P0"][0], dtype=np.float64))
    y2, _ = form(x, w, 2)
    assert y2.shape == (1, 1, 9, 9)
    assert y2.sum() == g["sum_P2"][0][0]
    c = g["corners_P2"][0]
    assert [y2[0, 0, 0, 0], y2[0, 0, 0, 8], y2[0, 0, 8, 0], y2[0, 0, 8, 8]] == c
    assert np.array_equal(y2[0, 0, 2:7, 2:7], y0[0, 0])
    # the fixture discriminates: a flipped or transposed kernel must NOT reproduce it
    for wrong in (w[:, :, ::-1, ::-1], w.transpose(0, 1, 3, 2)):
        yw, _ = form(x, np.ascontiguousarray(wrong), 0)
        assert not np.array_equal(yw, y0)


@pytest.mark.parametrize("form", FORMS)
def test_worked_2x2_k3(golden_dir, form):
    g = _read_golden(os.path.join(golden_dir, "worked_2x2_k3.txt"))
    x = np.array(g["x"][0], dtype=np.float64).reshape(1, 1, 2, 2)
    w = np.array(g["w"][0], dtype=np.float64).reshape(1, 1, 3, 3)
    assert form(x, w, 0)[0].ravel().tolist() == g["y_P0"][0]
    assert form(x, w, 2)[0].ravel().tolist() == g["y_P2"][0]


def test_paper_shapes(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "paper_shapes.txt"))
    for N, n, P, side in g["shape"]:
        assert oracle.out_shape(N, N, n, P) == (side, side)
        if N <= 8:
            y, _ = oracle.naive(np.ones((1, 1, N, N)), np.ones((1, 1, n, n)), P)
            assert y.shape == (1, 1, side, side)
    # 5x5 kernel: interior pixels of the four classes use 9, 6, 6, 4 taps (Sec. 3.2), 25 in all
    counts = g["subkernel_counts_n5"][0]
    for form in FORMS:
        y, _ = form(np.ones((1, 1, 8, 8)), np.ones((1, 1, 5, 5)), 0)
        quad = y[0, 0, 4:6, 4:6].ravel().tolist()
        assert quad == counts and sum(quad) == 25


# ---------------------------------------------------------------- three formulations, exact
def test_three_formulations_agree_exhaustive_single_channel():
    rng = np.random.default_rng(1)
    cases = 0
    for H, W, n, P in itertools.product(range(1, 5), range(1, 5), range(1, 7), range(0, 7)):
        if 2 * H + 2 * P - n < 1 or 2 * W + 2 * P - n < 1:
            continue
        x = rng.integers(-3, 4, size=(1, 1, H, W)).astype(np.float64)
        w = rng.integers(-3, 4, size=(1, 1, n, n)).astype(np.float64)
        (ya, sa), (yb, sb), (yc, sc) = (f(x, w, P) for f in FORMS)
        assert np.array_equal(ya, yb) and np.array_equal(ya, yc), (H, W, n, P)
        assert np.array_equal(sa, sb) and np.array_equal(sa, sc), (H, W, n, P)
        cases += 1
    assert cases > 500


def test_three_formulations_agree_multichannel():
    rng = np.random.default_rng(2)
    for B, Cin, Cout in itertools.product((1, 2, 3), repeat=3):
        for (H, W, n, P) in [(3, 5, 3, 0), (4, 2, 4, 2), (5, 3, 5, 1), (2, 6, 2, 3), (3, 3, 7, 6)]:
            x = rng.integers(-3, 4, size=(B, Cin, H, W)).astype(np.float64)
            w = rng.integers(-3, 4, size=(Cout, Cin, n, n)).astype(np.float64)
            ya, yb, yc = (f(x, w, P)[0] for f in FORMS)
            assert np.array_equal(ya, yb) and np.array_equal(ya, yc)


# ---------------------------------------------------------------- closed forms / invariants
@pytest.mark.parametrize("n,P", [(3, 0), (4, 2), (5, 1), (5, 4), (2, 0), (1, 0), (6, 3)])
def test_delta_input_stamps_kernel(n, P):
    H, W = 5, 6
    rng = np.random.default_rng(3)
    w = rng.standard_normal((2, 1, n, n))
    for (i, j) in [(0, 0), (2, 3), (4, 5), (1, 0)]:
        x = np.zeros((1, 1, H, W))
        x[0, 0, i, j] = 1.0
        y, _ = oracle.naive(x, w, P)
        OH, OW = y.shape[2:]
        expect = np.zeros_like(y)
        for a in range(n):
            for c in range(n):
                oy, ox = 2 * i + P - a, 2 * j + P - c
                if 0 <= oy < OH and 0 <= ox < OW:
                    expect[0, :, oy, ox] = w[:, 0, a, c]
        assert np.array_equal(y, expect)


@pytest.mark.parametrize("form", FORMS)
def test_all_ones_counts_taps(form):
    # with x = w = 1 the output counts in-range taps; rows and columns are independent, so the
    # plane is an outer product, and with full padding every input row meets all n tap rows.
    H, W, n, Cin = 4, 6, 5, 3
    for P in (0, 1, 2, 4):
        y, S = form(np.ones((1, Cin, H, W)), np.ones((2, Cin, n, n)), P)
        plane = y[0, 0] / Cin
        rows, cols = plane[:, plane.shape[1] // 2], plane[plane.shape[0] // 2, :]
        assert np.array_equal(y, S)
        assert np.array_equal(y[0, 0], y[0, 1])
        # separable: plane * plane[c,c] == outer(col profile, row profile)
        c0, c1 = plane.shape[0] // 2, plane.shape[1] // 2
        assert np.array_equal(plane * plane[c0, c1], np.outer(rows, cols))
        if P >= n - 1:
            assert plane.sum() == H * W * n * n
    # P = 0, n = 5: row tap counts alternate 3,2,3,... (ceil / floor of n/2)
    y, _ = form(np.ones((1, 1, 4, 4)), np.ones((1, 1, 5, 5)), 0)
    assert y[0, 0, :, 0].tolist() == [9, 6, 9] and y[0, 0, 1, :].tolist() == [6, 4, 6]


def test_full_padding_sum_invariant():
    rng = np.random.default_rng(4)
    B, Cin, Cout, H, W = 2, 3, 2, 3, 4
    for n in (2, 3, 4, 5):
        x = rng.integers(-3, 4, size=(B, Cin, H, W)).astype(np.float64)
        w = rng.integers(-3, 4, size=(Cout, Cin, n, n)).astype(np.float64)
        for P in (n - 1, n, n + 2):
            y, _ = oracle.naive(x, w, P)
            expect = np.einsum("bc,oc->bo", x.sum((2, 3)), w.sum((2, 3)))
            assert np.array_equal(y.sum((2, 3)), expect)


def test_linearity_and_crop_and_abs_scale():
    rng = np.random.default_rng(5)
    x1 = rng.integers(-3, 4, size=(2, 2, 4, 5)).astype(np.float64)
    x2 = rng.integers(-3, 4, size=(2, 2, 4, 5)).astype(np.float64)
    w1 = rng.integers(-3, 4, size=(3, 2, 4, 4)).astype(np.float64)
    w2 = rng.integers(-3, 4, size=(3, 2, 4, 4)).astype(np.float64)
    for P in (0, 1, 2, 3):
        y11 = oracle.naive(x1, w1, P)[0]
        assert np.array_equal(oracle.naive(x1 + 2 * x2, w1, P)[0],
                              y11 + 2 * oracle.naive(x2, w1, P)[0])
        assert np.array_equal(oracle.naive(x1, w1 - 3 * w2, P)[0],
                              y11 - 3 * oracle.naive(x1, w2, P)[0])
        # padding P is the central crop of padding P+1
        assert np.array_equal(oracle.naive(x1, w1, P + 1)[0][:, :, 1:-1, 1:-1], y11)
        # S is the same operation on absolute values
        assert np.array_equal(oracle.naive(x1, w1, P)[1],
                              oracle.naive(np.abs(x1), np.abs(w1), P)[0])


def test_padding_beyond_kernel_gives_zero_border():
    x = np.ones((1, 1, 2, 2))
    w = np.ones((1, 1, 2, 2))
    y, S = oracle.naive(x, w, 3)  # windows in the outer ring touch no input
    assert y.shape == (1, 1, 8, 8)
    assert not y[0, 0, 0, :].any() and not y[0, 0, :, 0].any() and not S[0, 0, -1, :].any()
    assert y.sum() == 4 * 4


def test_n1_has_three_empty_classes():
    x = np.arange(1.0, 7.0).reshape(1, 1, 2, 3)
    w = np.full((1, 1, 1, 1), 2.0)
    for form in FORMS:
        y, _ = form(x, w, 0)
        assert y[0, 0].tolist() == [[2, 0, 4, 0, 6], [0, 0, 0, 0, 0], [8, 0, 10, 0, 12]]


# ---------------------------------------------------------------- library routines
def test_matches_torch_conv_transpose2d_fp64():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(6)
    for (B, Cin, Cout, H, W, n) in [(2, 3, 2, 5, 7, 3), (1, 2, 4, 6, 4, 4), (2, 2, 2, 3, 3, 5),
                                    (1, 1, 1, 8, 8, 2), (1, 3, 2, 4, 9, 6)]:
        x = rng.standard_normal((B, Cin, H, W))
        w = rng.standard_normal((Cout, Cin, n, n))
        for P in range(0, n):
            y, _ = oracle.naive(x, w, P)
            wt = torch.from_numpy(w).flip(2, 3).transpose(0, 1).contiguous()
            ref = torch.nn.functional.conv_transpose2d(torch.from_numpy(x), wt, stride=2,
                                                       padding=n - 1 - P).numpy()
            assert ref.shape == y.shape
            assert np.abs(ref - y).max() <= 1e-12 * max(1.0, np.abs(y).max())


def test_matches_scipy_correlate_of_zero_inserted_map():
    signal = pytest.importorskip("scipy.signal")
    rng = np.random.default_rng(7)
    H, W, n, P = 5, 4, 4, 3
    x = rng.standard_normal((1, 2, H, W))
    w = rng.standard_normal((1, 2, n, n))
    y, _ = oracle.naive(x, w, P)
    acc = 0.0
    for ci in range(2):
        U = np.zeros((2 * H - 1, 2 * W - 1))
        U[::2, ::2] = x[0, ci]
        acc = acc + signal.correlate2d(np.pad(U, P), w[0, ci], mode="valid")
    assert np.abs(acc - y[0, 0]).max() < 1e-12


# ---------------------------------------------------------------- plane selection
def test_plane_subset_matches_full():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((3, 2, 4, 4))
    w = rng.standard_normal((4, 2, 3, 3))
    yf, Sf = oracle.naive(x, w, 1)
    planes = [0, 5, 11]
    ys, Ss = oracle.naive(x, w, 1, planes=planes)
    yf2, ys2 = yf.reshape(12, -1), ys.reshape(12, -1)
    for p in range(12):
        if p in planes:
            assert np.array_equal(yf2[p], ys2[p])
        else:
            assert not ys2[p].any()
    assert np.array_equal(Sf.reshape(12, -1)[planes], Ss.reshape(12, -1)[planes])


def test_bad_arguments_raise():
    with pytest.raises(ValueError):
        oracle.naive(np.ones((1, 1, 1, 1)), np.ones((1, 1, 3, 3)), 0)  # 2*1-3 < 1
    with pytest.raises(ValueError):
        oracle.naive(np.ones((1, 2, 3, 3)), np.ones((1, 1, 3, 3)), 0)  # Cin mismatch
