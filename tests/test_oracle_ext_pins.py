"""Pins of the CPU oracle's extension (no GPU): stride-s transpose convolution and dilated
convolution, the two generalisations Sec. 5 of the paper points to.  Each oracle of record is tied
to things other than itself: hand-worked fixtures, the already pinned stride-2 oracle, library
routines in fp64 (torch, scipy), closed forms, and an independently written segregated twin."""
import itertools
import os

import numpy as np
import pytest

import oracle


def _fixture(golden_dir, name):
    out = {}
    for line in open(os.path.join(golden_dir, name)):
        if line.startswith("#") or ":" not in line:
            continue
        k, v = line.split(":", 1)
        out[k.strip()] = [float(t) for t in v.split()]
    return out


def _ints(rng, shape):
    return rng.integers(-3, 4, size=shape).astype(np.float64)


# ------------------------------------------------------------------ stride-s transpose convolution
def test_strided_hand_worked_fixture(golden_dir):
    f = _fixture(golden_dir, "worked_stride3_2x2_k2.txt")
    H, W, n, s, P = (int(f[k][0]) for k in ("H", "W", "n", "s", "P"))
    x = np.array(f["x"]).reshape(1, 1, H, W)
    w = np.array(f["w"]).reshape(1, 1, n, n)
    want = np.array(f["y"]).reshape(5, 5)
    assert oracle.out_shape_strided(H, W, n, P, s) == (5, 5)
    for fn in (oracle.strided_naive, oracle.strided_segregated):
        y, S = fn(x, w, P, s)
        assert np.array_equal(y[0, 0], want)
        assert np.array_equal(S[0, 0], want)  # all terms positive
    # a flipped or transposed kernel must not reproduce the fixture
    assert not np.array_equal(oracle.strided_naive(x, w[:, :, ::-1, ::-1].copy(), P, s)[0][0, 0], want)
    assert not np.array_equal(oracle.strided_naive(x, w.transpose(0, 1, 3, 2).copy(), P, s)[0][0, 0], want)


def test_strided_s2_is_the_papers_case():
    # stride 2 must be Algorithm 1 itself: the pinned oracle of record
    rng = np.random.default_rng(1)
    for (B, Cin, Cout, H, W, n, P) in [(1, 1, 1, 4, 4, 3, 0), (2, 3, 2, 3, 5, 4, 2), (1, 2, 3, 5, 2, 5, 3),
                                       (2, 1, 1, 1, 6, 2, 1), (1, 2, 2, 4, 4, 1, 0)]:
        x, w = _ints(rng, (B, Cin, H, W)), _ints(rng, (Cout, Cin, n, n))
        y2, S2 = oracle.naive(x, w, P)
        y, S = oracle.strided_naive(x, w, P, 2)
        assert y.shape == y2.shape and np.array_equal(y, y2) and np.array_equal(S, S2)


def test_strided_naive_and_segregated_agree_exactly_on_a_tiny_grid():
    rng = np.random.default_rng(2)
    cases = 0
    for H, W, n, P, s in itertools.product(range(1, 5), range(1, 4), range(1, 6), range(0, 5), range(1, 5)):
        OH, OW = oracle.out_shape_strided(H, W, n, P, s)
        if OH < 1 or OW < 1:
            continue
        x, w = _ints(rng, (1, 1, H, W)), _ints(rng, (1, 1, n, n))
        a, Sa = oracle.strided_naive(x, w, P, s)
        b, Sb = oracle.strided_segregated(x, w, P, s)
        assert np.array_equal(a, b) and np.array_equal(Sa, Sb), (H, W, n, P, s)
        cases += 1
    assert cases > 800
    for (B, Cin, Cout, H, W, n, P, s) in [(2, 3, 2, 3, 4, 3, 1, 3), (1, 2, 3, 4, 2, 5, 4, 4), (3, 1, 2, 2, 2, 4, 0, 3)]:
        x, w = _ints(rng, (B, Cin, H, W)), _ints(rng, (Cout, Cin, n, n))
        assert np.array_equal(oracle.strided_naive(x, w, P, s)[0], oracle.strided_segregated(x, w, P, s)[0])


def test_strided_against_torch_and_scipy_fp64():
    torch = pytest.importorskip("torch")
    from scipy.signal import correlate2d
    rng = np.random.default_rng(3)
    for (B, Cin, Cout, H, W, n, s) in [(2, 3, 2, 4, 5, 3, 3), (1, 2, 3, 3, 3, 4, 3), (1, 1, 2, 5, 4, 5, 4),
                                       (2, 2, 2, 4, 4, 2, 1), (1, 3, 1, 3, 6, 3, 2)]:
        x, w = rng.standard_normal((B, Cin, H, W)), rng.standard_normal((Cout, Cin, n, n))
        for P in range(0, n):
            if min(oracle.out_shape_strided(H, W, n, P, s)) < 1:
                continue
            y, _ = oracle.strided_naive(x, w, P, s)
            ref = torch.nn.functional.conv_transpose2d(
                torch.from_numpy(x), torch.from_numpy(w).flip(2, 3).transpose(0, 1).contiguous(),
                stride=s, padding=n - 1 - P).numpy()
            assert ref.shape == y.shape and np.abs(ref - y).max() < 1e-12, (H, W, n, s, P)
    # stride 1: no inserted zeros at all, a plain correlation of the padded map
    x, w = rng.standard_normal((1, 1, 5, 4)), rng.standard_normal((1, 1, 3, 3))
    y, _ = oracle.strided_naive(x, w, 2, 1)
    assert np.abs(y[0, 0] - correlate2d(np.pad(x[0, 0], 2), w[0, 0], mode="valid")).max() < 1e-12


def test_strided_closed_forms():
    rng = np.random.default_rng(4)
    # delta input: the kernel stamped (flipped) at stride s
    H, W, n, P, s = 3, 4, 4, 2, 3
    w = _ints(rng, (1, 1, n, n))
    for (i, j) in [(0, 0), (1, 2), (2, 3)]:
        x = np.zeros((1, 1, H, W))
        x[0, 0, i, j] = 1.0
        y, _ = oracle.strided_naive(x, w, P, s)
        OH, OW = y.shape[2:]
        for oy, ox in itertools.product(range(OH), range(OW)):
            a, c = s * i + P - oy, s * j + P - ox
            want = w[0, 0, a, c] if 0 <= a < n and 0 <= c < n else 0.0
            assert y[0, 0, oy, ox] == want
    # full padding: every tap of every pixel lands inside the output
    x, w = _ints(rng, (2, 3, 3, 5)), _ints(rng, (2, 3, 4, 4))
    y, S = oracle.strided_naive(x, w, 3, 3)
    for b, co in itertools.product(range(2), range(2)):
        assert y[b, co].sum() == sum(x[b, ci].sum() * w[co, ci].sum() for ci in range(3))
    assert np.array_equal(S, oracle.strided_naive(np.abs(x), np.abs(w), 3, 3)[0])
    # all ones: an output row of class r = (P - oy) mod s counts ceil((n - r)/s) taps at most
    y, _ = oracle.strided_naive(np.ones((1, 1, 6, 6)), np.ones((1, 1, 5, 5)), 4, 3)
    oy = 8  # interior row: class r = (4 - 8) mod 3 = 2 -> taps 2 only ... ceil((5-2)/3) = 1
    assert y[0, 0, oy, oy] == 1 * 1 and y[0, 0, 7, 7] == 2 * 2 and y[0, 0, 7, 8] == 2 * 1


# ------------------------------------------------------------------ dilated convolution
def test_dilated_hand_worked_fixture(golden_dir):
    f = _fixture(golden_dir, "worked_dilated2_4x4_k2.txt")
    H, W, n, d, P = (int(f[k][0]) for k in ("H", "W", "n", "d", "P"))
    x = np.array(f["x"]).reshape(1, 1, H, W)
    w = np.array(f["w"]).reshape(1, 1, n, n)
    want = np.array(f["y"]).reshape(2, 2)
    assert oracle.out_shape_dilated(H, W, n, P, d) == (2, 2)
    for fn in (oracle.dilated_naive, oracle.dilated_segregated):
        y, S = fn(x, w, P, d)
        assert np.array_equal(y[0, 0], want) and np.array_equal(S[0, 0], want)
    assert not np.array_equal(oracle.dilated_naive(x, w[:, :, ::-1, ::-1].copy(), P, d)[0][0, 0], want)
    assert not np.array_equal(oracle.dilated_naive(x, w.transpose(0, 1, 3, 2).copy(), P, d)[0][0, 0], want)


def test_dilated_naive_and_segregated_agree_exactly_on_a_tiny_grid():
    rng = np.random.default_rng(5)
    cases = 0
    for H, W, n, P, d in itertools.product(range(1, 6), range(1, 5), range(1, 4), range(0, 4), range(1, 5)):
        OH, OW = oracle.out_shape_dilated(H, W, n, P, d)
        if OH < 1 or OW < 1:
            continue
        x, w = _ints(rng, (1, 1, H, W)), _ints(rng, (1, 1, n, n))
        a, Sa = oracle.dilated_naive(x, w, P, d)
        b, Sb = oracle.dilated_segregated(x, w, P, d)
        assert np.array_equal(a, b) and np.array_equal(Sa, Sb), (H, W, n, P, d)
        cases += 1
    assert cases > 400
    for (B, Cin, Cout, H, W, n, P, d) in [(2, 3, 2, 7, 6, 3, 1, 2), (1, 2, 3, 9, 5, 2, 0, 3), (3, 1, 2, 5, 5, 3, 4, 2)]:
        x, w = _ints(rng, (B, Cin, H, W)), _ints(rng, (Cout, Cin, n, n))
        assert np.array_equal(oracle.dilated_naive(x, w, P, d)[0], oracle.dilated_segregated(x, w, P, d)[0])


def test_dilated_against_torch_and_scipy_fp64():
    torch = pytest.importorskip("torch")
    from scipy.signal import correlate2d
    rng = np.random.default_rng(6)
    for (B, Cin, Cout, H, W, n, d, P) in [(2, 3, 2, 9, 8, 3, 2, 0), (1, 2, 3, 7, 7, 3, 3, 3), (1, 1, 2, 6, 9, 2, 4, 2),
                                          (2, 2, 2, 5, 5, 4, 1, 1), (1, 3, 1, 8, 6, 5, 2, 4)]:
        x, w = rng.standard_normal((B, Cin, H, W)), rng.standard_normal((Cout, Cin, n, n))
        y, _ = oracle.dilated_naive(x, w, P, d)
        ref = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w), dilation=d,
                                         padding=P).numpy()
        assert ref.shape == y.shape and np.abs(ref - y).max() < 1e-12, (H, W, n, d, P)
    # dilation 1: a plain correlation of the padded map
    x, w = rng.standard_normal((1, 1, 5, 4)), rng.standard_normal((1, 1, 3, 3))
    y, _ = oracle.dilated_naive(x, w, 1, 1)
    assert np.abs(y[0, 0] - correlate2d(np.pad(x[0, 0], 1), w[0, 0], mode="valid")).max() < 1e-12


def test_dilated_closed_forms():
    rng = np.random.default_rng(7)
    # delta kernel: the output is the padded input shifted by d times the tap position
    H, W, n, P, d = 6, 7, 3, 2, 2
    x = _ints(rng, (1, 1, H, W))
    xp = np.pad(x[0, 0], P)
    for (a, c) in [(0, 0), (1, 2), (2, 1)]:
        w = np.zeros((1, 1, n, n))
        w[0, 0, a, c] = 1.0
        y, _ = oracle.dilated_naive(x, w, P, d)
        OH, OW = y.shape[2:]
        assert np.array_equal(y[0, 0], xp[d * a:d * a + OH, d * c:d * c + OW])
    # all ones without padding: every output counts all n*n taps (none meets an inserted zero twice)
    y, _ = oracle.dilated_naive(np.ones((1, 2, 9, 9)), np.ones((1, 2, 3, 3)), 0, 3)
    assert y.shape == (1, 1, 3, 3) and (y == 18).all()
    x, w = _ints(rng, (2, 2, 6, 5)), _ints(rng, (3, 2, 2, 2))
    assert np.array_equal(oracle.dilated_naive(x, w, 1, 3)[1], oracle.dilated_naive(np.abs(x), np.abs(w), 1, 3)[0])
    # linearity in x
    x2 = _ints(rng, (2, 2, 6, 5))
    assert np.array_equal(oracle.dilated_naive(x + 2 * x2, w, 1, 3)[0],
                          oracle.dilated_naive(x, w, 1, 3)[0] + 2 * oracle.dilated_naive(x2, w, 1, 3)[0])
