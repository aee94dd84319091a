"""Pins for the backward-pass oracle (no GPU).  ``oracle.grad_input`` / ``oracle.grad_weight``
are checked against things other than themselves: hand-worked values, the forward oracle of
record through the adjoint identity (element by element, with unit vectors, in exact integer
arithmetic), closed forms, and a library autograd."""
import itertools
import os

import numpy as np
import pytest

import oracle
from test_oracle_pins import _read_golden


def _ints(rng, shape):
    return rng.integers(-3, 4, size=shape).astype(np.float64)


def test_worked_backward_2x2_k3(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "worked_backward_2x2_k3.txt"))
    x = np.array(g["x"][0], dtype=np.float64).reshape(1, 1, 2, 2)
    w = np.array(g["w"][0], dtype=np.float64).reshape(1, 1, 3, 3)
    one = np.ones((1, 1, 1, 1))
    assert oracle.grad_input(one, w, 2, 2, 0)[0].ravel().tolist() == g["dx_P0"][0]
    assert oracle.grad_weight(x, one, 3, 0)[0].ravel().tolist() == g["dw_P0"][0]
    oy, ox = g["dy_P2_delta_at"][0]
    d = np.zeros((1, 1, 5, 5))
    d[0, 0, oy, ox] = 1.0
    assert oracle.grad_input(d, w, 2, 2, 2)[0].ravel().tolist() == g["dx_P2_delta"][0]
    assert oracle.grad_weight(x, d, 3, 2)[0].ravel().tolist() == g["dw_P2_delta"][0]
    ones = np.ones((1, 1, 5, 5))
    assert oracle.grad_input(ones, w, 2, 2, 2)[0].ravel().tolist() == g["dx_P2_ones"][0]
    assert oracle.grad_weight(x, ones, 3, 2)[0].ravel().tolist() == g["dw_P2_ones"][0]
    # the fixture discriminates: a flipped or transposed kernel must not reproduce it
    for wrong in (w[:, :, ::-1, ::-1], w.transpose(0, 1, 3, 2)):
        assert oracle.grad_input(d, np.ascontiguousarray(wrong), 2, 2, 2)[0].ravel().tolist() \
            != g["dx_P2_delta"][0]


def _tiny_cases():
    for H, W, n, P in itertools.product((1, 2, 3), (1, 2, 3), (1, 2, 3, 4, 5), (0, 1, 2, 3, 5)):
        if 2 * H + 2 * P - n >= 1 and 2 * W + 2 * P - n >= 1:
            yield H, W, n, P


def test_every_gradient_element_is_the_forward_coefficient():
    """dx[e] = <dy, forward(unit_e, w)> and dw[t] = <dy, forward(x, unit_t)> for every element,
    forward = the oracle of record; integer data, exact.  A wrong index, sign, flip or a swapped
    channel in either gradient changes at least one element."""
    rng = np.random.default_rng(20493)
    count = 0
    for H, W, n, P in _tiny_cases():
        B, Cin, Cout = 1 + count % 2, 1 + (count // 2) % 2, 1 + (count // 4) % 2
        count += 1
        OH, OW = oracle.out_shape(H, W, n, P)
        x, w = _ints(rng, (B, Cin, H, W)), _ints(rng, (Cout, Cin, n, n))
        dy = _ints(rng, (B, Cout, OH, OW))
        dx, _ = oracle.grad_input(dy, w, H, W, P)
        dw, _ = oracle.grad_weight(x, dy, n, P)
        for idx in np.ndindex(x.shape):
            e = np.zeros_like(x)
            e[idx] = 1.0
            assert dx[idx] == np.sum(dy * oracle.naive(e, w, P)[0]), (H, W, n, P, idx)
        for idx in np.ndindex(w.shape):
            e = np.zeros_like(w)
            e[idx] = 1.0
            assert dw[idx] == np.sum(dy * oracle.naive(x, e, P)[0]), (H, W, n, P, idx)
    assert count > 150


@pytest.mark.parametrize("shape", [(2, 3, 4, 5, 7, 3, 0), (3, 4, 2, 6, 5, 4, 2), (2, 2, 3, 7, 4, 5, 1),
                                   (1, 5, 3, 4, 9, 5, 4), (2, 3, 3, 8, 8, 2, 0), (2, 2, 2, 3, 5, 4, 3)])
def test_adjoint_identity(shape):
    """<dy, forward(x, w)> = <dx, x> = <dw, w> (the map is bilinear); integers, exact."""
    B, Cin, Cout, H, W, n, P = shape
    rng = np.random.default_rng(sum(shape))
    OH, OW = oracle.out_shape(H, W, n, P)
    x, w = _ints(rng, (B, Cin, H, W)), _ints(rng, (Cout, Cin, n, n))
    dy = _ints(rng, (B, Cout, OH, OW))
    lhs = np.sum(dy * oracle.naive(x, w, P)[0])
    assert lhs == np.sum(x * oracle.grad_input(dy, w, H, W, P)[0])
    assert lhs == np.sum(w * oracle.grad_weight(x, dy, n, P)[0])


@pytest.mark.parametrize("n,P", [(3, 0), (3, 2), (4, 2), (4, 3), (5, 0), (5, 4), (2, 1), (1, 0)])
def test_against_library_autograd(n, P):
    """Special case that is a library routine: for 0 <= P <= n-1 the layer equals torch's
    conv_transpose2d (flipped, transposed weight, padding n-1-P); its fp64 autograd gives both
    gradients."""
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(100 * n + P)
    B, Cin, Cout, H, W = 2, 3, 2, 5, 6
    OH, OW = oracle.out_shape(H, W, n, P)
    x = rng.standard_normal((B, Cin, H, W))
    w = rng.standard_normal((Cout, Cin, n, n))
    dy = rng.standard_normal((B, Cout, OH, OW))
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    y = F.conv_transpose2d(xt, wt.flip(2, 3).transpose(0, 1), stride=2, padding=n - 1 - P)
    assert tuple(y.shape) == dy.shape
    y.backward(torch.tensor(dy))
    np.testing.assert_allclose(oracle.grad_input(dy, w, H, W, P)[0], xt.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.grad_weight(x, dy, n, P)[0], wt.grad.numpy(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("n,P", [(3, 2), (4, 3), (5, 4), (5, 6), (2, 3)])
def test_all_ones_closed_form(n, P):
    """With P >= n-1 every tap of every input pixel lands inside the output, so for dy = 1:
    dx[b,ci,i,j] = sum over co and taps of w[co,ci], dw[co,ci,a,c] = sum over b and pixels of
    x[b,ci]."""
    rng = np.random.default_rng(n * 10 + P)
    B, Cin, Cout, H, W = 2, 3, 2, 3, 4
    OH, OW = oracle.out_shape(H, W, n, P)
    x, w = _ints(rng, (B, Cin, H, W)), _ints(rng, (Cout, Cin, n, n))
    ones = np.ones((B, Cout, OH, OW))
    dx, Sx = oracle.grad_input(ones, w, H, W, P)
    dw, Sw = oracle.grad_weight(x, ones, n, P)
    for ci in range(Cin):
        assert (dx[:, ci] == w[:, ci].sum()).all()
        assert (Sx[:, ci] == np.abs(w[:, ci]).sum()).all()
        assert (dw[:, ci] == x[:, ci].sum()).all()
        assert (Sw[:, ci] == np.abs(x[:, ci]).sum()).all()


def test_delta_reads_back_the_stamp():
    """dy = 1 at one output pixel: dx is the kernel read back at stride 2 (the mirror of the
    forward delta-input stamp), dw is the window of the padded bed of nails under that pixel."""
    rng = np.random.default_rng(7)
    H, W, n, P = 4, 5, 5, 3
    OH, OW = oracle.out_shape(H, W, n, P)
    x, w = _ints(rng, (1, 1, H, W)), _ints(rng, (1, 1, n, n))
    U = np.zeros((2 * H - 1 + 2 * P, 2 * W - 1 + 2 * P))
    U[P:P + 2 * H:2, P:P + 2 * W:2] = x[0, 0]
    for oy, ox in [(0, 0), (3, 4), (OH - 1, OW - 1), (2, 7)]:
        d = np.zeros((1, 1, OH, OW))
        d[0, 0, oy, ox] = 1.0
        dx = oracle.grad_input(d, w, H, W, P)[0][0, 0]
        for i in range(H):
            for j in range(W):
                a, c = 2 * i + P - oy, 2 * j + P - ox
                want = w[0, 0, a, c] if 0 <= a < n and 0 <= c < n else 0.0
                assert dx[i, j] == want
        assert np.array_equal(oracle.grad_weight(x, d, n, P)[0][0, 0], U[oy:oy + n, ox:ox + n])
