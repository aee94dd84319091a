"""TEST INFRASTRUCTURE ONLY: CPU fp64 oracle for stride-2 transpose convolution.

Only the tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It shares nothing with the HIP library: no kernels, headers, helpers or
tables.  The arithmetic lives in ``ukst_oracle.c`` (plain C, fp64); this module compiles it with
gcc, loads it through ctypes and converts numpy arrays.

``strided_naive`` / ``dilated_naive`` (``ukst_oracle_ext.c``) are the oracles of record for the two
generalisations Sec. 5 points to (general stride s; dilated convolution), each pinned with its
``*_segregated`` twin by ``tests/test_oracle_ext_pins.py``.

``naive`` is the oracle of record (Algorithm 1 of the paper: bed-of-nails upsample, pad by P,
stride-1 n x n window).  ``scatter`` and ``segregated`` (Algorithm 2 / Eqs. 1-4 / Sec. 3.4) are
independent formulations used only to pin ``naive``.  ``grad_input`` and ``grad_weight`` are the
adjoints of Algorithm 1 (the backward pass of the layer; the paper treats the forward only).
Every function is pinned by ``tests/test_oracle_pins.py`` / ``tests/test_oracle_backward_pins.py``;
none is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ukst_oracle.c")
_SRC_EXT = os.path.join(_HERE, "ukst_oracle_ext.c")
_LIB = os.path.join(_HERE, "libukst_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP).  Returns the library path."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_EXT))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, _SRC_EXT, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        i = ctypes.c_int
        lib.ukst_oracle_naive.argtypes = [dp, dp, dp, dp, i, i, i, i, i, i, i, ip, i]
        lib.ukst_oracle_naive.restype = i
        for f in (lib.ukst_oracle_scatter, lib.ukst_oracle_segregated):
            f.argtypes = [dp, dp, dp, dp, i, i, i, i, i, i, i]
            f.restype = i
        for f in (lib.ukst_oracle_grad_input, lib.ukst_oracle_grad_weight):
            f.argtypes = [dp, dp, dp, dp, i, i, i, i, i, i, i]
            f.restype = i
        for f in (lib.ukst_oracle_strided_naive, lib.ukst_oracle_strided_segregated,
                  lib.ukst_oracle_dilated_naive, lib.ukst_oracle_dilated_segregated):
            f.argtypes = [dp, dp, dp, dp, i, i, i, i, i, i, i, i]
            f.restype = i
        lib.ukst_oracle_threads.restype = i
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the naive oracle will use."""
    return int(_load().ukst_oracle_threads())


def out_shape(H: int, W: int, n: int, P: int):
    """Sec. 1: an N x N map gives (2N-n) x (2N-n); padding the upsampled map by P adds 2P."""
    return 2 * H + 2 * P - n, 2 * W + 2 * P - n


def _prep(x, w):
    x = np.ascontiguousarray(np.asarray(x, dtype=np.float64))
    w = np.ascontiguousarray(np.asarray(w, dtype=np.float64))
    if x.ndim != 4 or w.ndim != 4 or w.shape[2] != w.shape[3] or w.shape[1] != x.shape[1]:
        raise ValueError("expected x[B,Cin,H,W] and w[Cout,Cin,n,n]")
    return x, w


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _call(name, x, w, P, planes=None):
    x, w = _prep(x, w)
    B, Cin, H, W = x.shape
    Cout, _, n, _ = w.shape
    OH, OW = out_shape(H, W, n, P)
    if OH < 1 or OW < 1 or P < 0:
        raise ValueError("empty output")
    y = np.zeros((B, Cout, OH, OW), dtype=np.float64)
    S = np.zeros(y.shape, dtype=np.float64)  # untouched planes stay unmapped pages
    lib = _load()
    if name == "naive":
        if planes is None:
            rc = lib.ukst_oracle_naive(_dp(x), _dp(w), _dp(y), _dp(S), B, Cin, Cout, H, W, n, P,
                                       None, 0)
        else:
            pl = np.ascontiguousarray(np.asarray(planes, dtype=np.int32))
            rc = lib.ukst_oracle_naive(_dp(x), _dp(w), _dp(y), _dp(S), B, Cin, Cout, H, W, n, P,
                                       pl.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), len(pl))
    else:
        rc = getattr(lib, "ukst_oracle_" + name)(_dp(x), _dp(w), _dp(y), _dp(S), B, Cin, Cout,
                                                 H, W, n, P)
    if rc != 0:
        raise RuntimeError(f"oracle {name} failed with code {rc}")
    return y, S


def naive(x, w, P, planes=None):
    """Oracle of record.  Returns (y, S) in fp64; S = sum |x*w| per output (tolerance scale).

    ``planes``: optional list of plane ids b*Cout+co; other planes of the result stay zero.
    """
    return _call("naive", x, w, P, planes)


def scatter(x, w, P):
    """Check-only formulation: each input pixel adds x*w at stride 2."""
    return _call("scatter", x, w, P)


def segregated(x, w, P):
    """Check-only formulation: four parity sub-kernels selected per output pixel."""
    return _call("segregated", x, w, P)


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def grad_input(dy, w, H, W, P):
    """Adjoint of Algorithm 1 w.r.t. the input.  dy[B,Cout,OH,OW], w[Cout,Cin,n,n] ->
    (dx[B,Cin,H,W], S) in fp64; S = sum |dy*w| per element (tolerance scale)."""
    dy, w = _f64(dy), _f64(w)
    B, Cout, OH, OW = dy.shape
    Cout2, Cin, n, n2 = w.shape
    if Cout2 != Cout or n != n2 or (OH, OW) != out_shape(H, W, n, P):
        raise ValueError("expected dy[B,Cout,2H+2P-n,2W+2P-n] and w[Cout,Cin,n,n]")
    dx = np.zeros((B, Cin, H, W), dtype=np.float64)
    S = np.zeros_like(dx)
    rc = _load().ukst_oracle_grad_input(_dp(dy), _dp(w), _dp(dx), _dp(S), B, Cin, Cout, H, W, n, P)
    if rc != 0:
        raise RuntimeError(f"oracle grad_input failed with code {rc}")
    return dx, S


def grad_weight(x, dy, n, P):
    """Adjoint of Algorithm 1 w.r.t. the kernel.  x[B,Cin,H,W], dy[B,Cout,OH,OW] ->
    (dw[Cout,Cin,n,n], S) in fp64; S = sum |x*dy| per element (tolerance scale)."""
    x, dy = _f64(x), _f64(dy)
    B, Cin, H, W = x.shape
    B2, Cout, OH, OW = dy.shape
    if B2 != B or (OH, OW) != out_shape(H, W, n, P):
        raise ValueError("expected x[B,Cin,H,W] and dy[B,Cout,2H+2P-n,2W+2P-n]")
    dw = np.zeros((Cout, Cin, n, n), dtype=np.float64)
    S = np.zeros_like(dw)
    rc = _load().ukst_oracle_grad_weight(_dp(x), _dp(dy), _dp(dw), _dp(S), B, Cin, Cout, H, W, n, P)
    if rc != 0:
        raise RuntimeError(f"oracle grad_weight failed with code {rc}")
    return dw, S


def out_shape_strided(H: int, W: int, n: int, P: int, s: int):
    """Stride-s transpose convolution: the map is upsampled to s(H-1)+1, padded by P, and an
    n x n window slides over it with stride 1."""
    return s * (H - 1) + 2 * P - n + 2, s * (W - 1) + 2 * P - n + 2


def out_shape_dilated(H: int, W: int, n: int, P: int, d: int):
    """Dilated convolution: the kernel is upsampled to d(n-1)+1 and slides over the input padded
    by P."""
    return H + 2 * P - d * (n - 1), W + 2 * P - d * (n - 1)


def _call_ext(name, x, w, P, k, shape_fn):
    x, w = _prep(x, w)
    B, Cin, H, W = x.shape
    Cout, _, n, _ = w.shape
    OH, OW = shape_fn(H, W, n, P, k)
    if OH < 1 or OW < 1 or P < 0 or k < 1:
        raise ValueError("empty output")
    y = np.zeros((B, Cout, OH, OW), dtype=np.float64)
    S = np.zeros_like(y)
    rc = getattr(_load(), "ukst_oracle_" + name)(_dp(x), _dp(w), _dp(y), _dp(S), B, Cin, Cout, H, W,
                                                 n, P, k)
    if rc != 0:
        raise RuntimeError(f"oracle {name} failed with code {rc}")
    return y, S


def strided_naive(x, w, P, s):
    """Oracle of record for stride-s transpose convolution (Algorithm 1 with s-1 inserted zeros).
    Returns (y, S) in fp64."""
    return _call_ext("strided_naive", x, w, P, s, out_shape_strided)


def strided_segregated(x, w, P, s):
    """Check-only formulation: s*s sub-kernels selected per output pixel."""
    return _call_ext("strided_segregated", x, w, P, s, out_shape_strided)


def dilated_naive(x, w, P, d):
    """Oracle of record for dilated convolution (bed-of-nails upsampled kernel, stride-1 window
    over the input padded by P).  Returns (y, S) in fp64."""
    return _call_ext("dilated_naive", x, w, P, d, out_shape_dilated)


def dilated_segregated(x, w, P, d):
    """Check-only formulation: d*d sub-sampled input maps, each convolved with the dense kernel."""
    return _call_ext("dilated_segregated", x, w, P, d, out_shape_dilated)
