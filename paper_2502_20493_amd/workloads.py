"""Seeded synthetic workloads shared by the tests, the smoke check and the benchmark.

This module only draws random numbers and names shapes.  It holds none of the method's
arithmetic (no output-size formula, no sub-kernel logic), so that the CPU oracle and the HIP
library can both be fed from it without sharing anything else.

Shapes and value laws stand in for the paper's workloads: 224x224x3 images (Sec. 4.1,
Tables 1-3) and the GAN generator layers of the ablation (Sec. 4.3, Table 4), plus odd-output
stress cases (the situation Sec. 1 and Sec. 3.2 are about).  All data is synthetic.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

SEED_BASE = 20493 * 10


@dataclass(frozen=True)
class Workload:
    name: str
    index: int          # seed offset
    B: int
    Cin: int
    Cout: int
    H: int
    W: int
    n: int
    P: int
    dtype: str          # "f32" or "bf16" (bf16 inputs, fp32 output)
    x_law: str          # "uniform_pm1" | "uniform01" | "relu_normal" | "normal" | "int3"
    w_law: str          # "uniform_pm1" | "normal:<sigma>" | "int3"
    stands_for: str = ""

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    w.name: w
    for w in [
        Workload("cfg1", 10, 1, 1, 1, 32, 32, 3, 0, "f32", "uniform_pm1", "uniform_pm1",
                 "single feature map toy case, odd 61x61 output"),
        Workload("cfg1_int", 11, 1, 1, 1, 32, 32, 3, 0, "f32", "int3", "int3",
                 "integer-valued copy of cfg1 for exact checking"),
        Workload("cfg2a", 20, 16, 3, 3, 224, 224, 3, 0, "f32", "uniform01", "normal:0.1",
                 "224x224x3 dataset images, n=3, odd 445x445 output"),
        Workload("cfg2b", 21, 16, 3, 3, 224, 224, 4, 2, "f32", "uniform01", "normal:0.1",
                 "224x224x3 dataset images, n=4, P=2, 448x448 output"),
        Workload("cfg3_L1", 30, 64, 512, 256, 4, 4, 4, 2, "f32", "relu_normal", "normal:0.02",
                 "DCGAN-style generator layer 4->8"),
        Workload("cfg3_L2", 31, 64, 256, 128, 8, 8, 4, 2, "f32", "relu_normal", "normal:0.02",
                 "DCGAN-style generator layer 8->16"),
        Workload("cfg3_L3", 32, 64, 128, 64, 16, 16, 4, 2, "f32", "relu_normal", "normal:0.02",
                 "DCGAN-style generator layer 16->32"),
        Workload("cfg3_L4", 33, 64, 64, 3, 32, 32, 4, 2, "f32", "relu_normal", "normal:0.02",
                 "DCGAN-style generator layer 32->64, RGB out"),
        Workload("cfg4a", 40, 32, 128, 128, 64, 64, 5, 0, "f32", "normal", "normal:0.05",
                 "odd-output stress, n=5, 123x123"),
        Workload("cfg4b", 41, 32, 128, 128, 63, 63, 3, 0, "f32", "normal", "normal:0.05",
                 "odd-output stress, n=3, odd input 63, 123x123"),
        Workload("cfg5a", 50, 32, 256, 128, 128, 128, 4, 2, "bf16", "relu_normal",
                 "normal:0.02", "wide-channel GAN layer, bf16 in / fp32 accumulate"),
        Workload("cfg5b", 51, 64, 1024, 512, 16, 16, 4, 2, "bf16", "relu_normal",
                 "normal:0.02", "wide-channel GAN layer, bf16 in / fp32 accumulate"),
    ]
}


def round_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even.  Finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _draw(rng: np.random.Generator, law: str, shape) -> np.ndarray:
    if law == "uniform_pm1":
        return (rng.random(shape, dtype=np.float32) * np.float32(2.0) - np.float32(1.0))
    if law == "uniform01":
        return rng.random(shape, dtype=np.float32)
    if law == "normal":
        return rng.standard_normal(shape, dtype=np.float32)
    if law == "relu_normal":
        a = rng.standard_normal(shape, dtype=np.float32)
        np.maximum(a, np.float32(0.0), out=a)
        return a
    if law == "int3":
        return rng.integers(-3, 4, size=shape).astype(np.float32)
    if law.startswith("normal:"):
        sigma = np.float32(float(law.split(":")[1]))
        return rng.standard_normal(shape, dtype=np.float32) * sigma
    raise ValueError(f"unknown law {law}")


def generate(wl: Workload, integer: bool = False):
    """Return a dict with host arrays for ``wl``.

    ``x``/``w``: float32 arrays holding exactly the values both sides consume (for bf16
    workloads they are already rounded to bf16).  ``x_bits``/``w_bits``: uint16 bf16 patterns
    (bf16 workloads only).  ``integer=True`` swaps both laws for integers in {-3..3}, which are
    exact in fp32 and bf16.
    """
    x_law, w_law = ("int3", "int3") if integer else (wl.x_law, wl.w_law)
    rx = np.random.Generator(np.random.PCG64(SEED_BASE + wl.index))
    rw = np.random.Generator(np.random.PCG64(SEED_BASE + wl.index + 1000))
    x = _draw(rx, x_law, (wl.B, wl.Cin, wl.H, wl.W))
    w = _draw(rw, w_law, (wl.Cout, wl.Cin, wl.n, wl.n))
    out = {"x": x, "w": w}
    if wl.dtype == "bf16":
        xb, wb = round_to_bf16_bits(x), round_to_bf16_bits(w)
        out.update(x=bf16_bits_to_f32(xb), w=bf16_bits_to_f32(wb), x_bits=xb, w_bits=wb)
    return out


def generate_dy(wl: Workload, out_hw, integer: bool = False):
    """Upstream gradient for the backward pass of ``wl``: N(0,1) (or integers in {-3..3}) of shape
    [B, Cout, *out_hw]; the caller supplies the output size.  Returns {"dy": float32 array holding
    the values both sides consume, "dy_bits": bf16 patterns for bf16 workloads}."""
    rd = np.random.Generator(np.random.PCG64(SEED_BASE + wl.index + 2000))
    dy = _draw(rd, "int3" if integer else "normal", (wl.B, wl.Cout, int(out_hw[0]), int(out_hw[1])))
    out = {"dy": dy}
    if wl.dtype == "bf16":
        db = round_to_bf16_bits(dy)
        out.update(dy=bf16_bits_to_f32(db), dy_bits=db)
    return out
