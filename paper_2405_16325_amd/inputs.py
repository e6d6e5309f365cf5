"""Seeded synthetic inputs for the double-pruned 2:4 sparse linear layer.

This module only draws numbers and rounds them to bf16.  It holds none of the
method's arithmetic (no pruning, packing or products), so both the HIP path's
tests and the CPU oracle's tests may take their operands from here.

bf16 tensors are carried on the host as ``numpy.uint16`` bit patterns.
Distributions follow the OPT-shaped layer recipe: activations X ~ N(0, 1),
weights W ~ N(0, 0.02), output gradients dY ~ N(0, 1e-3), adapter factors
L, R ~ N(0, 0.02).
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 0x5105E

# (d_out, d_in) of the linear layers of one transformer block, per model shape.
LAYER_SETS = {
    "opt125m_fc1": {"b": 2048, "layers": [("fc1", 3072, 768)], "rank": 0},
    "opt2.7b": {"b": 16384, "rank": 0,
                "layers": [("q", 2560, 2560), ("k", 2560, 2560), ("v", 2560, 2560),
                           ("o", 2560, 2560), ("fc1", 10240, 2560), ("fc2", 2560, 10240)]},
    "opt13b": {"b": 16384, "rank": 64,
               "layers": [("q", 5120, 5120), ("k", 5120, 5120), ("v", 5120, 5120),
                          ("o", 5120, 5120), ("fc1", 20480, 5120), ("fc2", 5120, 20480)]},
    "opt66b": {"b": 16384, "rank": 128,
               "layers": [("q", 9216, 9216), ("k", 9216, 9216), ("v", 9216, 9216),
                          ("o", 9216, 9216), ("fc1", 36864, 9216), ("fc2", 9216, 36864)]},
}

STD = {"X": 1.0, "W": 0.02, "dY": 1e-3, "L": 0.02, "R": 0.02}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round to nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = (u + (0x7FFF + ((u >> 16) & 1))) >> 16
    r = np.where(nan, (u >> 16) | 0x0040, r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[SEED_BASE + seed, stream]))


def gaussian_bf16(shape, std: float, seed: int, stream: int) -> np.ndarray:
    """N(0, std) drawn in fp32 from a counter-based generator, rounded to bf16 bits."""
    g = _rng(seed, stream).standard_normal(size=shape, dtype=np.float32) * np.float32(std)
    return f32_to_bf16_bits(g)


def layer_inputs(b: int, d_out: int, d_in: int, rank: int = 0, seed: int = 0) -> dict:
    """Operands of one linear layer: X[b,d_in], W[d_out,d_in], dY[b,d_out], L[d_in,r], R[r,d_out]."""
    out = {
        "X": gaussian_bf16((b, d_in), STD["X"], seed, 1),
        "W": gaussian_bf16((d_out, d_in), STD["W"], seed, 2),
        "dY": gaussian_bf16((b, d_out), STD["dY"], seed, 3),
    }
    if rank > 0:
        out["L"] = gaussian_bf16((d_in, rank), STD["L"], seed, 4)
        out["R"] = gaussian_bf16((rank, d_out), STD["R"], seed, 5)
    return out


def coarse_weights(d_out: int, d_in: int, seed: int, levels: int = 5) -> np.ndarray:
    """Weights drawn from a handful of magnitudes (zeros included) so that ties inside
    a group of four are the rule, not the exception.  Returns bf16 bits."""
    g = _rng(seed, 9)
    mag = g.integers(0, levels, size=(d_out, d_in)).astype(np.float32) * np.float32(0.25)
    sign = np.where(g.integers(0, 2, size=(d_out, d_in)) == 1, np.float32(-1), np.float32(1))
    return f32_to_bf16_bits(mag * sign)
