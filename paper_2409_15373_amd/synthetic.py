"""Seeded synthetic workloads for jagged attention (input generation only).

This module draws sequence lengths and Q/K/V/dOut values for the five benchmark
configurations.  It holds none of the attention arithmetic: it is the one piece
shared by the HIP path's tests, the CPU oracle's tests and the benchmark, so
that both sides consume bit-identical inputs.

The data stand in for the proprietary recommendation features of the paper
(Section 1: per-sample categorical histories of varying length, stored as a
jagged tensor, Section 2): a values tensor ``[sum_B, H, D]`` plus an ``int64``
offsets array ``[B+1]`` with ``offsets[0] = 0`` and ``offsets[B] = sum_B``.

All randomness comes from ``numpy.random.Generator(PCG64(seed))``; lengths are
drawn first, then q, k, v (and dout) as ``standard_normal(float32) * sigma`` in
that order.  For bf16 workloads the float32 draws are rounded to bf16 with
round-to-nearest-even and BOTH the raw bf16 bit patterns (``uint16``) and the
exactly-widened float32 values are returned.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

__all__ = [
    "Workload", "CONFIGS", "make_workload", "make_custom", "lengths_for",
    "offsets_from_lengths", "round_to_bf16_bits", "bf16_bits_to_f32",
]


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even.  No NaN inputs expected."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the float32 holding exactly the same value."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def offsets_from_lengths(lengths: np.ndarray) -> np.ndarray:
    off = np.zeros(len(lengths) + 1, dtype=np.int64)
    np.cumsum(np.asarray(lengths, dtype=np.int64), out=off[1:])
    return off


@dataclass
class Workload:
    name: str
    B: int
    H: int
    D: int
    max_len: int
    dtype: str                      # "f32" or "bf16"
    lengths: np.ndarray             # int64 [B]
    offsets: np.ndarray             # int64 [B+1]
    q: np.ndarray                   # float32 [sum_B, H, D] (bf16-representable when dtype == "bf16")
    k: np.ndarray
    v: np.ndarray
    dout: Optional[np.ndarray] = None
    bits: Dict[str, np.ndarray] = field(default_factory=dict)   # uint16 bf16 patterns per tensor name

    @property
    def sum_B(self) -> int:
        return int(self.offsets[-1])

    @property
    def S2(self) -> int:
        """Sum over samples of L_b^2 (number of (query, key) pairs per head)."""
        return int(np.sum(self.lengths.astype(np.int64) ** 2))

    def useful_flops_fwd(self) -> int:
        return 4 * self.H * self.D * self.S2

    def useful_flops_bwd(self) -> int:
        return 10 * self.H * self.D * self.S2


# name -> (B, H, D, max_len, dtype, sigma, seed, needs_dout, length recipe)
CONFIGS = {
    "c1_tiny_f32":     dict(B=4,    H=1, D=32,  max_len=64,   dtype="f32",  sigma=1.0, seed=0, dout=True,  lengths="uniform"),
    "c2_geom_bf16":    dict(B=256,  H=2, D=64,  max_len=256,  dtype="bf16", sigma=1.0, seed=1, dout=False, lengths="trunc_geom"),
    "c3_zipf_bf16":    dict(B=1024, H=4, D=128, max_len=1024, dtype="bf16", sigma=0.5, seed=2, dout=False, lengths="zipf"),
    "c4_bimodal_bf16": dict(B=512,  H=8, D=128, max_len=4096, dtype="bf16", sigma=1.0, seed=3, dout=False, lengths="bimodal"),
    "c5_uniform_bf16": dict(B=1024, H=4, D=128, max_len=1024, dtype="bf16", sigma=1.0, seed=4, dout=True,  lengths="uniform"),
}


def lengths_for(recipe: str, B: int, max_len: int, rng: np.random.Generator) -> np.ndarray:
    """Per-sample lengths, all >= 1.

    uniform     integers uniform on [1, max_len]
    trunc_geom  Geometric(p = 1/64) on {1, 2, ...}, redrawn while above max_len (true truncation)
    zipf        unbounded Zipf(a = 1.2) on {1, 2, ...}, then clipped to max_len (heavy tail piles up on max_len)
    bimodal     round(0.1 B) samples uniform on [max_len/2, max_len], the rest uniform on [1, max_len/16],
                followed by a seeded shuffle of the sample order
    """
    if recipe == "uniform":
        L = rng.integers(1, max_len + 1, size=B)
    elif recipe == "trunc_geom":
        L = rng.geometric(1.0 / 64.0, size=B)
        bad = L > max_len
        while bad.any():
            L[bad] = rng.geometric(1.0 / 64.0, size=int(bad.sum()))
            bad = L > max_len
    elif recipe == "zipf":
        L = np.minimum(rng.zipf(1.2, size=B), max_len)
    elif recipe == "bimodal":
        n_long = int(round(0.1 * B))
        long_ = rng.integers(max_len // 2, max_len + 1, size=n_long)
        short = rng.integers(1, max_len // 16 + 1, size=B - n_long)
        L = np.concatenate([long_, short])
        rng.shuffle(L)
    else:
        raise ValueError(f"unknown length recipe {recipe!r}")
    return np.asarray(L, dtype=np.int64)


_CHUNK = 1 << 20


def _draw(rng: np.random.Generator, shape, sigma: float, dtype: str):
    """N(0, sigma^2) float32 draws; for bf16 also the rounded bit patterns.  Works through the tensor in
    cache-sized chunks (the stream of draws is the same as one big call: samples are produced in order)."""
    n = int(np.prod(shape))
    x = np.empty(n, dtype=np.float32)
    bits = np.empty(n, dtype=np.uint16) if dtype == "bf16" else None
    sig = np.float32(sigma)
    for a in range(0, n, _CHUNK):
        c = x[a:a + _CHUNK]
        rng.standard_normal(size=c.shape[0], dtype=np.float32, out=c)
        if sigma != 1.0:
            c *= sig
        if bits is not None:
            u = c.view(np.uint32)
            u += ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)      # round to nearest even
            bits[a:a + _CHUNK] = u >> np.uint32(16)
            u &= np.uint32(0xFFFF0000)                                           # the bf16 value, widened
    return x.reshape(shape), (bits.reshape(shape) if bits is not None else None)


def make_custom(name: str, lengths, H: int, D: int, dtype: str = "bf16", sigma: float = 1.0,
                seed: int = 0, dout: bool = True, max_len: Optional[int] = None) -> Workload:
    """A workload with caller-chosen lengths (edge cases: zero-length samples, ragged tails, ...)."""
    lengths = np.asarray(lengths, dtype=np.int64)
    rng = np.random.Generator(np.random.PCG64(seed))
    return _fill(name, lengths, H, D, dtype, sigma, rng, dout,
                 int(max_len if max_len is not None else (lengths.max() if len(lengths) else 0)))


def _fill(name, lengths, H, D, dtype, sigma, rng, dout, max_len) -> Workload:
    offsets = offsets_from_lengths(lengths)
    shape = (int(offsets[-1]), H, D)
    bits = {}
    tensors = {}
    for t in ("q", "k", "v") + (("dout",) if dout else ()):
        s = 1.0 if t == "dout" else sigma
        tensors[t], b = _draw(rng, shape, s, dtype)
        if b is not None:
            bits[t] = b
    return Workload(name=name, B=len(lengths), H=H, D=D, max_len=max_len, dtype=dtype,
                    lengths=lengths, offsets=offsets, q=tensors["q"], k=tensors["k"], v=tensors["v"],
                    dout=tensors.get("dout"), bits=bits)


def make_workload(name: str, with_dout: Optional[bool] = None) -> Workload:
    """One of the five named configurations, fully seeded."""
    c = CONFIGS[name]
    rng = np.random.Generator(np.random.PCG64(c["seed"]))
    L = lengths_for(c["lengths"], c["B"], c["max_len"], rng)
    dout = c["dout"] if with_dout is None else with_dout
    return _fill(name, L, c["H"], c["D"], c["dtype"], c["sigma"], rng, dout, c["max_len"])
