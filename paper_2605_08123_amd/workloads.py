"""Seeded synthetic workloads shared by the tests, the smoke check and the benchmark.

This module only draws random tensors and rounds them to the storage dtype; it
holds none of the operator's arithmetic.  It is numpy-only so that the CPU
checker and the GPU path are fed the very same bytes.

The paper's own workloads are protein-pair shards that are not public and a
seed-0 synthetic BF16 tensor run (Appendix "Post-Submission Experimental
Controls"); the configurations below take their shapes and value
distributions and stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    index: int          # position in the benchmark's configuration list (seeds derive from it)
    B: int
    H: int
    L: int
    d: int
    W: int
    T: int
    R: int
    eps: float
    dtype: str          # "f32" or "bf16": storage type of Q, K, V, dO, O, dQ, dK, dV
    dustbin: bool = False
    dustbin_score: float = 0.0
    dist: str = "normal"  # "normal" | "mid" | "alphabet"

    @property
    def N(self) -> int:
        return self.B * self.H

    @property
    def edges(self) -> int:
        """Active band entries of one problem: L(2W+1) - W(W+1), W clipped to L-1."""
        w = min(self.W, self.L - 1)
        return self.L * (2 * w + 1) - w * (w + 1)

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


CONFIGS = {
    "tiny": Workload("tiny", 0, 1, 1, 256, 32, 16, 8, 2, 1.0, "f32"),
    "mid": Workload("mid", 1, 4, 8, 4096, 64, 128, 16, 2, 0.5, "bf16", dist="mid"),
    "dustbin": Workload("dustbin", 2, 2, 4, 16384, 64, 256, 20, 2, 0.5, "bf16", dustbin=True,
                        dustbin_score=0.0, dist="alphabet"),
    "long": Workload("long", 3, 1, 4, 65536, 64, 256, 20, 2, 0.5, "bf16"),
    "paper": Workload("paper", 4, 1, 2, 262144, 64, 256, 20, 2, 0.5, "bf16"),
    # the shape of the paper's own long-context run (half-band 1024, 15 base steps, one head):
    # a second benchmark point, four times the band edges per token-head
    "paper_w1024": Workload("paper_w1024", 5, 1, 1, 262144, 64, 1024, 15, 2, 0.5, "bf16"),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (uint16)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """float32 array holding values exactly representable in `dtype`."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x)).reshape(x.shape)
    raise ValueError(f"unknown dtype {dtype!r}")


def make_inputs(w: Workload, seed: int | None = None):
    """Q, K, V, dO as float32 arrays [B, H, L, d] already rounded to w.dtype.

    Draw order is Q, K, V, dO from one generator seeded with 1000*index
    (unless `seed` is given).
    """
    rng = np.random.default_rng(1000 * w.index if seed is None else seed)
    shape = (w.B, w.H, w.L, w.d)
    if w.dist == "normal":
        q, k, v, g = (rng.standard_normal(shape, dtype=np.float32) for _ in range(4))
    elif w.dist == "mid":
        # N(0, sigma^2) with sigma^2 = 1/sqrt(d) for Q and K; unit normal for V and dO.
        s = np.float32(w.d ** -0.25)
        q = rng.standard_normal(shape, dtype=np.float32) * s
        k = rng.standard_normal(shape, dtype=np.float32) * s
        v = rng.standard_normal(shape, dtype=np.float32)
        g = rng.standard_normal(shape, dtype=np.float32)
    elif w.dist == "alphabet":
        # Protein-like stand-in: token ids over a 20-letter alphabet, looked up in
        # per-head random embedding tables.
        A = 20
        x = rng.integers(0, A, size=(w.B, w.H, w.L))
        y = rng.integers(0, A, size=(w.B, w.H, w.L))
        eq, ek, ev, eg = (rng.standard_normal((w.B, w.H, A, w.d), dtype=np.float32)
                          for _ in range(4))
        take = lambda tab, ids: np.take_along_axis(tab, ids[..., None], axis=2)
        q, k, v, g = take(eq, x), take(ek, y), take(ev, y), take(eg, x)
    else:
        raise ValueError(w.dist)
    return tuple(round_to_dtype(t, w.dtype) for t in (q, k, v, g))
