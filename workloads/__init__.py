"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path's tests/bench.

This module holds none of the method's arithmetic: it only draws matrices.  The shapes and the
outlier structure stand in for the OPT / LLaMA activations the paper measures on (a few input
channels whose magnitude is at least 20x that of the rest -- Background section and Appendix A);
those models and datasets are not available, so nothing here reproduces them.

Recipe (identical for every consumer): ``numpy.random.Generator(PCG64(seed))``; draw the
entries in float32; pick the outlier channels with ``rng.choice(I, n, replace=False)``; multiply
each outlier channel by its scale; clip to the finite float16 range; cast to float16.
Weights use an independent stream ``PCG64(seed + 1000)`` and N(0, std=0.02).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

F16_MAX = 65504.0


@dataclass(frozen=True)
class Config:
    name: str
    T: int            # tokens (rows of X)
    I: int            # input channels (columns of X, rows of W)
    O: int            # output channels (columns of W)
    dist: str         # "normal" or "student_t3"
    n_outlier: int    # number of outlier channels
    scale_lo: float   # outlier scale: fixed if lo == hi, else U[lo, hi] per channel
    scale_hi: float
    bits: int
    alphas: tuple
    seed: int
    label: str


CONFIGS = {
    "C1": Config("C1", 64, 256, 256, "normal", 4, 60.0, 60.0, 8, (0.15,), 1,
                 "Tiny 64x256, 4 outlier channels x60"),
    "C2": Config("C2", 2048, 4096, 11008, "normal", 20, 50.0, 100.0, 8, (0.15,), 2,
                 "LLaMA-7B-shaped layer 2048x4096 . 4096x11008"),
    "C3": Config("C3", 4096, 5120, 20480, "student_t3", 10, 80.0, 80.0, 8, (0.0, 0.15, 0.5, 1.0), 3,
                 "OPT-13B-shaped layer 4096x5120 . 5120x20480, heavy-tailed"),
    "C4": Config("C4", 4096, 4096, 4096, "normal", 20, 50.0, 100.0, 4, (0.15,), 4,
                 "Low-bit 4096x4096, INT4 packed"),
    "C5": Config("C5", 4096, 8192, 28672, "normal", 41, 100.0, 100.0, 8, (0.15,), 5,
                 "LLaMA-70B-shaped MLP up-proj 4096x8192 . 8192x28672"),
}


def activation(T: int, I: int, *, dist: str = "normal", n_outlier: int = 0, scale_lo: float = 1.0,
               scale_hi: float = 1.0, seed: int = 0) -> np.ndarray:
    """A T x I float16 activation matrix with ``n_outlier`` scaled channels."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if dist == "normal":
        x = rng.standard_normal((T, I), dtype=np.float32)
    elif dist == "student_t3":
        x = rng.standard_t(3.0, size=(T, I)).astype(np.float32)
    else:
        raise ValueError("unknown distribution %r" % dist)
    if n_outlier:
        cols = rng.choice(I, n_outlier, replace=False)
        if scale_lo == scale_hi:
            sc = np.full(n_outlier, scale_lo, np.float32)
        else:
            sc = rng.uniform(scale_lo, scale_hi, n_outlier).astype(np.float32)
        x[:, cols] *= sc[None, :]
    np.clip(x, -F16_MAX, F16_MAX, out=x)
    return x.astype(np.float16)


def weight(I: int, O: int, *, seed: int = 0, std: float = 0.02) -> np.ndarray:
    """An I x O float16 weight matrix, N(0, std), drawn in row blocks to bound host memory."""
    rng = np.random.Generator(np.random.PCG64(seed + 1000))
    w = np.empty((I, O), np.float16)
    step = max(1, (1 << 24) // max(O, 1))
    for r0 in range(0, I, step):
        r1 = min(I, r0 + step)
        blk = rng.standard_normal((r1 - r0, O), dtype=np.float32)
        blk *= np.float32(std)
        w[r0:r1] = blk.astype(np.float16)
    return w


def config_activation(name: str) -> np.ndarray:
    c = CONFIGS[name]
    return activation(c.T, c.I, dist=c.dist, n_outlier=c.n_outlier, scale_lo=c.scale_lo,
                      scale_hi=c.scale_hi, seed=c.seed)


def config_weight(name: str) -> np.ndarray:
    c = CONFIGS[name]
    return weight(c.I, c.O, seed=c.seed)


def int8_codes(rows: int, cols: int, *, seed: int = 0, lo: int = -127, hi: int = 127) -> np.ndarray:
    """Uniform integer codes in [lo, hi], for exercising the integer GEMM alone."""
    rng = np.random.Generator(np.random.PCG64(seed + 2000))
    return rng.integers(lo, hi + 1, size=(rows, cols), dtype=np.int8)
