"""Seeded synthetic inputs for the five benchmark workloads.

This module holds no convolution arithmetic: it only draws the random arrays
that both the GPU path and the CPU oracle are fed.  The paper (Section 6)
states no value distribution and uses no public data set -- it launches
repeated synthetic convolutions -- so uniform fp32 data of the workloads'
shapes stand in.

Recipe: ``numpy.random.default_rng(seed)``; the signal / image is the first
draw, the taps the second, both ``uniform(lo, hi)`` in float64 rounded to
float32.  Seeds are 15884 (the arXiv number's tail) followed by the workload
number.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    ndim: int                      # 1 or 2
    x_shape: Tuple[int, ...]       # (n,) or (h, w)
    k_shape: Tuple[int, ...]       # (k,) or (kh, kw)
    x_range: Tuple[float, float]
    w_range: Tuple[float, float]
    seed: int

    @property
    def y_shape(self) -> Tuple[int, ...]:
        return tuple(a - b + 1 for a, b in zip(self.x_shape, self.k_shape))

    @property
    def n_outputs(self) -> int:
        return int(np.prod(self.y_shape, dtype=np.int64))

    @property
    def n_taps(self) -> int:
        """Multiply-adds of the definition: outputs x filter size."""
        return self.n_outputs * int(np.prod(self.k_shape, dtype=np.int64))

    @property
    def algorithmic_bytes(self) -> int:
        """Every input read once, every output written once, taps once (fp32)."""
        n_in = int(np.prod(self.x_shape, dtype=np.int64))
        n_w = int(np.prod(self.k_shape, dtype=np.int64))
        return 4 * (n_in + self.n_outputs + n_w)


WORKLOADS = {
    "conv1d_64k_k5": Workload("conv1d_64k_k5", 1, (65536,), (5,), (-1.0, 1.0), (-1.0, 1.0), 158841),
    "conv1d_64m_k16": Workload("conv1d_64m_k16", 1, (1 << 26,), (16,), (-1.0, 1.0), (-1.0, 1.0), 158842),
    "conv2d_1k_3x3": Workload("conv2d_1k_3x3", 2, (1024, 1024), (3, 3), (0.0, 1.0), (-1.0, 1.0), 158843),
    "conv2d_4k_5x5": Workload("conv2d_4k_5x5", 2, (4096, 4096), (5, 5), (0.0, 1.0), (-1.0, 1.0), 158844),
    "conv2d_8k_11x11": Workload("conv2d_8k_11x11", 2, (8192, 8192), (11, 11), (0.0, 1.0), (-1.0, 1.0), 158845),
}

ORDER = ["conv1d_64k_k5", "conv1d_64m_k16", "conv2d_1k_3x3", "conv2d_4k_5x5", "conv2d_8k_11x11"]


def uniform_f32(rng: np.random.Generator, lo: float, hi: float, shape) -> np.ndarray:
    return rng.uniform(lo, hi, size=shape).astype(np.float32)


def make(workload: Workload, x_shape: Optional[Tuple[int, ...]] = None):
    """Return (x, taps) for a workload; ``x_shape`` overrides the signal size
    (same seed, same distributions) for bounded samples of a big workload."""
    rng = np.random.default_rng(workload.seed)
    shape = workload.x_shape if x_shape is None else tuple(x_shape)
    x = uniform_f32(rng, *workload.x_range, shape)
    w = uniform_f32(rng, *workload.w_range, workload.k_shape)
    return x, w


def make_separable(workload: Workload):
    """2-D workload whose filter is an outer product u v^T of two random tap vectors."""
    assert workload.ndim == 2
    rng = np.random.default_rng(workload.seed + 1000)
    x = uniform_f32(rng, *workload.x_range, workload.x_shape)
    u = uniform_f32(rng, *workload.w_range, (workload.k_shape[0],))
    v = uniform_f32(rng, *workload.w_range, (workload.k_shape[1],))
    return x, u, v


def random_case(seed: int, x_shape, k_shape, x_range=(-1.0, 1.0), w_range=(-1.0, 1.0)):
    """Free-form seeded case for edge-shape tests."""
    rng = np.random.default_rng(seed)
    return uniform_f32(rng, *x_range, tuple(x_shape)), uniform_f32(rng, *w_range, tuple(k_shape))


def integer_case(seed: int, x_shape, k_shape, x_max: int = 15, w_max: int = 7):
    """Small-integer data: every fp32 product and partial sum is exact (|sum| < 2^24),
    so any summation order gives the same bits."""
    rng = np.random.default_rng(seed)
    x = rng.integers(-x_max, x_max + 1, size=tuple(x_shape)).astype(np.float32)
    w = rng.integers(-w_max, w_max + 1, size=tuple(k_shape)).astype(np.float32)
    return x, w
