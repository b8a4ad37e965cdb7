"""Seeded synthetic inputs for the LRQMM hot path.

This module only draws input matrices; it holds none of the method's arithmetic
(no quantizer, no sketch, no SVD).  Both the CPU oracle's tests and the GPU
path's tests/benchmark take their inputs from here so the two sides see the
same arrays.

The matrices stand in for the paper's evaluation inputs: the random matrices of
its precision tests (Evaluation, "Differential distribution", Tables 3-4: Normal,
Uniform, Exponent, ChiSquare, Poisson) and an im2col'd ResNet-50 convolution
(Evaluation, "Image recognition").  No dataset or trained weight is used.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class Workload:
    name: str
    M: int
    N: int
    K: int
    bits: int
    rank: int
    oversample: int
    power_iters: int
    sketch_seed: int = 1234
    seed_a: int = 0
    seed_b: int = 1
    kind: str = "normal"
    extra: dict = field(default_factory=dict)

    @property
    def ell(self) -> int:
        return self.rank + self.oversample


def _draw(kind: str, rng: np.random.Generator, shape, extra) -> np.ndarray:
    if kind == "uniform_pm1":
        x = rng.uniform(-1.0, 1.0, size=shape)
    elif kind == "uniform01":
        x = rng.uniform(0.0, 1.0, size=shape)
    elif kind == "normal":
        x = rng.standard_normal(size=shape)
    elif kind == "normal_outliers":
        x = rng.standard_normal(size=shape)
        mask = rng.random(size=shape) < extra.get("outlier_frac", 1e-3)
        out = rng.standard_normal(size=shape) * extra.get("outlier_sigma", 20.0)
        x = np.where(mask, out, x)
    elif kind == "exponential":
        x = rng.exponential(scale=extra.get("scale", 4.0), size=shape)
    elif kind == "chisquare":
        x = rng.chisquare(df=extra.get("df", 1.0), size=shape)
    elif kind == "poisson":
        x = rng.poisson(lam=extra.get("lam", 10.0), size=shape).astype(np.float64)
    elif kind == "relu_normal":
        x = np.maximum(rng.standard_normal(size=shape), 0.0)
    elif kind == "he_normal":
        x = rng.standard_normal(size=shape) * np.sqrt(2.0 / extra["fan_in"])
    else:
        raise ValueError(f"unknown kind {kind!r}")
    return np.ascontiguousarray(x, dtype=np.float32)


def make_inputs(w: Workload):
    """Return (A, B) as C-contiguous float32 arrays of shapes (M,K) and (K,N)."""
    ra = np.random.default_rng(w.seed_a)
    rb = np.random.default_rng(w.seed_b)
    kind_a = w.extra.get("kind_a", w.kind)
    kind_b = w.extra.get("kind_b", w.kind)
    A = _draw(kind_a, ra, (w.M, w.K), w.extra)
    B = _draw(kind_b, rb, (w.K, w.N), w.extra)
    return A, B


def random_matrix(kind: str, rows: int, cols: int, seed: int, **extra) -> np.ndarray:
    return _draw(kind, np.random.default_rng(seed), (rows, cols), extra)


def low_rank_matrix(rows: int, cols: int, rank: int, seed: int) -> np.ndarray:
    """Exactly rank-`rank` float64 matrix with well separated singular values."""
    rng = np.random.default_rng(seed)
    L = rng.standard_normal((rows, rank))
    R = rng.standard_normal((rank, cols))
    d = 2.0 ** (-np.arange(rank, dtype=np.float64))
    return (L * d) @ R


# The five benchmark configurations (shapes, value distributions, quantizer and
# RSVD parameters).  Where a configuration leaves oversampling / power
# iterations unstated they are 0 (the range finder then has exactly r columns,
# as in the paper's Algorithm 1).
CONFIGS = {
    "c1_256_int8_r8": Workload("c1_256_int8_r8", 256, 256, 256, 8, 8, 0, 0,
                               kind="uniform_pm1", seed_a=0, seed_b=1),
    "c2_4096_int8_r16": Workload("c2_4096_int8_r16", 4096, 4096, 4096, 8, 16, 8, 1,
                                 kind="normal"),
    "c3_4096_int4_r32_outliers": Workload("c3_4096_int4_r32_outliers", 4096, 4096, 4096,
                                          4, 32, 8, 1, kind="normal_outliers",
                                          extra={"outlier_frac": 1e-3, "outlier_sigma": 20.0}),
    "c4_16384_int4_r64": Workload("c4_16384_int4_r64", 16384, 16384, 16384, 4, 64, 16, 2,
                                  kind="normal"),
    "c5_resnet50_conv_int4_r8": Workload("c5_resnet50_conv_int4_r8", 100352, 64, 576, 4, 8, 0, 0,
                                         kind="relu_normal",
                                         extra={"kind_a": "relu_normal", "kind_b": "he_normal",
                                                "fan_in": 576}),
}


def scaled_config(name: str, M: int, N: int, K: int) -> Workload:
    """Same distribution / quantizer / RSVD parameters as CONFIGS[name] at another shape."""
    w = CONFIGS[name]
    return Workload(f"{name}@{M}x{N}x{K}", M, N, K, w.bits, w.rank, w.oversample,
                    w.power_iters, w.sketch_seed, w.seed_a, w.seed_b, w.kind, dict(w.extra))
