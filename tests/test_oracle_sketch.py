"""Pins for the oracle's counter-based Gaussian sketch (no GPU)."""
import math

import numpy as np
from scipy import stats

from oracle import lrqmm_oracle as o


def test_elementary_functions_against_libm():
    k = np.concatenate([np.arange(1, 5000), np.arange(1, 2**24 + 1, 4099), [2**24]])
    ref = np.array([math.log(int(v) / 2.0**24) for v in k])
    assert np.max(np.abs(o._det_log(k) - ref)) < 4e-15
    assert o._det_log(np.array([2**24]))[0] == 0.0
    x = np.linspace(0.0, math.pi / 4, 20001)
    s, c = o._det_sincos(x)
    assert np.max(np.abs(s - np.sin(x))) < 3e-16
    assert np.max(np.abs(c - np.cos(x))) < 3e-16
    v = np.concatenate([[0.0], np.geomspace(1e-8, 40.0, 5001)])
    assert np.max(np.abs(o._det_sqrt(v) - np.sqrt(v)) / np.maximum(np.sqrt(v), 1e-300)) < 3e-16
    assert o._det_sqrt(np.array([0.0]))[0] == 0.0


def test_mix64_known_sequence():
    # splitmix64 seeded with 0: first outputs of the published generator
    z = np.array([0], dtype=np.uint64)
    out = []
    state = np.uint64(0)
    for _ in range(3):
        out.append(int(o._mix64(np.array([state], dtype=np.uint64))[0]))
        with np.errstate(over="ignore"):
            state = state + o._GOLD
    assert out == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_octant_reduction_equals_direct_cosine():
    # drive the sketch's cosine branch directly: all octants, boundaries included
    k2 = np.concatenate([np.arange(0, 2**24, 65521), np.arange(8) << 21, (np.arange(8) << 21) + 1,
                         ((np.arange(8) + 1) << 21) - 1]).astype(np.int64)
    octant = k2 >> 21
    rem = k2 & ((1 << 21) - 1)
    odd = (octant & 1) == 1
    r = np.where(odd, (1 << 21) - rem, rem).astype(np.float64)
    sn, cs = o._det_sincos(o._TWO_PI * (r / 16777216.0))
    use_sin = (octant == 1) | (octant == 2) | (octant == 5) | (octant == 6)
    neg = (octant >= 2) & (octant <= 5)
    t = np.where(neg, -1.0, 1.0) * np.where(use_sin, sn, cs)
    assert np.max(np.abs(t - np.cos(2 * np.pi * k2 / 2.0**24))) < 1e-15


def test_moments_and_distribution():
    om = o.gaussian_sketch(1234, 0, 4096, 40).astype(np.float64)
    assert om.shape == (4096, 40)
    n = om.size
    assert abs(om.mean()) < 4 / math.sqrt(n)
    assert abs(om.var() - 1.0) < 4 * math.sqrt(2.0 / n)
    assert abs(stats.kurtosis(om.ravel())) < 0.05
    assert stats.kstest(om.ravel(), "norm").pvalue > 1e-3
    # columns and rows are uncorrelated
    g = om.T @ om / om.shape[0]
    assert np.max(np.abs(g - np.eye(40))) < 0.1
    lag = np.mean(om[:-1] * om[1:])
    assert abs(lag) < 4 / math.sqrt(n)


def test_counter_based_and_streams_independent():
    a = o.gaussian_sketch(7, 0, 64, 16)
    assert a.dtype == np.float32
    assert np.array_equal(a, o.gaussian_sketch(7, 0, 64, 16))
    # a sub-block is the same numbers: element (i,j) depends only on (seed, stream, i, j)
    assert np.array_equal(a[:10, :5], o.gaussian_sketch(7, 0, 10, 5))
    b = o.gaussian_sketch(7, 1, 64, 16)
    c = o.gaussian_sketch(8, 0, 64, 16)
    for other in (b, c):
        assert not np.array_equal(a, other)
        r = np.corrcoef(a.ravel(), other.ravel())[0, 1]
        assert abs(r) < 0.15
    assert np.all(np.isfinite(o.gaussian_sketch(2**63 + 5, 1, 33, 7)))
