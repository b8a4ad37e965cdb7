"""Pins for the oracle's quantizer and integer GEMM (no GPU).

Checked against: a hand-worked example (tests/golden/quantize_worked_example.txt),
exact rational arithmetic, the interval the floor residual must lie in
(Methodology, Eq. (get_ra2)), and a python big-integer triple loop for the
integer product (Background 2.2, Eq. (INTGEMM)).
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import lrqmm_oracle as o
import lrqmm_workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "quantize_worked_example.txt")


def _golden_cases():
    cases = []
    with open(GOLD) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            bits, mode, vals, codes = [p.strip() for p in line.split(";")]
            cases.append((int(bits), mode, [float(v) for v in vals.split()],
                          [int(c) for c in codes.split()]))
    return cases


@pytest.mark.parametrize("bits,mode,vals,codes", _golden_cases())
def test_worked_example_rows_and_columns(bits, mode, vals, codes):
    rm = o.FLOOR if mode == "floor" else o.NEAREST
    X = np.array([vals], dtype=np.float32)
    got = o.quantize(X, o.absmax(X, o.ROWWISE), o.ROWWISE, bits, rm)
    assert got.dtype == np.int8 and got.tolist() == [codes]
    Xc = X.T.copy()
    got_c = o.quantize(Xc, o.absmax(Xc, o.COLWISE), o.COLWISE, bits, rm)
    assert got_c.ravel().tolist() == codes
    got_t = o.quantize(X, o.absmax(X, o.TENSOR), o.TENSOR, bits, rm)
    assert got_t.tolist() == [codes]


def test_scale_groups_are_independent():
    # two rows with different maxima: each row is scaled by its own lambda
    X = np.array([[1.0, -0.5, 0.25], [100.0, 50.0, -25.0]], dtype=np.float32)
    got = o.quantize(X, o.absmax(X, o.ROWWISE), o.ROWWISE, 4)
    assert got.tolist() == [[7, -4, 1], [7, 3, -2]]
    # per column the same data gives different codes
    got_c = o.quantize(X, o.absmax(X, o.COLWISE), o.COLWISE, 4)
    assert got_c.tolist() == [[0, -1, 0], [7, 7, -7]]


@pytest.mark.parametrize("bits", [2, 3, 4, 5, 8])
@pytest.mark.parametrize("kind", ["normal", "uniform_pm1", "exponential"])
def test_floor_codes_match_exact_rational_floor(bits, kind):
    """code == floor(fl32(lambda) * x) evaluated exactly, when the single rounding of
    the product cannot cross an integer (checked per element, rest skipped)."""
    X = wl.random_matrix(kind, 7, 33, seed=bits)
    amax = o.absmax(X, o.ROWWISE)
    lam, s = o.scales(amax, bits)
    q = o.qmax_of(bits)
    codes = o.quantize(X, amax, o.ROWWISE, bits)
    n_checked = 0
    for i in range(X.shape[0]):
        lam_exact = Fraction(float(lam[i]))
        assert abs(lam_exact - Fraction(q) / Fraction(float(amax[i]))) <= Fraction(q, 1 << 23) / Fraction(float(amax[i]))
        for k in range(X.shape[1]):
            t = lam_exact * Fraction(float(X[i, k]))
            fl = t.numerator // t.denominator
            frac = t - fl
            # skip elements within one ulp-ish of an integer boundary
            if frac < Fraction(1, 1 << 16) or frac > 1 - Fraction(1, 1 << 16):
                continue
            assert codes[i, k] == max(-q - 1, min(q, fl))
            n_checked += 1
    assert n_checked > 200


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("axis", [o.ROWWISE, o.COLWISE, o.TENSOR])
def test_floor_residual_interval_and_code_range(bits, axis):
    X = wl.random_matrix("normal_outliers", 64, 96, seed=3, outlier_frac=0.01)
    amax = o.absmax(X, axis)
    lam, s = o.scales(amax, bits)
    q = o.qmax_of(bits)
    codes = o.quantize(X, amax, axis, bits)
    assert codes.min() >= -q - 1 and codes.max() <= q
    R = o.residual(X, codes, s, axis)
    S = np.broadcast_to(o._broadcast(s.astype(np.float64), axis, X.shape), X.shape)
    eps = 4 * q * 2.0 ** -24          # relative rounding of lambda, s and lambda*x
    assert np.all(R >= -S * eps)
    assert np.all(R < S * (1 + eps))
    # the largest |x| of each group maps to +-qmax (or one below after floor)
    if axis == o.ROWWISE:
        top = np.abs(codes.astype(int)).max(axis=1)
        assert np.all((top >= q - 1) & (top <= q + 1))
    # mean residual is about s/2 with floor (the method's key property), 0 with nearest
    assert abs((R / S).mean() - 0.5) < 0.05
    codes_n = o.quantize(X, amax, axis, bits, o.NEAREST)
    Rn = o.residual(X, codes_n, s, axis)
    inside = np.abs(codes_n.astype(int)) < q        # not clamped
    assert np.all(np.abs(Rn[inside]) <= 0.5 * S[inside] * (1 + 2 * eps))


def test_zero_and_tiny_groups():
    X = np.zeros((3, 5), dtype=np.float32)
    X[1] = [1e-35, -1e-36, 0, 0, 0]
    X[2] = [1.0, 0, 0, 0, -2.0]
    amax = o.absmax(X, o.ROWWISE)
    lam, s = o.scales(amax, 8)
    assert lam[0] == 0 and s[0] == 0 and lam[1] == 0 and s[1] == 0
    codes = o.quantize(X, amax, o.ROWWISE, 8)
    assert not codes[:2].any()
    assert codes[2].tolist() == [63, 0, 0, 0, -127]
    R = o.residual(X, codes, s, o.ROWWISE)
    assert np.array_equal(R[:2], X[:2].astype(np.float64))


def test_rejects_non_finite_and_bad_bits():
    X = np.array([[1.0, np.inf]], dtype=np.float32)
    with pytest.raises(ValueError):
        o.absmax(X, o.ROWWISE)
    with pytest.raises(ValueError):
        o.qmax_of(1)
    with pytest.raises(ValueError):
        o.qmax_of(9)


def test_int_gemm_matches_python_bigint_loop():
    rng = np.random.default_rng(5)
    Aq = rng.integers(-128, 128, size=(5, 9), dtype=np.int8)
    Bq = rng.integers(-128, 128, size=(9, 4), dtype=np.int8)
    C = o.int_gemm(Aq, Bq)
    assert C.dtype == np.int64
    for i in range(5):
        for j in range(4):
            acc = 0
            for k in range(9):
                acc += int(Aq[i, k]) * int(Bq[k, j])
            assert int(C[i, j]) == acc


def test_int_gemm_extremes_and_structure():
    K = 1000
    Aq = np.full((2, K), -128, dtype=np.int8)
    Bq = np.full((K, 3), -128, dtype=np.int8)
    assert np.all(o.int_gemm(Aq, Bq) == 128 * 128 * K)       # int8 would overflow, int64 does not
    P = np.eye(6, dtype=np.int8)[[3, 0, 5, 1, 2, 4]]
    Bq = np.arange(-18, 18, dtype=np.int8).reshape(6, 6)
    assert np.array_equal(o.int_gemm(P, Bq), Bq[[3, 0, 5, 1, 2, 4]].astype(np.int64))
    # not symmetric in its arguments: a transposed operand is detected
    Aq = np.arange(12, dtype=np.int8).reshape(3, 4)
    Bq = np.arange(8, dtype=np.int8).reshape(4, 2)
    assert o.int_gemm(Aq, Bq).tolist() == [[28, 34], [76, 98], [124, 162]]
    with pytest.raises(OverflowError):
        o.int_gemm(np.full((1, 140000), -128, np.int8), np.full((140000, 1), -128, np.int8))


def test_dequant_is_per_row_times_per_column():
    Cint = np.array([[2, -4], [6, 8]], dtype=np.int64)
    sA = np.array([0.5, 0.25], dtype=np.float32)
    sB = np.array([2.0, 4.0], dtype=np.float32)
    assert o.dequant(Cint, sA, sB).tolist() == [[2.0, -8.0], [3.0, 8.0]]
