"""GPU parity: lrqmm_quantize and lrqmm_fill_sketch against the oracle, bit for bit."""
import numpy as np
import pytest

from oracle import lrqmm_oracle as o
import lrqmm_workloads as wl
from gpu_util import say, to_dev, to_np

pytestmark = pytest.mark.gpu

SHAPES = [(256, 256), (300, 517), (64, 4096), (1000, 64), (1, 1), (5, 3), (129, 1030), (576, 64)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("axis", [o.ROWWISE, o.COLWISE])
def test_quantize_bit_exact(shape, bits, axis):
    import paper_2409_18772_amd as L
    rows, cols = shape
    say("quantize", shape, bits, axis)
    X = wl.random_matrix("normal_outliers", rows, cols, seed=rows + cols + bits, outlier_frac=0.01)
    if rows > 4 and cols > 4:
        X[2, :] = 0.0          # an all-zero row
        X[:, 3] = 0.0          # an all-zero column
    for mode in (o.FLOOR, o.NEAREST):
        codes, amax = L.lrqmm_quantize(to_dev(X), axis, bits, mode)
        am_ref = o.absmax(X, axis)
        c_ref = o.quantize(X, am_ref, axis, bits, mode)
        assert np.array_equal(to_np(amax), am_ref)
        got = to_np(codes)
        if axis == o.COLWISE:
            assert got.shape == (cols, rows)
            got = got.T
        assert np.array_equal(got, c_ref)


@pytest.mark.parametrize("kind", ["uniform_pm1", "relu_normal", "exponential"])
def test_quantize_other_distributions_and_bits(kind):
    import paper_2409_18772_amd as L
    X = wl.random_matrix(kind, 192, 320, seed=7)
    for bits in (2, 3, 5, 6, 7):
        for axis in (o.ROWWISE, o.COLWISE):
            codes, amax = L.lrqmm_quantize(to_dev(X), axis, bits)
            am_ref = o.absmax(X, axis)
            got = to_np(codes)
            got = got.T if axis == o.COLWISE else got
            assert np.array_equal(to_np(amax), am_ref)
            assert np.array_equal(got, o.quantize(X, am_ref, axis, bits))


def test_quantize_large_config_shape():
    """4096 x 4096 with outliers (the headline workload's operand), both axes."""
    import paper_2409_18772_amd as L
    w = wl.CONFIGS["c3_4096_int4_r32_outliers"]
    A, B = wl.make_inputs(w)
    say("quantize 4096 A")
    codes, amax = L.lrqmm_quantize(to_dev(A), o.ROWWISE, w.bits)
    am = o.absmax(A, o.ROWWISE)
    assert np.array_equal(to_np(amax), am)
    assert np.array_equal(to_np(codes), o.quantize(A, am, o.ROWWISE, w.bits))
    say("quantize 4096 B")
    codes, amax = L.lrqmm_quantize(to_dev(B), o.COLWISE, w.bits)
    am = o.absmax(B, o.COLWISE)
    assert np.array_equal(to_np(amax), am)
    assert np.array_equal(to_np(codes).T, o.quantize(B, am, o.COLWISE, w.bits))


def test_quantize_argument_errors_and_empty():
    import torch
    import paper_2409_18772_amd as L
    lib = L.load_library()
    x = torch.zeros((4, 4), dtype=torch.float32, device="cuda")
    c = torch.zeros((4, 4), dtype=torch.int8, device="cuda")
    a = torch.zeros(4, dtype=torch.float32, device="cuda")
    args = lambda **kw: None
    assert lib.lrqmm_quantize(x.data_ptr(), 4, 4, 0, 9, 0, c.data_ptr(), a.data_ptr(), None) == -2
    assert lib.lrqmm_quantize(x.data_ptr(), 4, 4, 2, 8, 0, c.data_ptr(), a.data_ptr(), None) == -1
    assert lib.lrqmm_quantize(x.data_ptr(), 4, 4, 0, 8, 3, c.data_ptr(), a.data_ptr(), None) == -1
    assert lib.lrqmm_quantize(None, 4, 4, 0, 8, 0, c.data_ptr(), a.data_ptr(), None) == -1
    assert lib.lrqmm_quantize(x.data_ptr(), -1, 4, 0, 8, 0, c.data_ptr(), a.data_ptr(), None) == -1
    assert lib.lrqmm_quantize(None, 0, 4, 0, 8, 0, None, None, None) == 0
    with pytest.raises(L.LrqmmError):
        L.lrqmm_quantize(x, 0, 1)


@pytest.mark.parametrize("seed,stream,rows,cols", [(1234, 0, 4096, 40), (1234, 1, 4096, 40), (0, 0, 1, 1),
                                                   (2**63 + 11, 1, 577, 24), (7, 0, 64, 80)])
def test_sketch_bit_exact(seed, stream, rows, cols):
    import paper_2409_18772_amd as L
    say("sketch", seed, stream, rows, cols)
    got = to_np(L.lrqmm_fill_sketch(seed, stream, rows, cols))
    ref = o.gaussian_sketch(seed, stream, rows, cols)
    assert got.dtype == np.float32
    assert np.array_equal(got, ref)
