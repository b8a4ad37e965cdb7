"""GPU parity of the complete-residual-compensation baseline (Eq. (gemm_r_split); QT(1,1,0) and
QT(1,1,1) in the Evaluation) against the oracle.

Second-level codes and maxima are bit-exact.  The product is a sum of up to four dequantized integer
GEMMs; each term is exact in int32 and picks up two float32 roundings in its dequantization, one in the
alpha product and one per accumulation into D, so
    |got - want|_F <= 6 * 2^-24 * |alpha| * sum_i |T_i|_F  +  3 * 2^-24 * |beta| * |D|_F.
"""
import numpy as np
import pytest

from oracle import lrqmm_oracle as o
import lrqmm_workloads as wl
from gpu_util import say, to_dev, to_np
from test_gpu_update_strides import window, SENTINEL

pytestmark = pytest.mark.gpu


def bound(ref, alpha=1.0, beta=0.0, D0=None):
    t = sum(np.linalg.norm(x) for x in ref["terms"])
    d = np.linalg.norm(D0) if D0 is not None else 0.0
    return 6 * 2.0 ** -24 * abs(alpha) * t + 3 * 2.0 ** -24 * abs(beta) * d


@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("tensor", [False, True])
@pytest.mark.parametrize("shape,pad", [((150, 328), 0), ((93, 203), 5), ((70, 5000), 8)])
def test_second_level_codes_bit_exact(axis, tensor, shape, pad):
    import paper_2409_18772_amd as L
    rows, cols = shape
    bits = 4
    X = wl.random_matrix("normal", rows, cols, seed=21 + pad)
    _, view = window(X, pad)
    mode = L.SCALE_TENSOR if tensor else L.SCALE_VECTOR
    say("quantize_residual", axis, tensor, shape, pad)
    _, amax0 = L.lrqmm_quantize_ex(view, axis, bits, o.FLOOR, mode)
    codesR, amaxR = L.lrqmm_quantize_residual(view, amax0, axis, bits, o.FLOOR, mode)
    oax = o.TENSOR if tensor else (o.ROWWISE if axis == 0 else o.COLWISE)
    am0 = o.absmax(X, oax)
    _, s0 = o.scales(am0, bits)
    q0 = o.quantize(X, am0, oax, bits, o.FLOOR)
    R = o.residual(X, q0, s0, oax).astype(np.float32)
    amR = o.absmax(R, oax)
    want = o.quantize(R, amR, oax, bits, o.FLOOR)
    got = to_np(codesR)
    assert np.array_equal(got if axis == 0 else got.T, want)
    n = rows if axis == 0 else cols
    assert np.array_equal(to_np(amaxR), np.broadcast_to(np.asarray(amR, dtype=np.float32), (n,)))


@pytest.mark.parametrize("terms", [1, 3, 4])
@pytest.mark.parametrize("bits,tensor", [(4, False), (8, True)])
def test_residual_matmul_small(terms, bits, tensor):
    import torch
    import paper_2409_18772_amd as L
    M, N, K = 210, 136, 328
    A = wl.random_matrix("normal", M, K, seed=1)
    B = wl.random_matrix("uniform01", K, N, seed=2)
    D = torch.empty((M, N), dtype=torch.float32, device="cuda")
    say("residual_matmul", terms, bits, tensor)
    L.lrqmm_residual_matmul(to_dev(A), to_dev(B), D, bits, terms,
                            scale_mode=L.SCALE_TENSOR if tensor else L.SCALE_VECTOR)
    ref = o.residual_compensation(A, B, bits, terms, per_tensor=tensor)
    got = to_np(D).astype(np.float64)
    err = np.linalg.norm(got - ref["C"])
    say("err", err, "bound", bound(ref))
    assert err <= bound(ref)
    if terms > 1:       # a missing term would be far outside the bound
        assert np.linalg.norm(got - (ref["C"] - ref["terms"][-1])) > 100 * bound(ref)


def test_residual_matmul_update_and_windows():
    import paper_2409_18772_amd as L
    M, N, K, bits = 150, 123, 200, 4
    A = wl.random_matrix("normal", M, K, seed=3)
    B = wl.random_matrix("normal", K, N, seed=4)
    D0 = wl.random_matrix("uniform01", M, N, seed=5)
    _, dA = window(A, 4)
    _, dB = window(B, 3)
    bigD, dD = window(D0, 7, pad_rows=1)
    alpha, beta = 0.5, -2.0
    L.lrqmm_residual_matmul(dA, dB, dD, bits, 4, alpha=alpha, beta=beta)
    ref = o.residual_compensation(A, B, bits, 4)
    want = o.scaled_update(ref["C"], alpha, beta, D0)
    got = to_np(dD).astype(np.float64)
    assert np.linalg.norm(got - want) <= bound(ref, alpha, beta, D0)
    b = to_np(bigD)
    assert np.all(b[:, N:] == SENTINEL) and np.all(b[M:] == SENTINEL)


def test_residual_matmul_large_tiles_sampled_rows():
    import torch
    import paper_2409_18772_amd as L
    M, N, K, bits = 4096, 2048, 512, 4
    A = wl.random_matrix("normal", M, K, seed=12)
    B = wl.random_matrix("normal", K, N, seed=13)
    D = torch.empty((M, N), dtype=torch.float32, device="cuda")
    say("residual_matmul large")
    L.lrqmm_residual_matmul(to_dev(A), to_dev(B), D, bits, 4)
    rows = np.random.default_rng(8).choice(M, size=48, replace=False)
    ref = o.residual_compensation(A, B, bits, 4, row_sample=rows)
    got = to_np(D)[rows].astype(np.float64)
    assert np.linalg.norm(got - ref["C"]) <= bound(ref)
    exact = o.exact_product(A[rows], B)
    e4, e1 = o.rel_err(exact, got), o.rel_err(exact, ref["C0"])
    say("err four terms", e4, "direct quant", e1)
    assert e4 < e1 / 5


def test_bad_terms_rejected():
    import torch
    import paper_2409_18772_amd as L
    A = torch.zeros((8, 8), dtype=torch.float32, device="cuda")
    D = torch.zeros((8, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(L.LrqmmError):
        L.lrqmm_residual_matmul(A, A, D, 8, 2)
    L.lrqmm_residual_matmul(A, A, D, 8, 4)
    torch.cuda.synchronize()
    assert torch.all(D == 0)
