"""GPU parity of the extended entry points against the oracle: the last step of Algorithm 2
(D <- alpha C_F + beta D), operands that are windows of larger row-major arrays, and one
scale per matrix (Eq. (quantA) as printed).

Tolerance of the scaled update.  The kernel forms fl(fl(alpha * c) + fl(beta * d)) from the
float32 c it would have stored without the update, the oracle alpha C + beta D in float64.
So the absolute error is at most |alpha| * (error of c) plus three float32 roundings of
terms no larger than |alpha c| + |beta d|:
    |got - want|_F <= |alpha| * tol_C * |C|_F + 3 * 2^-24 * (|alpha| |C|_F + |beta| |D|_F)
with tol_C the tolerance of the plain product (see test_gpu_matmul.py).
"""
import numpy as np
import pytest

from oracle import lrqmm_oracle as o
import lrqmm_workloads as wl
from gpu_util import say, to_dev, to_np
from test_gpu_matmul import tol_for

pytestmark = pytest.mark.gpu

SENTINEL = np.float32(-12345.5)


def window(x, pad_cols, pad_rows=0):
    """A device copy of x living inside a larger array: returns (big, view)."""
    import torch
    rows, cols = x.shape
    big = torch.full((rows + pad_rows, cols + pad_cols), float(SENTINEL), dtype=torch.float32, device="cuda")
    view = big[:rows, :cols]
    view.copy_(torch.from_numpy(np.ascontiguousarray(x)))
    return big, view


def update_bound(ref, alpha, beta, D0):
    nc = np.linalg.norm(ref["C"])
    nd = np.linalg.norm(D0) if D0 is not None else 0.0
    return abs(alpha) * tol_for(ref) * nc + 3 * 2.0 ** -24 * (abs(alpha) * nc + abs(beta) * nd)


@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("pad", [0, 5, 8])
@pytest.mark.parametrize("tensor", [False, True])
def test_quantize_strided_and_per_tensor(axis, pad, tensor):
    """Codes and maxima are bit-exact for windows (vector and scalar load variants) and both granularities."""
    import paper_2409_18772_amd as L
    rows, cols = (150, 328) if pad != 5 else (93, 203)
    X = wl.random_matrix("normal", rows, cols, seed=11 + pad)
    X[3, 7] = 9.0          # a single dominant entry: the per-matrix scale differs from every per-row one
    big, view = window(X, pad, pad_rows=2)
    say("quantize_ex", axis, pad, tensor)
    codes, amax = L.lrqmm_quantize_ex(view, axis, 4, o.FLOOR, L.SCALE_TENSOR if tensor else L.SCALE_VECTOR)
    oax = o.TENSOR if tensor else (o.ROWWISE if axis == 0 else o.COLWISE)
    am = o.absmax(X, oax)
    want = o.quantize(X, am, oax, 4, o.FLOOR)
    got = to_np(codes)
    assert np.array_equal(got if axis == 0 else got.T, want)
    n = rows if axis == 0 else cols
    assert np.array_equal(to_np(amax), np.broadcast_to(np.asarray(am, dtype=np.float32), (n,)))
    # nothing outside the window was written
    b = to_np(big)
    assert np.all(b[:, cols:] == SENTINEL) and np.all(b[rows:] == SENTINEL)


@pytest.mark.parametrize("pad_a,pad_b,pad_d", [(0, 0, 0), (4, 8, 12), (3, 1, 5)])
def test_matmul_ex_alpha_beta_windows(pad_a, pad_b, pad_d):
    import paper_2409_18772_amd as L
    M, N, K, bits, r, p, q = 210, 136, 328, 4, 6, 3, 1
    A = wl.random_matrix("normal", M, K, seed=1)
    B = wl.random_matrix("uniform01", K, N, seed=2)
    D0 = wl.random_matrix("normal", M, N, seed=3)
    alpha, beta = -0.75, 2.5
    _, dA = window(A, pad_a)
    _, dB = window(B, pad_b)
    bigD, dD = window(D0, pad_d, pad_rows=1)
    say("matmul_ex windows", pad_a, pad_b, pad_d)
    L.lrqmm_matmul_ex(dA, dB, dD, bits, r, p, q, seed=9, alpha=alpha, beta=beta)
    ref = o.lrqmm(A, B, bits, r, p, q, seed=9)
    want = o.scaled_update(ref["C"], alpha, beta, D0)
    got = to_np(dD).astype(np.float64)
    err, bound = np.linalg.norm(got - want), update_bound(ref, alpha, beta, D0)
    say("err", err, "bound", bound)
    assert err <= bound
    b = to_np(bigD)
    assert np.all(b[:, N:] == SENTINEL) and np.all(b[M:] == SENTINEL)
    # a dropped or swapped term would be far outside the bound
    assert np.linalg.norm(got - o.scaled_update(ref["C"], beta, alpha, D0)) > 100 * bound


def test_matmul_ex_defaults_equal_matmul_bitwise():
    """alpha = 1, beta = 0, dense operands: the same bits as lrqmm_matmul, and NaNs in D are not read."""
    import torch
    import paper_2409_18772_amd as L
    A = wl.random_matrix("normal", 130, 96, seed=4)
    B = wl.random_matrix("normal", 96, 72, seed=5)
    dA, dB = to_dev(A), to_dev(B)
    C = L.lrqmm_matmul(dA, dB, 8, 5, 2, 1, seed=3)
    D = torch.full((130, 72), float("nan"), dtype=torch.float32, device="cuda")
    L.lrqmm_matmul_ex(dA, dB, D, 8, 5, 2, 1, seed=3)
    assert torch.equal(C, D)


@pytest.mark.parametrize("bits,r,p,q", [(8, 6, 2, 1), (4, 10, 0, 0)])
def test_matmul_ex_one_scale_per_matrix(bits, r, p, q):
    import paper_2409_18772_amd as L
    M, N, K = 170, 140, 260
    A = wl.random_matrix("uniform01", M, K, seed=6)
    B = wl.random_matrix("normal", K, N, seed=7)
    import torch
    D = torch.empty((M, N), dtype=torch.float32, device="cuda")
    say("matmul_ex per-tensor", bits, r)
    L.lrqmm_matmul_ex(to_dev(A), to_dev(B), D, bits, r, p, q, seed=2, scale_mode=L.SCALE_TENSOR)
    ref = o.lrqmm(A, B, bits, r, p, q, seed=2, per_tensor=True)
    got = to_np(D).astype(np.float64)
    assert np.linalg.norm(got - ref["C"]) <= tol_for(ref) * np.linalg.norm(ref["C"])
    # and it is not the per-row/per-column result
    ref_v = o.lrqmm(A, B, bits, r, p, q, seed=2)
    assert np.linalg.norm(got - ref_v["C"]) > 100 * tol_for(ref) * np.linalg.norm(ref["C"])


def test_gemm_ex_with_factors_and_int_output():
    import torch
    import paper_2409_18772_amd as L
    M, N, K, bits, r = 150, 123, 200, 4, 5
    A = wl.random_matrix("normal", M, K, seed=8)
    B = wl.random_matrix("normal", K, N, seed=9)
    ref = o.lrqmm(A, B, bits, r, 2, 1, seed=4)
    D0 = wl.random_matrix("uniform01", M, N, seed=10)
    bigD, dD = window(D0, 7)
    f32 = lambda x: to_dev(np.asarray(x, dtype=np.float32))
    fa = (f32(ref["U"]), f32(ref["Sig"]), f32(ref["Vt"]))
    fb = (f32(ref["W"]), f32(ref["Gam"]), f32(ref["Zt"]))
    Aq, BqT = to_dev(ref["Aq"]), to_dev(np.ascontiguousarray(ref["Bq"].T))
    alpha, beta = 3.0, -0.5
    _, Cint = L.lrqmm_gemm_ex(Aq, f32(ref["amax_a"]), BqT, f32(ref["amax_b"]), bits, dD, alpha, beta, fa, fb,
                              want_cint=True)
    assert np.array_equal(to_np(Cint), ref["Cint"])
    # the factors were rounded to float32 on the way in: compare with the oracle on those
    Cf = o.compensate(ref["Aq"], ref["sa"], ref["Bq"], ref["sb"], *[to_np(t) for t in fa], *[to_np(t) for t in fb])
    want = o.scaled_update(Cf, alpha, beta, D0)
    got = to_np(dD).astype(np.float64)
    bound = update_bound({"C": Cf, "C0": ref["C0"]}, alpha, beta, D0)
    assert np.linalg.norm(got - want) <= bound
    assert np.all(to_np(bigD)[:, N:] == SENTINEL)


@pytest.mark.parametrize("alpha,beta,pad_d", [(1.5, 0.0, 0), (1.5, -0.5, 4)])
def test_large_tile_paths_sampled_rows(alpha, beta, pad_d):
    """Sizes on the large-tile kernel: beta = 0 on a dense D takes the early-product schedule (alpha is
    applied by the update kernel), any other case the fused store phase."""
    import paper_2409_18772_amd as L
    M, N, K, bits, r, p, q = 4096, 2048, 512, 4, 28, 4, 1
    A = wl.random_matrix("normal", M, K, seed=12)
    B = wl.random_matrix("normal", K, N, seed=13)
    D0 = wl.random_matrix("normal", M, N, seed=14)
    _, dD = window(D0, pad_d)
    say("matmul_ex large", alpha, beta, pad_d)
    L.lrqmm_matmul_ex(to_dev(A), to_dev(B), dD, bits, r, p, q, seed=21, alpha=alpha, beta=beta)
    rows = np.random.default_rng(8).choice(M, size=48, replace=False)
    ref = o.lrqmm(A, B, bits, r, p, q, seed=21, row_sample=rows, want_cint=False)
    want = o.scaled_update(ref["C"], alpha, beta, D0[rows])
    got = to_np(dD)[rows].astype(np.float64)
    err, bound = np.linalg.norm(got - want), update_bound(ref, alpha, beta, D0[rows])
    say("err", err, "bound", bound)
    assert err <= bound


def test_bad_strides_are_rejected():
    import torch
    import paper_2409_18772_amd as L
    lib = L.load_library()
    A = torch.zeros((8, 8), dtype=torch.float32, device="cuda")
    ws = L.Workspace.for_problem(8, 8, 8, 0, 0)
    import ctypes
    args = lambda lda, ldb, ldd, mode: (8, 8, 8, 8, 0, 0, 0, 0, 0, mode, 0, A.data_ptr(), lda, A.data_ptr(), ldb, 1.0, 0.0,
                                        A.data_ptr(), ldd, ctypes.c_void_p(ws.ptr), ws.nbytes, None)
    assert lib.lrqmm_matmul_ex(*args(7, 8, 8, 0)) == -1
    assert lib.lrqmm_matmul_ex(*args(8, 7, 8, 0)) == -1
    assert lib.lrqmm_matmul_ex(*args(8, 8, 7, 0)) == -1
    assert lib.lrqmm_matmul_ex(*args(8, 8, 8, 2)) == -1
    assert lib.lrqmm_matmul_ex(*args(8, 8, 8, 0)) == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("K", [512, 2112])
def test_early_product_equals_fused_store_phase_bitwise(K):
    """256 tiles on a chip whose two SVD workgroups leave 254 CUs: the early integer product cuts its last
    tiles along K (evenly at K = 512, unevenly at 33 K-tiles) and sums them with integer atomics.  The dense
    call takes that schedule, the call into a window of a wider array the fused kernel: same bits."""
    import torch
    import paper_2409_18772_amd as L
    M = N = 4096
    A = wl.random_matrix("normal", M, K, seed=31)
    B = wl.random_matrix("normal", K, N, seed=32)
    dA, dB = to_dev(A), to_dev(B)
    say("early vs fused", K)
    D1 = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    L.lrqmm_matmul_ex(dA, dB, D1, 4, 28, 4, 1, seed=5)
    big, D2 = window(np.zeros((M, N), dtype=np.float32), 4)
    L.lrqmm_matmul_ex(dA, dB, D2, 4, 28, 4, 1, seed=5)
    assert torch.equal(D1, D2)
    # twice in a row on the same output: the zeroing of the summed tiles is part of every call
    L.lrqmm_matmul_ex(dA, dB, D1, 4, 28, 4, 1, seed=5)
    assert torch.equal(D1, D2)


@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("ell,round_mode,rows,cols", [(24, 0, 640, 512), (40, 0, 640, 512), (72, 0, 640, 512),
                                                       (40, 1, 640, 512), (40, 0, 4096, 4096)])
def test_guard_free_pass_kernels_equal_the_guarded_ones_bitwise(axis, ell, round_mode, rows, cols):
    """A dense operand whose sizes are multiples of 128 takes the guard-free instantiations of the two
    residual products; the same values inside an array with an odd row stride take the guarded scalar-load
    kernels.  Same arithmetic in the same order: the factors must agree bit for bit.  (At 640 x 512 only R.W
    has whole chunks; at 4096 x 4096 the row chunks of Rt.W are multiples of 128 as well.)"""
    import torch
    import paper_2409_18772_amd as L
    X = wl.random_matrix("normal", rows, cols, seed=41 + ell)
    oax = o.ROWWISE if axis == 0 else o.COLWISE
    amax = to_dev(np.asarray(o.absmax(X, oax), dtype=np.float32).reshape(-1))
    dense = to_dev(X)
    _, view = window(X, 1)
    rank, p = ell - 8, 8
    say("guard-free vs guarded", axis, ell, round_mode)
    a = L.lrqmm_rsvd_ex(dense, amax, axis, 4, rank, p, 1, seed=13, round_mode=round_mode)
    b = L.lrqmm_rsvd_ex(view, amax, axis, 4, rank, p, 1, seed=13, round_mode=round_mode)
    for x, y, name in zip(a, b, ("U", "Sigma", "Vt")):
        assert torch.equal(x, y), name


@pytest.mark.parametrize("M,N,K,r,p,mode,tensor", [(640, 512, 768, 24, 8, 0, False), (512, 640, 1024, 16, 8, 1, False),
                                                   (640, 512, 768, 60, 12, 0, True)])
def test_fused_quantize_and_sketch_equals_the_separate_calls_bitwise(M, N, K, r, p, mode, tensor):
    """For shapes on the guard-free pass kernels, lrqmm_matmul takes the group maxima first and lets the first
    residual product write the codes and the step vectors as well (one read of each operand fewer).  The same
    arithmetic in the same order as quantizing and factoring separately: the chain of lrqmm_quantize_ex,
    lrqmm_rsvd and lrqmm_gemm must give the same C bit for bit (both rounding modes, both scale granularities)."""
    import torch
    import paper_2409_18772_amd as L
    A = wl.random_matrix("normal", M, K, seed=51)
    B = wl.random_matrix("uniform01", K, N, seed=52)
    dA, dB = to_dev(A), to_dev(B)
    say("fused quantize + sketch", M, N, K, r, p, mode, tensor)
    sm = L.SCALE_TENSOR if tensor else L.SCALE_VECTOR
    D = torch.empty((M, N), dtype=torch.float32, device="cuda")
    L.lrqmm_matmul_ex(dA, dB, D, 4, r, p, 1, seed=17, round_mode=mode, scale_mode=sm)
    Aq, amA = L.lrqmm_quantize_ex(dA, 0, 4, mode, sm)
    BqT, amB = L.lrqmm_quantize_ex(dB, 1, 4, mode, sm)
    fa = L.lrqmm_rsvd(dA, amA, 0, 4, r, p, 1, seed=17, round_mode=mode)
    fb = L.lrqmm_rsvd(dB, amB, 1, 4, r, p, 1, seed=17, round_mode=mode)
    C = L.lrqmm_gemm(Aq, amA, BqT, amB, 4, fa, fb)
    assert torch.equal(C, D)
    # and against the oracle, like every other path
    ref = o.lrqmm(A, B, 4, r, p, 1, seed=17, round_mode=mode, per_tensor=tensor)
    from gpu_util import rel_fro, check_elementwise
    assert rel_fro(ref["C"], to_np(D)) < tol_for(ref)
    check_elementwise(to_np(D), ref, r, what="fused quantize + sketch")
