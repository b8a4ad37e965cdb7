"""GPU parity: lrqmm_rsvd and lrqmm_gemm stage by stage (oracle outputs as inputs).

Singular vectors are unique only up to sign, so factors are compared through
Sigma, through the rank-r product U diag(Sigma) Vt and through orthonormality.
Tolerances (float32 kernels against the float64 oracle):
  Sigma            rtol 2e-5
  U Sigma Vt       relative Frobenius 2e-4 (truncation inside a near-degenerate
                   bulk amplifies float32 rounding of the sketch products)
  C from factors   relative Frobenius 3e-6 (float32 accumulation of 2r terms + dequant)
  integer GEMM     bit exact
"""
import numpy as np
import pytest

from oracle import lrqmm_oracle as o
import lrqmm_workloads as wl
from gpu_util import say, to_dev, to_np, rel_fro

pytestmark = pytest.mark.gpu


def _residual_parts(X, axis, bits):
    amax = o.absmax(X, axis)
    _, s = o.scales(amax, bits)
    codes = o.quantize(X, amax, axis, bits)
    return amax, s, codes, o.residual(X, codes, s, axis)


RSVD_CASES = [
    # rows, cols, axis, bits, rank, p, q, kind
    (256, 256, o.ROWWISE, 8, 8, 0, 0, "uniform_pm1"),
    (256, 256, o.COLWISE, 8, 8, 0, 0, "uniform_pm1"),
    (300, 517, o.ROWWISE, 4, 12, 5, 1, "normal"),
    (517, 300, o.COLWISE, 4, 12, 5, 1, "normal"),
    (1000, 130, o.ROWWISE, 8, 16, 8, 2, "uniform01"),
    (130, 1000, o.COLWISE, 8, 16, 8, 2, "relu_normal"),
    (1024, 768, o.ROWWISE, 4, 32, 8, 1, "normal_outliers"),
    (768, 1024, o.COLWISE, 4, 64, 16, 2, "normal"),
    (96, 80, o.ROWWISE, 8, 80, 0, 0, "normal"),
    # 4100 rows make fewer Gram workgroups (33 of 128 rows) than 4096 columns (64 of 64): the scratch for the
    # Gram partials has to cover the larger of the two
    (4100, 4096, o.ROWWISE, 4, 24, 8, 1, "normal"),
    # a tall operand with a narrow sketch: more than 64 Gram workgroups, summed in several batches
    (20000, 64, o.ROWWISE, 4, 8, 0, 1, "relu_normal"),
    (64, 20000, o.COLWISE, 4, 8, 0, 1, "normal"),
    # the same with a sketch of 32 padded columns (71 partials of 1024 entries)
    (9000, 200, o.ROWWISE, 4, 20, 8, 1, "normal"),
    (200, 9000, o.COLWISE, 4, 20, 8, 1, "relu_normal"),
]


@pytest.mark.parametrize("rows,cols,axis,bits,rank,p,q,kind", RSVD_CASES)
def test_rsvd_against_oracle(rows, cols, axis, bits, rank, p, q, kind):
    import paper_2409_18772_amd as L
    say("rsvd", rows, cols, axis, bits, rank, p, q, kind)
    X = wl.random_matrix(kind, rows, cols, seed=rows * 3 + cols)
    amax, s, codes, R = _residual_parts(X, axis, bits)
    om = o.gaussian_sketch(99, axis, cols, rank + p)
    U0, S0, Vt0 = o.rsvd(R, rank, om, q)
    # with the oracle's sketch handed in
    U, S, Vt = L.lrqmm_rsvd(to_dev(X), to_dev(amax), axis, bits, rank, p, q, seed=99, omega=to_dev(om))
    U, S, Vt = to_np(U), to_np(S), to_np(Vt)
    assert np.allclose(S, S0, rtol=2e-5, atol=0)
    assert np.all(S[:-1] >= S[1:])
    Rr0 = (U0 * S0) @ Vt0
    Rr = (U.astype(np.float64) * S) @ Vt
    assert rel_fro(Rr0, Rr) < 2e-4
    assert np.max(np.abs(U.T.astype(np.float64) @ U - np.eye(rank))) < 2e-5
    assert np.max(np.abs(Vt.astype(np.float64) @ Vt.T - np.eye(rank))) < 2e-5
    # with the library's own generator (same counter-based stream as the oracle's)
    U2, S2, Vt2 = L.lrqmm_rsvd(to_dev(X), to_dev(amax), axis, bits, rank, p, q, seed=99)
    assert np.array_equal(to_np(S2), S) and np.array_equal(to_np(U2), U) and np.array_equal(to_np(Vt2), Vt)


def test_rsvd_truncation_between_nearly_equal_singular_values():
    """A case in which the rank-r truncation is not determined at float32 resolution: the residual of the tall
    conv-shaped operand (100352 x 576, ReLU inputs) with l = 16, one power iteration, truncated to r = 8.  The
    power iteration packs the captured bulk singular values together (44.06 and 44.00 at positions 8 and 9:
    sigma_r / (sigma_r - sigma_r+1) = 778), so the singular vectors on the two sides of the cut mix under a
    perturbation of the projected matrix of a few 1e-6 -- what float32 accumulation over 10^5 rows leaves --
    by a few 1e-3, and U S V^T moves by about 2e-4 of its norm although every singular value stands to 1e-7.
    Both truncations are equally good rank-8 approximations.  So the comparison is on what is unique -- the
    singular values, the orthonormality of the factors, and the approximation error |R - U S V^T|_F, which
    must equal the oracle's to 1e-6 -- and the distance itself is only held to the perturbation estimate
    gap factor x 1e-5 relative to the part of U S V^T at the cut."""
    import paper_2409_18772_amd as L
    w = wl.CONFIGS["c5_resnet50_conv_int4_r8"]
    X, _ = wl.make_inputs(w)
    rank, p, q = 8, 8, 1
    amax, s, codes, R = _residual_parts(X, o.ROWWISE, w.bits)
    om = o.gaussian_sketch(w.sketch_seed, 0, X.shape[1], rank + p)
    Q = o.range_finder(R, om, q)
    spectrum = np.linalg.svd(Q.T @ R, compute_uv=False)
    gap = spectrum[rank - 1] / (spectrum[rank - 1] - spectrum[rank])
    U0, S0, Vt0 = o.rsvd(R, rank, om, q)
    U, S, Vt = L.lrqmm_rsvd(to_dev(X), to_dev(amax), 0, w.bits, rank, p, q, seed=w.sketch_seed)
    U, S, Vt = (to_np(t).astype(np.float64) for t in (U, S, Vt))
    Rr0, Rr = (U0 * S0) @ Vt0, (U * S) @ Vt
    e0, e1 = np.linalg.norm(R - Rr0), np.linalg.norm(R - Rr)
    d = rel_fro(Rr0, Rr)
    say("gap factor", gap, "sigma rel", np.max(np.abs(S - S0) / S0), "U S Vt distance", d, "approximation error",
        e1, "oracle", e0)
    assert gap > 100                                    # the case is what it is meant to be
    assert np.allclose(S, S0, rtol=2e-5, atol=0)
    assert np.max(np.abs(U.T @ U - np.eye(rank))) < 2e-5 and np.max(np.abs(Vt @ Vt.T - np.eye(rank))) < 2e-5
    assert abs(e1 - e0) <= 1e-6 * e0
    assert d <= gap * 1e-5 * S0[rank - 1] / np.linalg.norm(S0)


def test_rsvd_zero_residual_and_errors():
    import torch
    import paper_2409_18772_amd as L
    # entries are exact multiples of the step: residual is exactly zero
    codes = np.random.default_rng(0).integers(-7, 8, size=(64, 48)).astype(np.float32)
    codes[:, 0] = 7
    X = codes * np.float32(0.25)
    X = np.ascontiguousarray(X)
    amax = o.absmax(X, o.ROWWISE)
    assert np.all(o.residual(X, o.quantize(X, amax, 0, 4), o.scales(amax, 4)[1], 0) == 0)
    U, S, Vt = L.lrqmm_rsvd(to_dev(X), to_dev(amax), 0, 4, 4, 2, 1, seed=1)
    U, S, Vt = to_np(U), to_np(S), to_np(Vt)
    assert np.all(np.isfinite(U)) and np.all(np.isfinite(Vt))
    assert np.all(S == 0) and np.all((U * S) @ Vt == 0)
    x = to_dev(X)
    a = to_dev(amax)
    with pytest.raises(L.LrqmmError):
        L.lrqmm_rsvd(x, a, 0, 4, 0)                 # rank 0
    with pytest.raises(L.LrqmmError):
        L.lrqmm_rsvd(x, a, 0, 4, 40, 10)            # l > cols
    with pytest.raises(L.LrqmmError):
        L.lrqmm_rsvd(x, a, 0, 4, 4, workspace=L.Workspace(1024))   # workspace too small


GEMM_CASES = [
    # M, N, K, bits, rank
    (256, 256, 256, 8, 8),
    (128, 128, 64, 8, 0),
    (200, 136, 328, 4, 5),
    (129, 257, 1000, 8, 16),
    (1, 1, 16, 8, 1),
    (64, 640, 576, 4, 8),
    (500, 300, 77, 8, 3),       # K not a multiple of 16: byte-wise operand path
    (384, 512, 2048, 4, 32),
    (1000, 64, 576, 4, 8),      # at most 64 columns: the 128 x 64 tile
    (300, 40, 100, 8, 4),       # ... ragged, byte-wise operand path
    (257, 65, 128, 4, 0),       # one column more: back to the 128-wide tile
]


@pytest.mark.parametrize("M,N,K,bits,rank", GEMM_CASES)
def test_gemm_int_exact_and_compensation(M, N, K, bits, rank):
    import paper_2409_18772_amd as L
    say("gemm", M, N, K, bits, rank)
    A = wl.random_matrix("normal", M, K, seed=M + K)
    B = wl.random_matrix("normal", K, N, seed=N + K + 1)
    amA, sA, Aq, Ra = _residual_parts(A, o.ROWWISE, bits)
    amB, sB, Bq, Rb = _residual_parts(B, o.COLWISE, bits)
    fa = fb = None
    U = None
    if rank:
        U, S, Vt = o.rsvd(Ra, rank, o.gaussian_sketch(1, 0, K, rank), 1)
        W, G, Zt = o.rsvd(Rb, rank, o.gaussian_sketch(1, 1, N, rank), 1)
        f32 = lambda x: np.ascontiguousarray(x, dtype=np.float32)
        U, S, Vt, W, G, Zt = map(f32, (U, S, Vt, W, G, Zt))
        fa = tuple(map(to_dev, (U, S, Vt)))
        fb = tuple(map(to_dev, (W, G, Zt)))
    C, Cint = L.lrqmm_gemm(to_dev(Aq), to_dev(amA), to_dev(np.ascontiguousarray(Bq.T)), to_dev(amB), bits,
                           fa, fb, want_cint=True)
    ref_int = o.int_gemm(Aq, Bq)
    assert np.array_equal(to_np(Cint).astype(np.int64), ref_int)
    if rank:
        Cref = o.compensate(Aq, sA, Bq, sB, U, S, Vt, W, G, Zt)
    else:
        Cref = o.compensate(Aq, sA, Bq, sB, None, None, None, None, None, None)
    assert rel_fro(Cref, to_np(C)) < 3e-6
    # without the int32 side output the float result is identical
    C2 = L.lrqmm_gemm(to_dev(Aq), to_dev(amA), to_dev(np.ascontiguousarray(Bq.T)), to_dev(amB), bits, fa, fb)
    assert np.array_equal(to_np(C2), to_np(C))


def test_gemm_extreme_codes_and_limits():
    import torch
    import paper_2409_18772_amd as L
    M, N, K = 96, 160, 4096
    Aq = np.full((M, K), -128, dtype=np.int8)
    Bq = np.full((K, N), -128, dtype=np.int8)
    Aq[::3] = 127
    am = np.full(M, 127.0, dtype=np.float32)
    bm = np.full(N, 127.0, dtype=np.float32)
    C, Cint = L.lrqmm_gemm(to_dev(Aq), to_dev(am), to_dev(np.ascontiguousarray(Bq.T)), to_dev(bm), 8,
                           want_cint=True)
    assert np.array_equal(to_np(Cint).astype(np.int64), o.int_gemm(Aq, Bq))
    lib = L.load_library()
    ws = L.Workspace(1 << 20)
    z = torch.zeros(16, device="cuda")
    # K too large for int32 accumulation at 8 bits
    assert lib.lrqmm_gemm(1, 1, 131072, 8, 0, z.data_ptr(), z.data_ptr(), z.data_ptr(), z.data_ptr(), None, None,
                          None, None, None, None, z.data_ptr(), None, ws.ptr, ws.nbytes, None) == -2
    # empty output
    assert lib.lrqmm_gemm(0, 5, 16, 8, 0, None, None, None, None, None, None, None, None, None, None, None, None,
                          None, 0, None) == 0
    # missing workspace
    assert lib.lrqmm_gemm(1, 1, 16, 8, 0, z.data_ptr(), z.data_ptr(), z.data_ptr(), z.data_ptr(), None, None, None,
                          None, None, None, z.data_ptr(), None, None, 0, None) == -3
