"""GPU tests of the reduced-precision compensation path (Methodology, text after Eq. (gemm_r_split): the
compensation terms may be computed in half precision).

Modes (lrqmm.h): PREC_FP32 -- three bfloat16 planes per float32 operand, six plane products (float32
accuracy); PREC_BF16X2 -- two planes, three products, relative error of a product 2^-16; PREC_BF16 -- one
plane, 2^-8; PREC_SUBSPACE_BF16X2 -- two planes in the products that only shape the subspace, three in the
last projection and the panel code products: held to the two-plane bounds.  What the modes must keep, and what they are allowed to lose:

* The approximation quality of the method does not depend on the mode: the error against the exact
  float64 product stays that of the float32 mode to within a few percent.  A reduced mode perturbs the
  sketch and the projected matrix by e = 2^-16 resp. 2^-8 relative to their entries; the rank-r
  factors then capture the residual's dominant (mean) direction with relative error ~e and the bulk
  directions about as well as any other random sketch would.
* Parity with the float64 oracle is lost in proportion: the compensation (of size kappa |C|, kappa as in
  test_gpu_matmul.py) carries a relative error of about e / sqrt(n) in its dominant part (the plane
  truncation errors of the n terms of a dot product are independent), so
      |C_mode - C_oracle|_F / |C|_F  <~  4 e kappa / sqrt(min(M, N, K)) + tol_fp32,
  the factor 4 covering the two factorizations and the two code products.  The measured values sit a
  factor 3-10 below this bound.
* Singular values of the residual: relative error <= 4 e (dominant value much closer).
"""
import numpy as np
import pytest

from oracle import lrqmm_oracle as o
import lrqmm_workloads as wl
from gpu_util import say, to_dev, to_np, rel_fro
from test_gpu_matmul import tol_for

pytestmark = pytest.mark.gpu

EPS = {0: 2.0 ** -24, 1: 2.0 ** -16, 2: 2.0 ** -8, 3: 2.0 ** -16}

CASES = [
    # name, M, N, K
    ("c3_4096_int4_r32_outliers", 640, 512, 768),
    ("c2_4096_int8_r16", 512, 640, 1024),
    ("c3_4096_int4_r32_outliers", 333, 517, 260),     # ragged: guarded kernels
]


@pytest.mark.parametrize("name,M,N,K", CASES)
def test_reduced_precision_end_to_end(name, M, N, K):
    import torch
    import paper_2409_18772_amd as L
    w = wl.scaled_config(name, M, N, K)
    A, B = wl.make_inputs(w)
    ref = o.lrqmm(A, B, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed)
    exact = o.exact_product(A, B)
    kappa = (np.linalg.norm(ref["C0"]) + np.linalg.norm(ref["C"] - ref["C0"])) / np.linalg.norm(ref["C"])
    dA, dB = to_dev(A), to_dev(B)
    errs = {}
    for mode in (L.PREC_FP32, L.PREC_SUBSPACE_BF16X2, L.PREC_BF16X2, L.PREC_BF16):
        D = torch.empty((M, N), dtype=torch.float32, device="cuda")
        L.lrqmm_matmul_ex(dA, dB, D, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed, precision=mode)
        C = to_np(D)
        parity = rel_fro(ref["C"], C)
        bound = 4 * EPS[mode] * kappa / np.sqrt(min(M, N, K)) + tol_for(ref)
        errs[mode] = o.rel_err(exact, C)
        say(w.name, "mode", mode, "parity", parity, "bound", bound, "err vs exact", errs[mode])
        assert parity < bound
        if mode == L.PREC_FP32:
            # the default mode is the path of lrqmm_matmul, bit for bit
            C1 = to_np(L.lrqmm_matmul(dA, dB, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed))
            assert np.array_equal(C, C1)
    # the method's accuracy does not depend on the arithmetic of the compensation path
    assert errs[L.PREC_BF16X2] < 1.02 * errs[L.PREC_FP32]
    assert errs[L.PREC_SUBSPACE_BF16X2] < 1.02 * errs[L.PREC_FP32]
    assert errs[L.PREC_BF16] < 1.10 * errs[L.PREC_FP32]
    assert errs[L.PREC_BF16] < o.rel_err(exact, ref["C0"])


@pytest.mark.parametrize("axis", [0, 1])
def test_reduced_precision_rsvd(axis):
    import paper_2409_18772_amd as L
    rows, cols, bits, r, p, q = 512, 640, 4, 16, 8, 1
    X = wl.random_matrix("normal", rows, cols, seed=71)
    oax = o.ROWWISE if axis == 0 else o.COLWISE
    amax = o.absmax(X, oax)
    _, s = o.scales(amax, bits)
    R = o.residual(X, o.quantize(X, amax, oax, bits), s, oax)
    omega = o.gaussian_sketch(5, axis, cols, r + p)
    U, S, Vt = o.rsvd(R, r, omega, q)
    want = (U * S) @ Vt
    for mode in (L.PREC_FP32, L.PREC_SUBSPACE_BF16X2, L.PREC_BF16X2, L.PREC_BF16):
        u, sg, vt = L.lrqmm_rsvd_ex(to_dev(X), to_dev(amax), axis, bits, r, p, q, seed=5, precision=mode)
        u, sg, vt = (to_np(t).astype(np.float64) for t in (u, sg, vt))
        ds = np.max(np.abs(sg - S) / S)
        # captured energy: |U S Vt|_F against the oracle's (the reduced modes keep the approximation quality)
        got = (u * sg) @ vt
        energy = np.linalg.norm(got) / np.linalg.norm(want)
        resid = np.linalg.norm(R - got) / np.linalg.norm(R - want)
        say("rsvd axis", axis, "mode", mode, "sigma rel err", ds, "energy ratio", energy, "residual ratio", resid,
            "orth", np.abs(u.T @ u - np.eye(r)).max())
        assert ds < max(2e-5, 4 * EPS[mode])
        assert abs(energy - 1) < max(1e-5, EPS[mode])
        assert resid < 1 + max(1e-4, 4 * EPS[mode])
        assert np.abs(u.T @ u - np.eye(r)).max() < 2e-5       # orthonormalization is float64 in every mode
