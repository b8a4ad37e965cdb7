"""Pins for the oracle's randomized SVD (Background 2.1, Algorithm 1, Eq. (k-svd))."""
import numpy as np
import pytest

from oracle import lrqmm_oracle as o
import lrqmm_workloads as wl


def _approx(U, S, Vt):
    return (U * S) @ Vt


@pytest.mark.parametrize("p,q", [(0, 0), (4, 0), (3, 2)])
def test_exactly_rank_r_matrix_is_recovered(p, q):
    r = 5
    R = wl.low_rank_matrix(40, 28, r, seed=11)
    om = o.gaussian_sketch(3, 0, 28, r + p)
    U, S, Vt = o.rsvd(R, r, om, q)
    assert U.shape == (40, r) and S.shape == (r,) and Vt.shape == (r, 28)
    assert np.linalg.norm(R - _approx(U, S, Vt)) <= 1e-11 * np.linalg.norm(R)
    assert np.allclose(S, np.linalg.svd(R, compute_uv=False)[:r], rtol=1e-10)


def test_full_width_sketch_reproduces_input():
    R = wl.random_matrix("uniform01", 24, 17, seed=2).astype(np.float64)
    om = o.gaussian_sketch(9, 1, 17, 17)
    U, S, Vt = o.rsvd(R, 17, om, 0)
    assert np.linalg.norm(R - _approx(U, S, Vt)) <= 1e-12 * np.linalg.norm(R)


def test_factors_are_orthonormal_and_sorted():
    R = wl.random_matrix("normal", 50, 30, seed=4).astype(np.float64)
    om = o.gaussian_sketch(1, 0, 30, 12)
    U, S, Vt = o.rsvd(R, 8, om, 1)
    assert np.allclose(U.T @ U, np.eye(8), atol=1e-12)
    assert np.allclose(Vt @ Vt.T, np.eye(8), atol=1e-12)
    assert np.all(S[:-1] >= S[1:]) and np.all(S >= 0)
    Q = o.range_finder(R, om, 1)
    assert np.allclose(Q.T @ Q, np.eye(12), atol=1e-12)
    # Pythagoras for an orthogonal projector
    lhs = np.linalg.norm(R - Q @ (Q.T @ R)) ** 2
    rhs = np.linalg.norm(R) ** 2 - np.linalg.norm(Q.T @ R) ** 2
    assert abs(lhs - rhs) <= 1e-10 * np.linalg.norm(R) ** 2


def test_converges_to_eckart_young_optimum():
    """With many power iterations the rank-r result is the truncated SVD (Eq. (k-svd))."""
    rng = np.random.default_rng(0)
    Uo, _ = np.linalg.qr(rng.standard_normal((32, 24)))
    Vo, _ = np.linalg.qr(rng.standard_normal((24, 24)))
    sig = np.concatenate([[10.0, 6.0, 4.0, 3.0], 0.5 * 0.9 ** np.arange(20)])
    R = (Uo * sig) @ Vo.T
    r = 4
    best = (Uo[:, :r] * sig[:r]) @ Vo[:, :r].T
    om = o.gaussian_sketch(5, 0, 24, r + 2)
    errs = []
    for q in (0, 1, 2, 6):
        U, S, Vt = o.rsvd(R, r, om, q)
        errs.append(np.linalg.norm(_approx(U, S, Vt) - best))
    assert errs[-1] < 1e-6 * np.linalg.norm(best)
    assert errs[0] > errs[1] > errs[2] > errs[3]
    U, S, Vt = o.rsvd(R, r, om, 6)
    assert np.allclose(S, sig[:r], rtol=1e-8)
    # never better than the optimum, and close to it
    opt = np.sqrt(np.sum(sig[r:] ** 2))
    e = np.linalg.norm(R - _approx(U, S, Vt))
    assert opt * (1 - 1e-12) <= e <= opt * (1 + 1e-6)


def test_floor_residual_has_one_dominant_singular_value():
    """Methodology (Eq. (get_ra2)) and Error analysis (Eq. (maxlambda_copy)): the floor
    residual is a rank-one mean plus a Marchenko-Pastur bulk."""
    n = 256
    A = wl.random_matrix("uniform_pm1", n, n, seed=0)
    amax = o.absmax(A, o.ROWWISE)
    _, s = o.scales(amax, 8)
    R = o.residual(A, o.quantize(A, amax, o.ROWWISE, 8), s, o.ROWWISE)
    sv = np.linalg.svd(R, compute_uv=False)
    sigma1_pred = 0.5 * np.sqrt(n * np.sum(s.astype(np.float64) ** 2))
    edge_pred = np.mean(s) / np.sqrt(12.0) * 2 * np.sqrt(n)
    assert abs(sv[0] - sigma1_pred) < 0.05 * sigma1_pred
    assert abs(sv[1] - edge_pred) < 0.1 * edge_pred
    # with round-to-nearest there is no dominant direction
    Rn = o.residual(A, o.quantize(A, amax, o.ROWWISE, 8, o.NEAREST), s, o.ROWWISE)
    svn = np.linalg.svd(Rn, compute_uv=False)
    assert svn[0] < 1.2 * edge_pred


def test_argument_checks():
    R = np.ones((6, 5))
    with pytest.raises(ValueError):
        o.rsvd(R, 0, np.ones((5, 2)))
    with pytest.raises(ValueError):
        o.rsvd(R, 3, np.ones((5, 2)))
    with pytest.raises(ValueError):
        o.rsvd(R, 2, np.ones((5, 6)))
    with pytest.raises(ValueError):
        o.rsvd(R, 2, np.ones((4, 3)))
