"""GPU test of lrqmm_gemm_static, the entry point that allocates nothing: its scratch memory is a fixed
array inside the library's device image instead of a caller workspace.  It runs the kernels of
lrqmm_gemm_ex with the same arguments, so its output must be bit-identical to lrqmm_gemm_ex's -- on two
calls in a row, the second with a smaller input (the shared array then still holds the first call's
contents), and once more with the first shape."""
import ctypes

import numpy as np
import pytest

from oracle import lrqmm_oracle as o
import lrqmm_workloads as wl
from gpu_util import say, to_dev, to_np

pytestmark = pytest.mark.gpu


def _problem(M, N, K, bits, rank, seed):
    A = wl.random_matrix("normal", M, K, seed=seed)
    B = wl.random_matrix("uniform01", K, N, seed=seed + 1)
    amA = o.absmax(A, o.ROWWISE)
    amB = o.absmax(B, o.COLWISE)
    Aq = o.quantize(A, amA, o.ROWWISE, bits)
    Bq = o.quantize(B, amB, o.COLWISE, bits)
    rng = np.random.default_rng(seed + 2)
    f32 = lambda x: np.ascontiguousarray(x, dtype=np.float32)
    fa = (f32(rng.standard_normal((M, rank))), f32(rng.uniform(0.5, 2.0, rank)), f32(rng.standard_normal((rank, K))))
    fb = (f32(rng.standard_normal((K, rank))), f32(rng.uniform(0.5, 2.0, rank)), f32(rng.standard_normal((rank, N))))
    D0 = wl.random_matrix("normal", M, N, seed=seed + 3)
    return dict(Aq=to_dev(Aq), amA=to_dev(amA), BqT=to_dev(np.ascontiguousarray(Bq.T)), amB=to_dev(amB),
                fa=tuple(map(to_dev, fa)), fb=tuple(map(to_dev, fb)), D0=D0)


def _both(p, bits, alpha, beta, want_cint):
    """(static result, workspace result) for one problem; D starts from the same contents in both."""
    import paper_2409_18772_amd as L
    D1, D2 = to_dev(p["D0"]), to_dev(p["D0"])
    r1 = L.lrqmm_gemm_static(p["Aq"], p["amA"], p["BqT"], p["amB"], bits, D1, alpha, beta, p["fa"], p["fb"],
                             want_cint=want_cint)
    r2 = L.lrqmm_gemm_ex(p["Aq"], p["amA"], p["BqT"], p["amB"], bits, D2, alpha, beta, p["fa"], p["fb"],
                         want_cint=want_cint)
    return r1, r2


def test_static_scratch_entry_point_equals_workspace_entry_point():
    import torch
    big = _problem(700, 520, 1040, 4, 12, seed=50)          # splits along K, 128 x 128 tiles, ragged
    small = _problem(130, 77, 96, 4, 5, seed=60)
    for name, p, rank in (("first call", big, 12), ("second call, smaller input", small, 5), ("third call", big, 12)):
        say("lrqmm_gemm_static:", name)
        (D1, I1), (D2, I2) = _both(p, 4, alpha=1.25, beta=-0.5, want_cint=True)
        torch.cuda.synchronize()
        assert torch.equal(I1, I2), name
        assert torch.equal(D1, D2), name
        assert bool(torch.isfinite(D1).all())
    # beta = 0 must not read D; rank 0 takes no factors
    p = small
    import paper_2409_18772_amd as L
    D1 = torch.full((130, 77), float("nan"), device="cuda")
    D2 = torch.full((130, 77), float("nan"), device="cuda")
    L.lrqmm_gemm_static(p["Aq"], p["amA"], p["BqT"], p["amB"], 4, D1)
    L.lrqmm_gemm_ex(p["Aq"], p["amA"], p["BqT"], p["amB"], 4, D2)
    torch.cuda.synchronize()
    assert torch.equal(D1, D2) and bool(torch.isfinite(D1).all())


def test_static_scratch_limit_and_arguments():
    import paper_2409_18772_amd as L
    lib = L.load_library()
    f = ctypes.c_float
    none10 = [None] * 10
    # a problem whose scratch need exceeds the static array: refused before any pointer is looked at
    assert lib.lrqmm_gemm_static(16384, 16384, 4096, 4, 64, *none10, f(1.0), f(0.0), None, 16384, None, None) \
        == L.ERR_STATIC_LIMIT
    assert "static" in L.lrqmm_status_string(L.ERR_STATIC_LIMIT)
    # row stride below the row length; empty output
    assert lib.lrqmm_gemm_static(4, 4, 4, 8, 0, *none10, f(1.0), f(0.0), None, 3, None, None) == -1
    assert lib.lrqmm_gemm_static(0, 4, 4, 8, 0, *none10, f(1.0), f(0.0), None, 4, None, None) == 0
    # the headline shape fits
    need = L.lrqmm_workspace_bytes(4096, 4096, 4096, 32, 0)
    assert need > 0
