"""GPU parity: the whole hot path (lrqmm_matmul) against the oracle's Algorithm 2.

Tolerance: relative Frobenius error of C against the float64 oracle
    tol = max(1e-5, 2 * 2^-24 * kappa),   kappa = (|C0|_F + |C - C0|_F) / |C|_F.
The GPU path computes the sketch products and the epilogue in float32 (Gram /
Cholesky / Jacobi in float64); emulating the factorization arithmetic on the CPU
gives 6e-9 (int8, Gaussian) to 5e-7 (int4 with outliers), so 1e-5 covers it with
room for accumulation-order differences.  The epilogue adds the compensation to
the dequantized product C0 in float32, so each output carries about one float32
rounding of |C0| and one of |C - C0|: when the two nearly cancel (floor
quantization of zero-mean data at 4 bits: |C0| is 40-200 times |C|) that
rounding, 2^-24 * kappa relative to C, is the floor of what float32 can deliver;
the factor 2 is margin for the 2r-term accumulation.
"""
import numpy as np
import pytest

from oracle import lrqmm_oracle as o
import lrqmm_workloads as wl
from gpu_util import say, to_dev, to_np, rel_fro, check_elementwise

pytestmark = pytest.mark.gpu

TOL = 1e-5


def tol_for(ref):
    C, C0 = ref["C"], ref["C0"]
    kappa = (np.linalg.norm(C0) + np.linalg.norm(C - C0)) / np.linalg.norm(C)
    return max(TOL, 2 * 2.0 ** -24 * kappa)


def _run_gpu(w, A, B):
    import paper_2409_18772_amd as L
    return to_np(L.lrqmm_matmul(to_dev(A), to_dev(B), w.bits, w.rank, w.oversample, w.power_iters,
                                seed=w.sketch_seed))


def test_config_one_full():
    w = wl.CONFIGS["c1_256_int8_r8"]
    A, B = wl.make_inputs(w)
    say("matmul", w.name)
    C = _run_gpu(w, A, B)
    ref = o.lrqmm(A, B, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed)
    assert rel_fro(ref["C"], C) < TOL
    check_elementwise(C, ref, w.rank, what=w.name)
    exact = o.exact_product(A, B)
    assert o.rel_err(exact, C) <= o.rel_err(exact, ref["C0"])
    # bit-identical on a second run (no atomics on floats, fixed reduction orders)
    assert np.array_equal(C, _run_gpu(w, A, B))


SMALL = [
    # name, M, N, K   (ragged: not multiples of any tile size)
    ("c2_4096_int8_r16", 200, 136, 328),
    ("c3_4096_int4_r32_outliers", 333, 517, 260),
    ("c4_16384_int4_r64", 640, 512, 768),
    ("c5_resnet50_conv_int4_r8", 3000, 64, 576),
    ("c1_256_int8_r8", 77, 50, 93),
]


@pytest.mark.parametrize("name,M,N,K", SMALL)
def test_scaled_configs_full_output(name, M, N, K):
    w = wl.scaled_config(name, M, N, K)
    A, B = wl.make_inputs(w)
    say("matmul", w.name)
    C = _run_gpu(w, A, B)
    ref = o.lrqmm(A, B, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed)
    d = rel_fro(ref["C"], C)
    say(w.name, "gpu vs oracle", d, "tol", tol_for(ref))
    assert d < tol_for(ref)
    check_elementwise(C, ref, w.rank, what=w.name)


SHORT_ROWS = [
    # M, N, K, rank, oversample, power_iters: K a multiple of 16 up to 576 (A's rows are kept in registers), ragged M,
    # K / 16 a multiple of 4 and not (the four waves of a row group then take unequal shares)
    (130, 70, 96, 4, 4, 1),
    (1000, 64, 576, 8, 0, 0),
    (257, 40, 640, 12, 4, 2),
    (64, 33, 400, 12, 8, 0),
    (500, 80, 272, 16, 8, 1),
    (90, 48, 16, 4, 0, 0),
    (2100, 24, 208, 5, 0, 1),
    (33, 40, 336, 16, 0, 0),
    (700, 64, 544, 8, 8, 1),
    (20, 24, 64, 4, 0, 0),
]


@pytest.mark.parametrize("mode", [o.FLOOR, o.NEAREST])
@pytest.mark.parametrize("M,N,K,r,p,q", SHORT_ROWS)
def test_short_rows_of_a_single_read(M, N, K, r, p, q, mode):
    """A with short rows and a sketch of at most 16 columns: row maxima, codes and the sketch product come from
    one read of A (the third, fourth and fifth shape have longer rows or wider sketches and take the separate
    kernels).  Checked against
    the oracle, and against the same call on a copy of A whose row stride (K + 1) rules that kernel out, so that
    the separate quantization and sketch kernels run: the two differ only in the order in which the sketch
    product is summed."""
    import torch
    import paper_2409_18772_amd as L
    A = wl.random_matrix("relu_normal", M, K, seed=51)
    B = wl.random_matrix("normal", K, N, seed=52)
    say("short rows", M, N, K, "rank", r, "p", p, "q", q, "mode", mode)
    dA, dB = to_dev(A), to_dev(B)
    C = to_np(L.lrqmm_matmul(dA, dB, 4, r, p, q, seed=9, round_mode=mode))
    ref = o.lrqmm(A, B, 4, r, p, q, seed=9, round_mode=mode)
    d = rel_fro(ref["C"], C)
    say("gpu vs oracle", d, "tol", tol_for(ref))
    assert d < tol_for(ref)
    check_elementwise(C, ref, r, what=f"short rows {M}x{N}x{K}")
    wide = torch.zeros((M, K + 1), dtype=torch.float32, device="cuda")
    wide[:, :K] = dA
    D = torch.empty((M, N), dtype=torch.float32, device="cuda")
    L.lrqmm_matmul_ex(wide[:, :K], dB, D, 4, r, p, q, seed=9, round_mode=mode)
    assert rel_fro(C, to_np(D)) < tol_for(ref)
    # a row stride the one-read kernel accepts (K + 4): the same kernel on a window, the same bits
    wide4 = torch.zeros((M, K + 4), dtype=torch.float32, device="cuda")
    wide4[:, :K] = dA
    D4 = torch.empty((M, N), dtype=torch.float32, device="cuda")
    L.lrqmm_matmul_ex(wide4[:, :K], dB, D4, 4, r, p, q, seed=9, round_mode=mode)
    assert np.array_equal(C, to_np(D4))


def test_rank_zero_is_direct_quant_and_modes():
    import paper_2409_18772_amd as L
    A = wl.random_matrix("normal", 150, 200, seed=1)
    B = wl.random_matrix("normal", 200, 170, seed=2)
    for mode in (o.FLOOR, o.NEAREST):
        C = to_np(L.lrqmm_matmul(to_dev(A), to_dev(B), 8, 0, round_mode=mode))
        ref = o.lrqmm(A, B, 8, 0, round_mode=mode)
        assert rel_fro(ref["C"], C) < 1e-6
        check_elementwise(C, ref, 0, what=f"rank 0, round mode {mode}")
    C = to_np(L.lrqmm_matmul(to_dev(A), to_dev(B), 4, 6, 2, 1, seed=3, round_mode=o.NEAREST))
    ref = o.lrqmm(A, B, 4, 6, 2, 1, seed=3, round_mode=o.NEAREST)
    assert rel_fro(ref["C"], C) < TOL


def test_degenerate_inputs():
    import torch
    import paper_2409_18772_amd as L
    A = np.zeros((64, 96), dtype=np.float32)
    B = wl.random_matrix("normal", 96, 80, seed=2)
    C = to_np(L.lrqmm_matmul(to_dev(A), to_dev(B), 8, 4, 2, 1))
    assert np.all(C == 0)
    A = wl.random_matrix("normal", 64, 96, seed=1)
    A[5] = 0
    B[:, 7] = 0
    C = to_np(L.lrqmm_matmul(to_dev(A), to_dev(B), 8, 4, 2, 1, seed=5))
    ref = o.lrqmm(A, B, 8, 4, 2, 1, seed=5)
    assert rel_fro(ref["C"], C) < TOL
    assert np.all(C[5] == 0) and np.all(C[:, 7] == 0)
    with pytest.raises(L.LrqmmError):
        L.lrqmm_matmul(to_dev(A), to_dev(B), 8, 60, 30)          # l > K
    with pytest.raises(L.LrqmmError):
        L.lrqmm_matmul(to_dev(A), to_dev(B), 8, 81, 0)
    e = torch.empty((0, 96), dtype=torch.float32, device="cuda")
    assert L.lrqmm_matmul(e, to_dev(B), 8, 0).shape == (0, 80)


FULL = ["c2_4096_int8_r16", "c3_4096_int4_r32_outliers"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_sampled_rows(name):
    """Full-size run in the benchmark's launch configuration, checked on sampled rows of C."""
    w = wl.CONFIGS[name]
    A, B = wl.make_inputs(w)
    say("matmul full", w.name)
    C = _run_gpu(w, A, B)
    rows = np.random.default_rng(5).choice(w.M, size=24, replace=False)
    say("oracle on", len(rows), "rows")
    ref = o.lrqmm(A, B, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed, row_sample=rows,
                  want_cint=False)
    d = rel_fro(ref["C"], C[rows])
    say(name, "gpu vs oracle", d, "tol", tol_for(ref))
    assert d < tol_for(ref)
    check_elementwise(C[rows], ref, w.rank, rows, what=name)
    exact = o.exact_product(A[rows], B)
    e_lr, e_dq = o.rel_err(exact, C[rows]), o.rel_err(exact, ref["C0"])
    say(name, "err lrqmm", e_lr, "err direct quant", e_dq)
    assert e_lr < e_dq
    if "int4" in name:
        assert e_dq / e_lr >= 10.0        # the headline claim on the outlier workload


@pytest.mark.parametrize("oversample,power_iters", [(0, 0), (8, 1)])
def test_resnet_conv_shape_sampled_rows(oversample, power_iters):
    """The conv-shaped workload at full size (100352 x 64 x 576), with the configured sketch (no oversampling, no
    power iteration) and with the alternative setting p = 8, q = 1."""
    import paper_2409_18772_amd as L
    w = wl.CONFIGS["c5_resnet50_conv_int4_r8"]
    A, B = wl.make_inputs(w)
    say("matmul full", w.name, "p", oversample, "q", power_iters)
    C = to_np(L.lrqmm_matmul(to_dev(A), to_dev(B), w.bits, w.rank, oversample, power_iters, seed=w.sketch_seed))
    rows = np.random.default_rng(6).choice(w.M, size=512, replace=False)
    ref = o.lrqmm(A, B, w.bits, w.rank, oversample, power_iters, seed=w.sketch_seed, row_sample=rows,
                  want_cint=False)
    d = rel_fro(ref["C"], C[rows])
    say(w.name, "gpu vs oracle", d, "tol", tol_for(ref))
    if (oversample, power_iters) == (0, 0):
        assert d < tol_for(ref)
        check_elementwise(C[rows], ref, w.rank, rows, what=w.name)
        return
    # With p = 8, q = 1 the cut at r = 8 falls between two singular values of R_A that agree to 0.13 %
    # (test_rsvd_truncation_between_nearly_equal_singular_values in test_gpu_rsvd_gemm.py): the rank-8 part is
    # then fixed only to ~2e-4 of its norm at float32 resolution, and C inherits that through the compensation.
    # What is unique is compared tightly -- the error against the exact product, which must equal the
    # oracle's -- and the distance itself against the factorization's own tolerance carried to C.
    exact = o.exact_product(A[rows], B)
    e_gpu, e_ref = o.rel_err(exact, C[rows]), o.rel_err(exact, ref["C"])
    comp = np.linalg.norm(ref["C"] - ref["C0"]) / np.linalg.norm(ref["C"])
    say(w.name, "err vs exact: gpu", e_gpu, "oracle", e_ref, "compensation / C", comp)
    assert abs(e_gpu - e_ref) <= 1e-4 * e_ref
    assert d < tol_for(ref) + 2 * 2e-4 * comp


# Rows of C checked against the oracle at 16384^3.  The 64 x 64 grid of 256 x 256 tiles is dealt to the 8 XCDs as
# rectangles of 32 x 16 tiles, each worked through in 16 rounds of 32 tiles; tile rows 31 and 63 (rows 7936-8191
# and 16128-16383) are the last rows of the two bands of rectangles, i.e. tiles of the last round, next to the
# band boundary.  The sample takes three rows from each and eight drawn at random.  (At this size the early
# product is not cut along K: that happens only below four rounds, and is covered at 4096^3.)
C4_ROWS = np.concatenate([[7936, 8050, 8191, 16128, 16250, 16383],
                          np.random.default_rng(7).choice(16384, size=8, replace=False)])


def test_largest_config_oracle_rows():
    """c4 (16384^3, int4, r = 64, l = 80, two power iterations) at full size, in the benchmark's launch
    configuration, against the oracle: both residual factorizations in full, C on sampled rows (rows of C
    are independent given the factors)."""
    import torch
    import paper_2409_18772_amd as L
    w = wl.CONFIGS["c4_16384_int4_r64"]
    say("inputs", w.name)
    A, B = wl.make_inputs(w)
    dA, dB = to_dev(A), to_dev(B)
    ws = L.Workspace.for_problem(w.M, w.N, w.K, w.rank, w.oversample)
    say("matmul full", w.name)
    C = L.lrqmm_matmul(dA, dB, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed, workspace=ws)
    rows = np.sort(C4_ROWS)
    Cr = C[torch.from_numpy(rows).cuda()].cpu().numpy()
    del C, dA, dB, ws
    torch.cuda.empty_cache()
    say("oracle: factorizations in full, C on", len(rows), "rows")
    ref = o.lrqmm(A, B, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed, row_sample=rows,
                  want_cint=False)
    d = rel_fro(ref["C"], Cr)
    say(w.name, "gpu vs oracle", d, "tol", tol_for(ref))
    assert d < tol_for(ref)
    check_elementwise(Cr, ref, w.rank, rows, what=w.name)
    exact = o.exact_product(A[rows], B)
    e_lr, e_dq = o.rel_err(exact, Cr), o.rel_err(exact, ref["C0"])
    say(w.name, "err lrqmm", e_lr, "err direct quant", e_dq)
    # against floor rounding, the quantizer of the method (Eq. (get_ra2)); against round-to-nearest direct
    # quantization of zero-mean data the two errors are about equal
    assert e_lr * 10.0 < e_dq


RAGGED_LARGE = [
    # shapes on the 256 x 256 tile kernel that are no multiples of its tile: guarded loads, guarded
    # epilogue, clamped rows and columns of the rank update
    (4100, 2052, 528),      # K % 16 == 0: 16-byte operand loads with guards
    (4100, 2052, 500),      # byte-wise operand loads
]


@pytest.mark.parametrize("M,N,K", RAGGED_LARGE)
@pytest.mark.parametrize("fused", [False, True])
def test_ragged_large_tile_shapes(M, N, K, fused):
    """fused = False: beta = 0 and a dense D, the schedule with the early integer product and the rank
    update as a kernel of its own; fused = True: a strided D with beta != 0, the GEMM with the fused
    epilogue.  Oracle on sampled rows, including the last (partial) tile row."""
    import torch
    import paper_2409_18772_amd as L
    bits, r, p, q = 4, 28, 4, 1      # a sketch of 32 columns: the width from which the early-product schedule is used
    A = wl.random_matrix("normal", M, K, seed=41)
    B = wl.random_matrix("uniform01", K, N, seed=42)
    rows = np.sort(np.concatenate([[0, 255, 256, 4095, 4096, M - 1],
                                   np.random.default_rng(8).choice(M, size=10, replace=False)]))
    say("ragged large tiles", M, N, K, "fused" if fused else "early product")
    ref = o.lrqmm(A, B, bits, r, p, q, seed=11, row_sample=rows, want_cint=False)
    if not fused:
        C = to_np(L.lrqmm_matmul(to_dev(A), to_dev(B), bits, r, p, q, seed=11))
        d = rel_fro(ref["C"], C[rows])
        say("gpu vs oracle", d, "tol", tol_for(ref))
        assert d < tol_for(ref)
        check_elementwise(C[rows], ref, r, rows, what="ragged early")
        return
    alpha, beta = 1.5, -0.5
    D0 = wl.random_matrix("normal", M, N, seed=43)
    big = torch.full((M, N + 3), -7.0, dtype=torch.float32, device="cuda")
    dD = big[:, :N]
    dD.copy_(torch.from_numpy(D0))
    L.lrqmm_matmul_ex(to_dev(A), to_dev(B), dD, bits, r, p, q, seed=11, alpha=alpha, beta=beta)
    got = to_np(dD)[rows].astype(np.float64)
    want = o.scaled_update(ref["C"], alpha, beta, D0[rows])
    # the update of the plain product: |alpha| times its error plus three roundings (see test_gpu_update_strides.py)
    nc, nd = np.linalg.norm(ref["C"]), np.linalg.norm(D0[rows])
    bound = abs(alpha) * tol_for(ref) * nc + 3 * 2.0 ** -24 * (abs(alpha) * nc + abs(beta) * nd)
    err = np.linalg.norm(got - want)
    say("gpu vs oracle", err, "bound", bound)
    assert err < bound
    # element-wise: the product's budget scaled by |alpha| plus the three roundings of the update
    from gpu_util import elementwise_budget
    budget, _ = elementwise_budget(ref, r, rows)
    lim = abs(alpha) * budget + 3 * 2.0 ** -24 * (abs(alpha) * np.abs(ref["C"]) + abs(beta) * np.abs(D0[rows]))
    assert np.all(np.abs(got - want) <= lim)
    assert np.all(to_np(big)[:, N:] == -7.0)


def test_wide_panels_large_tiles_sampled_rows():
    """Rank 64 on the large-tile schedule (early integer product, rank update as its own kernel): panels of
    2r = 128 columns take the update kernel that forms the panel products from bfloat16 planes.  Oracle on
    sampled rows, Frobenius and element-wise."""
    import paper_2409_18772_amd as L
    M, N, K, bits, r, p, q = 4096, 2048, 512, 4, 64, 16, 1
    A = wl.random_matrix("normal", M, K, seed=61)
    B = wl.random_matrix("normal", K, N, seed=62)
    rows = np.sort(np.random.default_rng(9).choice(M, size=16, replace=False))
    say("wide panels", M, N, K, r)
    C = to_np(L.lrqmm_matmul(to_dev(A), to_dev(B), bits, r, p, q, seed=13))
    ref = o.lrqmm(A, B, bits, r, p, q, seed=13, row_sample=rows, want_cint=False)
    d = rel_fro(ref["C"], C[rows])
    say("gpu vs oracle", d, "tol", tol_for(ref))
    assert d < tol_for(ref)
    check_elementwise(C[rows], ref, r, rows, what="wide panels")


def test_three_stream_schedule_is_repeatable():
    """The two factorization chains, the early integer product on the third stream and the K-cut tiles involve
    no atomics on floating-point data and no order that depends on timing: 300 calls at the headline shape,
    with other calls through the same workspace in between, all give the first call's bits.  (A missing event
    wait between the three streams would show up here as an occasional difference.)"""
    import torch
    import paper_2409_18772_amd as L
    w = wl.CONFIGS["c3_4096_int4_r32_outliers"]
    A, B = wl.make_inputs(w)
    dA, dB = to_dev(A), to_dev(B)
    ws = L.Workspace.for_problem(w.M, w.N, w.K, w.rank, w.oversample)
    C = torch.empty((w.M, w.N), dtype=torch.float32, device="cuda")
    first, differing = None, 0
    for it in range(300):
        L.lrqmm_matmul(dA, dB, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed, workspace=ws, C=C)
        if first is None:
            first = C.clone()
        elif not torch.equal(first, C):
            differing += 1
        if it % 7 == 3:     # a direct-quantization call and another sketch seed through the same workspace
            L.lrqmm_matmul(dA, dB, w.bits, 0, workspace=ws, C=C)
            L.lrqmm_matmul(dA, dB, w.bits, w.rank, w.oversample, w.power_iters, seed=it, workspace=ws, C=C)
    say("calls differing from the first:", differing)
    assert differing == 0


def test_call_is_ordered_like_one_stream_on_a_caller_stream():
    """On a caller's stream the call must wait for earlier work of that stream (its operands may still be in
    the making) and later work of that stream must see its result, although two library streams do part of it:
    the operands are produced by kernels enqueued on the stream right before the call, the result is copied on
    the stream right after it, nothing is synchronized in between, and the copy must equal the result of the
    same call on settled inputs, bit for bit."""
    import torch
    import paper_2409_18772_amd as L
    w = wl.CONFIGS["c3_4096_int4_r32_outliers"]
    A, B = wl.make_inputs(w)
    dA, dB = to_dev(A), to_dev(B)
    ws = L.Workspace.for_problem(w.M, w.N, w.K, w.rank, w.oversample)
    want = L.lrqmm_matmul(dA, dB, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed, workspace=ws).clone()
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    A2, B2 = torch.empty_like(dA), torch.empty_like(dB)
    C = torch.empty((w.M, w.N), dtype=torch.float32, device="cuda")
    with torch.cuda.stream(s):
        for _ in range(3):
            # operands rebuilt on the stream just before the call (x * 0.5 + x * 0.5 is exact in binary)
            torch.add(dA * 0.5, dA * 0.5, out=A2)
            torch.add(dB * 0.5, dB * 0.5, out=B2)
            L.lrqmm_matmul(A2, B2, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed, workspace=ws, C=C)
            got = C.clone()             # consumer on the same stream
            A2.zero_(); B2.zero_()      # and the operands are destroyed right behind the call
        s.synchronize()
    assert torch.equal(got, want)


def test_empty_reduction_reads_no_operand():
    """K = 0 with M, N > 0: C_F = 0, so D <- beta D (zeros when beta = 0); the GEMM kernels are not
    launched at all (they load their first operand tile unconditionally)."""
    import torch
    import paper_2409_18772_amd as L
    M, N = 300, 260
    A = torch.empty((M, 0), dtype=torch.float32, device="cuda")
    B = torch.empty((0, N), dtype=torch.float32, device="cuda")
    say("K = 0: matmul")
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    L.lrqmm_matmul(A, B, 8, 0, C=C)
    assert torch.all(C == 0)
    D0 = wl.random_matrix("normal", M, N, seed=3)
    D = to_dev(D0)
    L.lrqmm_matmul_ex(A, B, D, 4, 0, alpha=2.0, beta=-1.5)
    assert np.array_equal(to_np(D), np.float32(-1.5) * D0)
    say("K = 0: gemm")
    Aq = torch.empty((M, 0), dtype=torch.int8, device="cuda")
    BqT = torch.empty((N, 0), dtype=torch.int8, device="cuda")
    am, an = torch.ones(M, device="cuda"), torch.ones(N, device="cuda")
    C2, Cint = L.lrqmm_gemm(Aq, am, BqT, an, 8, want_cint=True)
    assert torch.all(C2 == 0) and torch.all(Cint == 0)
    say("K = 0: residual_matmul")
    D = to_dev(D0)
    L.lrqmm_residual_matmul(A, B, D, 4, 4, alpha=1.0, beta=1.0)
    assert np.array_equal(to_np(D), D0)
    # large enough for the 256 x 256 tile kernel's dispatch
    M, N = 4096, 2048
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    L.lrqmm_matmul(torch.empty((M, 0), dtype=torch.float32, device="cuda"),
                   torch.empty((0, N), dtype=torch.float32, device="cuda"), 4, 0, C=C)
    assert torch.all(C == 0)


def test_largest_config_properties():
    """c4 (16384^3, l = 80, two power iterations) at full size, properties beside the oracle comparison
    above: finite output, bit-identical repeat, and on sampled rows an error against the exact float64
    product far below that of direct (floor) quantization computed by the same library."""
    import torch
    import paper_2409_18772_amd as L
    w = wl.CONFIGS["c4_16384_int4_r64"]
    say("inputs", w.name)
    A, B = wl.make_inputs(w)
    dA, dB = to_dev(A), to_dev(B)
    ws = L.Workspace.for_problem(w.M, w.N, w.K, w.rank, w.oversample)
    say("matmul full", w.name)
    C = L.lrqmm_matmul(dA, dB, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed, workspace=ws)
    rows = np.random.default_rng(7).choice(w.M, size=12, replace=False)
    ridx = torch.from_numpy(rows).cuda()
    Cr = C[ridx].cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(Cr))
    C2 = L.lrqmm_matmul(dA, dB, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed, workspace=ws)
    assert torch.equal(C, C2)
    del C2
    C0 = L.lrqmm_matmul(dA, dB, w.bits, 0, workspace=ws)
    C0r = C0[ridx].cpu().numpy().astype(np.float64)
    say("exact product on", len(rows), "rows")
    exact = A[rows].astype(np.float64) @ B.astype(np.float64)
    e_lr, e_dq = o.rel_err(exact, Cr), o.rel_err(exact, C0r)
    say(w.name, "err lrqmm", e_lr, "err direct quant", e_dq)
    assert e_lr * 10.0 < e_dq


@pytest.mark.parametrize("shape", [(4096, 2048, 512, 28, 4, 1), (300, 200, 260, 28, 4, 1), (3000, 64, 576, 8, 0, 0)])
def test_call_can_be_captured_in_a_graph(shape):
    """The call only enqueues kernels and event waits (its clears are fill kernels), so it may be recorded
    into a HIP graph, side streams included; every replay must reproduce the eager result, with eager work
    and synchronizations between the replays.  The first shape takes the three-stream schedule (sketch of 32
    columns on the large-tile kernel), the third the persistent kernels for short rows of A (their launchers
    ask the runtime for the device's CU count, which a capture has to tolerate)."""
    import torch
    import paper_2409_18772_amd as L
    M, N, K, r, p, q = shape
    A = to_dev(wl.random_matrix("normal", M, K, seed=31))
    B = to_dev(wl.random_matrix("normal", K, N, seed=32))
    ws = L.Workspace.for_problem(M, N, K, r, p)
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")

    def step():
        L.lrqmm_matmul(A, B, 4, r, p, q, seed=7, workspace=ws, C=C)

    step()
    torch.cuda.synchronize()
    ref = C.clone()
    say("capture", shape)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        step()                       # first use of the library's streams and events outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        step()
    torch.cuda.synchronize()
    for i in range(3):
        C.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, ref), i
        step()                       # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(C, ref), i


def test_capture_with_profiling_on_is_refused():
    """Timing events do not belong in a graph: a call under stream capture with stage timing enabled
    returns LRQMM_ERR_UNSUPPORTED before it enqueues anything, and the capture stays valid (empty)."""
    import torch
    import paper_2409_18772_amd as L
    M, N, K = 300, 200, 260
    A = to_dev(wl.random_matrix("normal", M, K, seed=31))
    B = to_dev(wl.random_matrix("normal", K, N, seed=32))
    ws = L.Workspace.for_problem(M, N, K, 28, 4)
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    L.lrqmm_matmul(A, B, 4, 28, 4, 1, seed=7, workspace=ws, C=C)      # library streams exist from here on
    torch.cuda.synchronize()
    ref = C.clone()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    tmp = torch.ones(16, device="cuda")
    L.lrqmm_profile_enable(True)
    status = None
    try:
        with torch.cuda.graph(g, stream=s):
            tmp.zero_()                  # (the graph is not empty)
            try:
                L.lrqmm_matmul(A, B, 4, 28, 4, 1, seed=7, workspace=ws, C=C)
            except L.LrqmmError as e:
                status = e.status
    finally:
        L.lrqmm_profile_enable(False)
    torch.cuda.synchronize()
    assert status == -2
    L.lrqmm_matmul(A, B, 4, 28, 4, 1, seed=7, workspace=ws, C=C)      # the library still works
    torch.cuda.synchronize()
    assert torch.equal(C, ref)


def test_gemm_only_profiling_mode():
    import torch
    import paper_2409_18772_amd as L
    M, N, K = 4096, 2048, 512
    A = to_dev(wl.random_matrix("normal", M, K, seed=33))
    B = to_dev(wl.random_matrix("normal", K, N, seed=34))
    ws = L.Workspace.for_problem(M, N, K, 28, 4)
    L.lrqmm_profile_enable(L.PROF_GEMM_ONLY)
    try:
        for _ in range(3):
            L.lrqmm_matmul(A, B, 4, 28, 4, 1, workspace=ws)         # early product: stage int_gemm
        torch.cuda.synchronize()
        st, n = L.lrqmm_profile_read()
        assert n == 3 and st["int_gemm"] > 0 and st["gemm"] == 0 and st["rsvd_a"] == 0
        L.lrqmm_matmul(A, B, 4, 0, workspace=ws)                    # rank 0: fused kernel, stage gemm
        torch.cuda.synchronize()
        st, n = L.lrqmm_profile_read()
        assert n == 1 and st["gemm"] > 0 and st["int_gemm"] == 0
    finally:
        L.lrqmm_profile_enable(False)
