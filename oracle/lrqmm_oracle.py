"""CPU oracle for LRQMM (low-rank residual quantized matrix multiplication).

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, step-by-step CPU
statement of what the hot path computes.  It shares no code with the HIP
library, imports nothing from it, and may be imported only by tests, by the
smoke check and by the benchmark's CPU-baseline leg.  The product path never
calls it.

Every function names the passage of the paper it follows (section, equation or
algorithm).  Integer-valued stages use exactly specified IEEE single-precision
operations so codes are bit-comparable; everything after the integer stage is
carried in float64.  Library primitives used as steps: numpy matmul, Householder
QR (numpy.linalg.qr) and a dense SVD (numpy.linalg.svd).

Pins (tests/test_oracle_*.py, no GPU):
  quantizer      hand-worked example, range/residual-interval properties, exact
                 rational brute force
  int_gemm       python big-int triple loop, permutation/identity cases
  sketch         own log/cos/sqrt against libm, moments + KS test, stream independence
  rsvd           exactly rank-r input recovered, full-rank sketch reproduces the
                 input, Eckart-Young optimum on tiny inputs, Q^T Q = I
  lrqmm          dense identity (A~ + R_Ar)(B~ + R_Br), full rank equals A.B,
                 err(LRQMM) <= err(direct quant), printed Table 3-4 values
                 (direct-quant column tight, LRQMM column order of magnitude)
  residual_compensation  dense identity (A~ + R~_A)(B~ + R~_B) for four terms, second-level
                 residual inside [0, s_R), first term equal to direct quantization,
                 printed QT-110 / QT-111 columns of Tables 3-4
  scaled_update  hand-worked 2x2 example in exact fractions, alpha = 1 / beta = 0
                 identity, beta = 0 ignoring NaNs in D, full-rank case equal to
                 alpha A.B + beta D
Parity unpinned: none of the functions below lacks a pin; the end-to-end
tolerance between float32 GPU arithmetic and this float64 oracle is not fixed by
the paper and is derived in the design notes.
"""
from __future__ import annotations

import numpy as np

FLOOR = 0      # Methodology, Eq. (get_ra2): round down, residual entries >= 0
NEAREST = 1    # Background, Eq. (quantAB): round to nearest (ties to even)

ROWWISE = 0    # one scale per row   (operand A; vector-wise quantization, Background 2.2)
COLWISE = 1    # one scale per column (operand B)
TENSOR = -1    # one scale per matrix (the paper's own equations, Eq. (quantA))

_TINY_AMAX = np.float32(1e-30)


def qmax_of(bits: int) -> int:
    """Largest positive code, 2^(N-1) - 1 (Eq. (quantA))."""
    if not (2 <= bits <= 8):
        raise ValueError("bits must be in [2, 8]")
    return (1 << (bits - 1)) - 1


# --------------------------------------------------------------------------
# Quantizer  (Background 2.2, Eq. (quantA)/(quantAB); floor variant Eq. (get_ra2))
# --------------------------------------------------------------------------
def absmax(X: np.ndarray, axis: int) -> np.ndarray:
    """a_max of Eq. (quantA): per row, per column or for the whole matrix."""
    X = np.asarray(X, dtype=np.float32)
    if not np.all(np.isfinite(X)):
        raise ValueError("inputs must be finite")
    a = np.abs(X)
    if axis == ROWWISE:
        return a.max(axis=1) if X.shape[1] else np.zeros(X.shape[0], np.float32)
    if axis == COLWISE:
        return a.max(axis=0) if X.shape[0] else np.zeros(X.shape[1], np.float32)
    if axis == TENSOR:
        return np.array([a.max() if a.size else 0.0], dtype=np.float32)
    raise ValueError("axis")


def scales(amax: np.ndarray, bits: int):
    """lambda = fl32(qmax / a_max) and its inverse step s = fl32(a_max / qmax).

    Eq. (quantA).  Both are one IEEE single division.  A row/column whose a_max
    is zero (or below 1e-30) gets lambda = s = 0: all its codes are 0.
    """
    amax = np.asarray(amax, dtype=np.float32)
    q = np.float32(qmax_of(bits))
    live = amax >= _TINY_AMAX
    safe = np.where(live, amax, np.float32(1.0)).astype(np.float32)
    lam = np.where(live, q / safe, np.float32(0.0)).astype(np.float32)
    s = np.where(live, safe / q, np.float32(0.0)).astype(np.float32)
    return lam, s


def _broadcast(v: np.ndarray, axis: int, shape):
    if axis == ROWWISE:
        return v.reshape(shape[0], 1)
    if axis == COLWISE:
        return v.reshape(1, shape[1])
    return v.reshape(1, 1)


def quantize(X: np.ndarray, amax: np.ndarray, axis: int, bits: int,
             round_mode: int = FLOOR) -> np.ndarray:
    """Codes a_int = cast(lambda * a) clamped to [-qmax-1, qmax], as int8.

    t = fl32(lambda * x) is one single-precision multiply; FLOOR takes
    floor(t) (Eq. (get_ra2)), NEAREST rounds ties to even (Eq. (quantAB)).
    Returned array has X's shape (no transposition).
    """
    X = np.asarray(X, dtype=np.float32)
    q = qmax_of(bits)
    lam, _ = scales(amax, bits)
    t = (_broadcast(lam, axis, X.shape) * X).astype(np.float32)
    if round_mode == FLOOR:
        c = np.floor(t)
    elif round_mode == NEAREST:
        c = np.rint(t)
    else:
        raise ValueError("round_mode")
    c = np.clip(c, -q - 1, q)
    return c.astype(np.int8)


# --------------------------------------------------------------------------
# Integer GEMM and dequantization (Eq. (INTGEMM), Eq. (QUANTGEMM); Alg. 2, integer product and dequantization steps)
# --------------------------------------------------------------------------
def int_gemm(Aq: np.ndarray, Bq: np.ndarray) -> np.ndarray:
    """C_int = A_int . B_int accumulated in int64; must fit int32."""
    C = np.asarray(Aq, dtype=np.int64) @ np.asarray(Bq, dtype=np.int64)
    if C.size and (C.max() > 2**31 - 1 or C.min() < -2**31):
        raise OverflowError("integer product does not fit int32")
    return C


def dequant(Cint: np.ndarray, sA: np.ndarray, sB: np.ndarray) -> np.ndarray:
    """C_F = C_int / (lambda_A lambda_B), in per-row / per-column form C_int * sA_i * sB_j."""
    sA = np.asarray(sA, dtype=np.float64).reshape(-1, 1)
    sB = np.asarray(sB, dtype=np.float64).reshape(1, -1)
    return Cint.astype(np.float64) * sA * sB


def dequant_matrix(codes: np.ndarray, s: np.ndarray, axis: int) -> np.ndarray:
    """A_F = Dequant(A_int) (Alg. 2, operand dequantization step), float64."""
    return codes.astype(np.float64) * _broadcast(np.asarray(s, np.float64), axis, codes.shape)


def residual(X: np.ndarray, codes: np.ndarray, s: np.ndarray, axis: int) -> np.ndarray:
    """R = X - Dequant(Quant(X)) (Eq. (AFP); Alg. 2, residual step), float64, exact."""
    return np.asarray(X, dtype=np.float64) - dequant_matrix(codes, s, axis)


# --------------------------------------------------------------------------
# Counter-based Gaussian sketch.  The paper leaves the sampling to the RSVD
# literature it cites (Background 2.1, "various sampling techniques"); this
# build draws i.i.d. N(0,1) entries.  Element (i, j) of stream `stream` under
# `seed` depends only on (seed, stream, i, j), so any sub-block can be produced
# independently.  Every step is an exactly rounded IEEE operation in a fixed
# order (integer mixing, then float64 + - * / only), so a second implementation
# that follows the same steps produces the same float32 bits.
# --------------------------------------------------------------------------
_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function (Steele, Lea, Flood 2014) on uint64 arrays."""
    with np.errstate(over="ignore"):
        z = (z + _GOLD) & _M64
        z = ((z ^ (z >> np.uint64(30))) * _C1) & _M64
        z = ((z ^ (z >> np.uint64(27))) * _C2) & _M64
        return z ^ (z >> np.uint64(31))


_LN2 = 0.6931471805599453
_TWO_PI = 6.283185307179586
_SQRT_HALF = 0.7071067811865476


def _det_log(k: np.ndarray) -> np.ndarray:
    """ln(k / 2^24) for integer k in [1, 2^24], float64, fixed operation order.

    k = m 2^e with m in [sqrt(1/2), sqrt(2)); ln m = 2 atanh((m-1)/(m+1)) by its
    odd power series through s^21 (Horner).
    """
    m, e = np.frexp(k.astype(np.float64))          # m in [0.5, 1)
    small = m < _SQRT_HALF
    m = np.where(small, m * 2.0, m)
    e = np.where(small, e - 1, e)
    s = (m - 1.0) / (m + 1.0)
    s2 = s * s
    p = np.full_like(s, 1.0 / 21.0)
    for d in (19.0, 17.0, 15.0, 13.0, 11.0, 9.0, 7.0, 5.0, 3.0):
        p = p * s2 + 1.0 / d
    p = p * s2 + 1.0
    lnm = (2.0 * s) * p
    return lnm + (e - 24).astype(np.float64) * _LN2


def _det_sincos(x: np.ndarray):
    """sin and cos of x in [0, pi/4] by Taylor polynomials through x^17 / x^16."""
    x2 = x * x
    ps = np.full_like(x, 1.0 / 355687428096000.0)            # 1/17!
    for f in (-1.0 / 1307674368000.0, 1.0 / 6227020800.0, -1.0 / 39916800.0,
              1.0 / 362880.0, -1.0 / 5040.0, 1.0 / 120.0, -1.0 / 6.0, 1.0):
        ps = ps * x2 + f
    pc = np.full_like(x, 1.0 / 20922789888000.0)             # 1/16!
    for f in (-1.0 / 87178291200.0, 1.0 / 479001600.0, -1.0 / 3628800.0,
              1.0 / 40320.0, -1.0 / 720.0, 1.0 / 24.0, -1.0 / 2.0, 1.0):
        pc = pc * x2 + f
    return x * ps, pc


def _det_sqrt(x: np.ndarray) -> np.ndarray:
    """sqrt by two Heron steps from the single-precision square root; 0 -> 0."""
    y0 = np.sqrt(x.astype(np.float32)).astype(np.float64)
    ok = y0 > 0.0
    y0s = np.where(ok, y0, 1.0)
    y1 = 0.5 * (y0s + x / y0s)
    y2 = 0.5 * (y1 + x / y1)
    return np.where(ok, y2, 0.0)


def gaussian_sketch(seed: int, stream: int, rows: int, cols: int) -> np.ndarray:
    """Omega (rows x cols) float32 with i.i.d. N(0,1) entries.

    h = mix64(mix64(seed + GOLD*(stream+1)) + (i << 32 | j)); the top 24 bits give
    u1 = (k1+1)/2^24 in (0,1], the next 24 bits u2 = k2/2^24 in [0,1);
    z = sqrt(-2 ln u1) cos(2 pi u2)  (Box-Muller), cos by octant reduction on k2.
    """
    i = np.arange(rows, dtype=np.uint64).reshape(-1, 1)
    j = np.arange(cols, dtype=np.uint64).reshape(1, -1)
    with np.errstate(over="ignore"):
        key = _mix64(np.array([(np.uint64(seed & 0xFFFFFFFFFFFFFFFF)
                                + _GOLD * np.uint64(stream + 1)) & _M64], dtype=np.uint64))[0]
        ctr = (i << np.uint64(32)) | j
        h = _mix64((ctr + key) & _M64)
    k1 = (h >> np.uint64(40)).astype(np.int64) + 1                 # 1 .. 2^24
    k2 = ((h >> np.uint64(16)) & np.uint64(0xFFFFFF)).astype(np.int64)  # 0 .. 2^24-1
    x = -2.0 * _det_log(k1)
    rad = _det_sqrt(x)
    octant = k2 >> 21
    rem = k2 & ((1 << 21) - 1)
    odd = (octant & 1) == 1
    r = np.where(odd, (1 << 21) - rem, rem).astype(np.float64)
    phi = _TWO_PI * (r / 16777216.0)
    sn, cs = _det_sincos(phi)
    # cos(2 pi (octant/8) + ...) in terms of sin/cos of the reduced angle
    use_sin = (octant == 1) | (octant == 2) | (octant == 5) | (octant == 6)
    neg = (octant >= 2) & (octant <= 5)
    t = np.where(use_sin, sn, cs)
    t = np.where(neg, -t, t)
    return (rad * t).astype(np.float32)


# --------------------------------------------------------------------------
# Randomized SVD (Background 2.1, two-stage description and Algorithm 1; error
# bound Eq. (rsvderror) for the role of power iterations q)
# --------------------------------------------------------------------------
def orth(Y: np.ndarray) -> np.ndarray:
    """Orthonormal basis of range(Y) (stage 1 of the RSVD description)."""
    Q, _ = np.linalg.qr(np.asarray(Y, dtype=np.float64), mode="reduced")
    return Q


def range_finder(R: np.ndarray, omega: np.ndarray, power_iters: int) -> np.ndarray:
    """Q with l orthonormal columns, R ~ Q Q^T R.

    Y = R Omega, then `power_iters` rounds of Z = orth(R^T Q), Q = orth(R Z),
    re-orthonormalizing after every product.
    """
    R = np.asarray(R, dtype=np.float64)
    Q = orth(R @ np.asarray(omega, dtype=np.float64))
    for _ in range(power_iters):
        Z = orth(R.T @ Q)
        Q = orth(R @ Z)
    return Q


def rsvd(R: np.ndarray, rank: int, omega: np.ndarray, power_iters: int = 0):
    """Algorithm 1 with truncation to `rank` (Eq. (k-svd)).

    B = Q^T R; B = U' S V^T; U = Q U'.  omega has l = rank + oversample columns;
    the l-term factorization is truncated to its `rank` largest singular values.
    Returns U (rows x rank), S (rank), Vt (rank x cols), float64.
    """
    R = np.asarray(R, dtype=np.float64)
    ell = omega.shape[1]
    if not (0 < rank <= ell <= min(R.shape)):
        raise ValueError("need 0 < rank <= rank+oversample <= min(rows, cols)")
    if omega.shape[0] != R.shape[1]:
        raise ValueError("omega must be cols x l")
    Q = range_finder(R, omega, power_iters)
    Bsm = Q.T @ R
    Up, S, Vt = np.linalg.svd(Bsm, full_matrices=False)
    U = Q @ Up[:, :rank]
    return U, S[:rank].copy(), Vt[:rank].copy()


# --------------------------------------------------------------------------
# LRQMM (Methodology, Algorithm 2)
# --------------------------------------------------------------------------
STREAM_A = 0   # sketch stream for R_A
STREAM_B = 1   # sketch stream for R_B


def lrqmm(A: np.ndarray, B: np.ndarray, bits: int, rank: int, oversample: int = 0,
          power_iters: int = 0, seed: int = 0, round_mode: int = FLOOR,
          per_tensor: bool = False, omega_a: np.ndarray | None = None,
          omega_b: np.ndarray | None = None, want_cint: bool = True,
          row_sample: np.ndarray | None = None) -> dict:
    """Algorithm 2 step by step (its final alpha/beta update excluded).

    rank == 0 gives the direct-quantization product only (first term of
    Eq. (gemm_r_split)).  Returns every intermediate by name.

    row_sample: optional row indices of C.  Quantization and both residual
    factorizations always use the full operands; with a sample the M x N
    outputs (Cint, C0, C) hold only those rows (rows of C are independent
    given the factors), which keeps full-size checks affordable.
    """
    A = np.asarray(A, dtype=np.float32)
    B = np.asarray(B, dtype=np.float32)
    M, K = A.shape
    K2, N = B.shape
    if K != K2:
        raise ValueError("shape")
    ax_a, ax_b = (TENSOR, TENSOR) if per_tensor else (ROWWISE, COLWISE)
    out = {}
    # quantize both operands
    amax_a, amax_b = absmax(A, ax_a), absmax(B, ax_b)
    _, sa = scales(amax_a, bits)
    _, sb = scales(amax_b, bits)
    Aq = quantize(A, amax_a, ax_a, bits, round_mode)
    Bq = quantize(B, amax_b, ax_b, bits, round_mode)
    sa_rows = np.broadcast_to(sa, (M,)) if per_tensor else sa
    sb_cols = np.broadcast_to(sb, (N,)) if per_tensor else sb
    out.update(amax_a=amax_a, amax_b=amax_b, sa=sa, sb=sb, Aq=Aq, Bq=Bq)
    # integer product and its dequantization
    sel = slice(None) if row_sample is None else np.asarray(row_sample, dtype=np.int64)
    Cint = int_gemm(Aq[sel], Bq)
    C0 = dequant(Cint, np.asarray(sa_rows)[sel], sb_cols)
    if want_cint:
        out["Cint"] = Cint
    out["C0"] = C0
    if rank == 0:
        out["C"] = C0
        return out
    # dequantized operands and residuals
    Af = dequant_matrix(Aq, sa, ax_a)
    Bf = dequant_matrix(Bq, sb, ax_b)
    Ra = A.astype(np.float64) - Af
    Rb = B.astype(np.float64) - Bf
    # rank-r factorizations of the residuals (RSVD)
    ell = rank + oversample
    if omega_a is None:
        omega_a = gaussian_sketch(seed, STREAM_A, K, ell)
    if omega_b is None:
        omega_b = gaussian_sketch(seed, STREAM_B, N, ell)
    U, Sig, Vt = rsvd(Ra, rank, omega_a, power_iters)
    W, Gam, Zt = rsvd(Rb, rank, omega_b, power_iters)
    # fold the singular values into the left factors
    Ut = U * Sig.reshape(1, -1)
    Ztp = Gam.reshape(-1, 1) * Zt
    # the three compensation terms
    RC1 = Ut[sel] @ (Vt @ Bf)
    RC2 = (Af[sel] @ W) @ Ztp
    RC3 = (Ut[sel] @ (Vt @ W)) @ Ztp
    # sum of the dequantized product and the compensation terms
    C = C0 + RC1 + RC2 + RC3
    out.update(Ra=Ra, Rb=Rb, omega_a=omega_a, omega_b=omega_b, U=U, Sig=Sig, Vt=Vt,
               W=W, Gam=Gam, Zt=Zt, Af=Af, Bf=Bf, C=C)
    return out


def compensate(Aq, sa, Bq, sb, U, Sig, Vt, W, Gam, Zt) -> np.ndarray:
    """Alg. 2 integer product, dequantization and compensation steps from given codes, steps and factors (row/column scales)."""
    Af = dequant_matrix(Aq, sa, ROWWISE)
    Bf = dequant_matrix(Bq, sb, COLWISE)
    C0 = dequant(int_gemm(Aq, Bq), sa, sb)
    if U is None:
        return C0
    Ut = np.asarray(U, np.float64) * np.asarray(Sig, np.float64).reshape(1, -1)
    Ztp = np.asarray(Gam, np.float64).reshape(-1, 1) * np.asarray(Zt, np.float64)
    Vt = np.asarray(Vt, np.float64)
    W = np.asarray(W, np.float64)
    return C0 + Ut @ (Vt @ Bf) + (Af @ W) @ Ztp + (Ut @ (Vt @ W)) @ Ztp


def residual_compensation(A: np.ndarray, B: np.ndarray, bits: int, terms: int, round_mode: int = FLOOR,
                          per_tensor: bool = False, row_sample: np.ndarray | None = None) -> dict:
    """Complete residual compensation, Eq. (gemm_r_split): the residuals are quantized a second
    time, with scales of their own, and the product is the sum of the first `terms` of

        A~ B~  +  A~ R~_B  +  R~_A B~  +  R~_A R~_B

    (terms = 1: direct quantization; 3: the three terms called QT(1,1,0) in the Evaluation;
    4: all four, QT(1,1,1)).  Each term is an integer product dequantized with the two scales of
    its operands.  The residual that is quantized is the float32 value fl32(x - code * s) (the
    exact difference rounded once), so that its codes are defined by float32 operations only.
    """
    if terms not in (1, 3, 4):
        raise ValueError("terms must be 1, 3 or 4")
    A = np.asarray(A, dtype=np.float32)
    B = np.asarray(B, dtype=np.float32)
    ax_a, ax_b = (TENSOR, TENSOR) if per_tensor else (ROWWISE, COLWISE)
    out = {}

    def two_levels(X, axis):
        amax = absmax(X, axis)
        _, s = scales(amax, bits)
        q = quantize(X, amax, axis, bits, round_mode)
        r = residual(X, q, s, axis).astype(np.float32)
        amax_r = absmax(r, axis)
        _, s_r = scales(amax_r, bits)
        q_r = quantize(r, amax_r, axis, bits, round_mode)
        return amax, s, q, r, amax_r, s_r, q_r

    amax_a, sa, Aq, Ra, amax_ra, sra, RAq = two_levels(A, ax_a)
    amax_b, sb, Bq, Rb, amax_rb, srb, RBq = two_levels(B, ax_b)
    M, N = A.shape[0], B.shape[1]
    bc = lambda v, n: np.broadcast_to(np.asarray(v, dtype=np.float32), (n,))
    sa_r, sra_r, sb_c, srb_c = bc(sa, M), bc(sra, M), bc(sb, N), bc(srb, N)
    sel = slice(None) if row_sample is None else np.asarray(row_sample, dtype=np.int64)
    T = [dequant(int_gemm(Aq[sel], Bq), sa_r[sel], sb_c)]
    if terms >= 3:
        T.append(dequant(int_gemm(Aq[sel], RBq), sa_r[sel], srb_c))
        T.append(dequant(int_gemm(RAq[sel], Bq), sra_r[sel], sb_c))
    if terms == 4:
        T.append(dequant(int_gemm(RAq[sel], RBq), sra_r[sel], srb_c))
    C = T[0]
    for t in T[1:]:
        C = C + t
    out.update(amax_a=amax_a, amax_b=amax_b, amax_ra=amax_ra, amax_rb=amax_rb, sa=sa, sb=sb, sra=sra, srb=srb,
               Aq=Aq, Bq=Bq, RAq=RAq, RBq=RBq, Ra=Ra, Rb=Rb, terms=T, C0=T[0], C=C)
    return out


def scaled_update(C_F: np.ndarray, alpha: float, beta: float, D: np.ndarray | None) -> np.ndarray:
    """Last step of Algorithm 2: D <- alpha * C_F + beta * D, in float64.

    alpha and beta are float32 scalars (the origin precision of the algorithm's
    inputs).  With beta == 0 the old contents of D are not read at all, as in
    the BLAS convention the algorithm's caption (D = alpha A.B + beta D) borrows,
    so D may then be None or hold anything.
    """
    a = float(np.float32(alpha))
    b = float(np.float32(beta))
    out = a * np.asarray(C_F, dtype=np.float64)
    if b != 0.0:
        if D is None:
            raise ValueError("beta != 0 needs D")
        D = np.asarray(D, dtype=np.float32).astype(np.float64)
        if D.shape != out.shape:
            raise ValueError("shape")
        out = out + b * D
    return out


def rel_err(C_ref: np.ndarray, X: np.ndarray) -> float:
    """Relative error in the Frobenius norm (Evaluation, Precision test)."""
    C_ref = np.asarray(C_ref, dtype=np.float64)
    d = np.linalg.norm(C_ref)
    n = np.linalg.norm(C_ref - np.asarray(X, dtype=np.float64))
    return float(n / d) if d > 0 else float(n)


def exact_product(A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """C_ref = A . B in float64 from the float32 inputs."""
    return np.asarray(A, dtype=np.float64) @ np.asarray(B, dtype=np.float64)
