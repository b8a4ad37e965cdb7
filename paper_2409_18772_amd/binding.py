"""ctypes binding of include/lrqmm.h.  Same names as the C entry points.

torch is used for device memory and the current stream only.
"""
from __future__ import annotations

import ctypes
import os

AXIS_ROW, AXIS_COL = 0, 1
ROUND_FLOOR, ROUND_NEAREST = 0, 1
SCALE_VECTOR, SCALE_TENSOR = 0, 1
PREC_FP32, PREC_BF16X2, PREC_BF16, PREC_SUBSPACE_BF16X2 = 0, 1, 2, 3
MAX_SKETCH = 80

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTS = ("lrqmm_status_string", "lrqmm_workspace_bytes", "lrqmm_quantize", "lrqmm_fill_sketch",
           "lrqmm_rsvd", "lrqmm_gemm", "lrqmm_matmul", "lrqmm_profile_enable", "lrqmm_profile_read",
           "lrqmm_quantize_ex", "lrqmm_rsvd_ex", "lrqmm_gemm_ex", "lrqmm_matmul_ex",
           "lrqmm_quantize_residual", "lrqmm_residual_workspace_bytes", "lrqmm_residual_matmul",
           "lrqmm_gemm_static")
PROF_STAGES = ("quantize_a", "rsvd_a", "quantize_b", "rsvd_b", "panels", "gemm", "int_gemm")


class LrqmmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lrqmm_status_string(status)} ({status})")


def lib_path() -> str:
    return os.path.join(_HERE, "liblrqmm.so")


def load_library() -> ctypes.CDLL:
    """Load liblrqmm.so (built in-tree by paper_2409_18772_amd/build.py); never falls back."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: run `python -m paper_2409_18772_amd.build` "
                          "(or __graft_entry__.build()) first; there is no CPU fallback")
    lib = ctypes.CDLL(path)
    c_int, c_vp, c_sz, c_u64 = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64
    lib.lrqmm_status_string.restype = ctypes.c_char_p
    lib.lrqmm_status_string.argtypes = [c_int]
    lib.lrqmm_workspace_bytes.restype = c_sz
    lib.lrqmm_workspace_bytes.argtypes = [c_int] * 5
    lib.lrqmm_quantize.restype = c_int
    lib.lrqmm_quantize.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp]
    lib.lrqmm_fill_sketch.restype = c_int
    lib.lrqmm_fill_sketch.argtypes = [c_u64, c_int, c_int, c_int, c_vp, c_vp]
    lib.lrqmm_rsvd.restype = c_int
    lib.lrqmm_rsvd.argtypes = [c_vp, c_vp, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_int,
                               c_u64, c_vp, c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    lib.lrqmm_gemm.restype = c_int
    lib.lrqmm_gemm.argtypes = [c_int] * 5 + [c_vp] * 12 + [c_vp, c_sz, c_vp]
    lib.lrqmm_matmul.restype = c_int
    lib.lrqmm_matmul.argtypes = [c_int] * 7 + [c_u64, c_int, c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    c_f = ctypes.c_float
    lib.lrqmm_quantize_ex.restype = c_int
    lib.lrqmm_quantize_ex.argtypes = [c_vp] + [c_int] * 7 + [c_vp, c_vp, c_vp]
    lib.lrqmm_rsvd_ex.restype = c_int
    lib.lrqmm_rsvd_ex.argtypes = [c_vp, c_int, c_vp] + [c_int] * 8 + [c_u64, c_vp, c_int, c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    lib.lrqmm_gemm_ex.restype = c_int
    lib.lrqmm_gemm_ex.argtypes = [c_int] * 5 + [c_vp] * 10 + [c_f, c_f, c_vp, c_int, c_vp, c_vp, c_sz, c_vp]
    lib.lrqmm_gemm_static.restype = c_int
    lib.lrqmm_gemm_static.argtypes = [c_int] * 5 + [c_vp] * 10 + [c_f, c_f, c_vp, c_int, c_vp, c_vp]
    lib.lrqmm_matmul_ex.restype = c_int
    lib.lrqmm_matmul_ex.argtypes = [c_int] * 7 + [c_u64, c_int, c_int, c_int, c_vp, c_int, c_vp, c_int, c_f, c_f, c_vp,
                                    c_int, c_vp, c_sz, c_vp]
    lib.lrqmm_quantize_residual.restype = c_int
    lib.lrqmm_quantize_residual.argtypes = [c_vp, c_int, c_vp] + [c_int] * 6 + [c_vp, c_vp, c_vp]
    lib.lrqmm_residual_workspace_bytes.restype = c_sz
    lib.lrqmm_residual_workspace_bytes.argtypes = [c_int] * 3
    lib.lrqmm_residual_matmul.restype = c_int
    lib.lrqmm_residual_matmul.argtypes = [c_int] * 7 + [c_vp, c_int, c_vp, c_int, c_f, c_f, c_vp, c_int, c_vp, c_sz,
                                          c_vp]
    lib.lrqmm_profile_enable.restype = c_int
    lib.lrqmm_profile_enable.argtypes = [c_int]
    lib.lrqmm_profile_read.restype = c_int
    lib.lrqmm_profile_read.argtypes = [c_vp, c_vp]
    _LIB = lib
    return lib


def lrqmm_status_string(status: int) -> str:
    return load_library().lrqmm_status_string(int(status)).decode()


def lrqmm_workspace_bytes(M: int, N: int, K: int, rank: int, oversample: int) -> int:
    return int(load_library().lrqmm_workspace_bytes(M, N, K, rank, oversample))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != 0:
        raise LrqmmError(status, where)


def _dev(t, dtype, name):
    import torch
    if t is None:
        return
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous CUDA tensor of dtype {dtype}")


def _dev2d(t, dtype, name) -> int:
    """A 2-D CUDA tensor whose rows are contiguous (a window of a row-major array); returns its row stride."""
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.dim() == 2):
        raise TypeError(f"{name}: expected a 2-D CUDA tensor of dtype {dtype}")
    rows, cols = t.shape
    if cols > 1 and t.stride(1) != 1:
        raise TypeError(f"{name}: elements of a row must be adjacent")
    ld = t.stride(0) if rows > 1 else max(cols, t.stride(0))
    if ld < cols:
        raise TypeError(f"{name}: row stride below the row length")
    return int(ld)


class Workspace:
    """A 256-byte aligned device buffer (a torch uint8 tensor) handed to the library."""

    def __init__(self, nbytes: int, device="cuda"):
        import torch
        self.nbytes = int(nbytes)
        self._buf = torch.empty(self.nbytes + 256, dtype=torch.uint8, device=device)
        base = self._buf.data_ptr()
        self.ptr = (base + 255) // 256 * 256

    @classmethod
    def for_problem(cls, M, N, K, rank, oversample, device="cuda"):
        return cls(lrqmm_workspace_bytes(M, N, K, rank, oversample), device)


def lrqmm_quantize(X, axis: int, bits: int, round_mode: int = ROUND_FLOOR, codes=None, amax=None):
    """codes (int8; transposed for AXIS_COL) and amax (float32) of X (rows x cols float32)."""
    import torch
    _dev(X, torch.float32, "X")
    rows, cols = X.shape
    if codes is None:
        shape = (rows, cols) if axis == AXIS_ROW else (cols, rows)
        codes = torch.empty(shape, dtype=torch.int8, device=X.device)
    if amax is None:
        amax = torch.empty(rows if axis == AXIS_ROW else cols, dtype=torch.float32, device=X.device)
    _dev(codes, torch.int8, "codes")
    _dev(amax, torch.float32, "amax")
    st = load_library().lrqmm_quantize(_ptr(X), rows, cols, axis, bits, round_mode, _ptr(codes),
                                       _ptr(amax), _stream())
    _check(st, "lrqmm_quantize")
    return codes, amax


def lrqmm_quantize_ex(X, axis: int, bits: int, round_mode: int = ROUND_FLOOR, scale_mode: int = SCALE_VECTOR,
                      codes=None, amax=None):
    """lrqmm_quantize for a row-strided X and a choice of scale granularity."""
    import torch
    ldx = _dev2d(X, torch.float32, "X")
    rows, cols = X.shape
    if codes is None:
        shape = (rows, cols) if axis == AXIS_ROW else (cols, rows)
        codes = torch.empty(shape, dtype=torch.int8, device=X.device)
    if amax is None:
        amax = torch.empty(rows if axis == AXIS_ROW else cols, dtype=torch.float32, device=X.device)
    _dev(codes, torch.int8, "codes")
    _dev(amax, torch.float32, "amax")
    st = load_library().lrqmm_quantize_ex(_ptr(X), ldx, rows, cols, axis, bits, round_mode, scale_mode,
                                          _ptr(codes), _ptr(amax), _stream())
    _check(st, "lrqmm_quantize_ex")
    return codes, amax


def lrqmm_quantize_residual(X, amax0, axis: int, bits: int, round_mode: int = ROUND_FLOOR,
                            scale_mode: int = SCALE_VECTOR):
    """Second-level codes and maxima of X's quantization residual (amax0: first-level maxima)."""
    import torch
    ldx = _dev2d(X, torch.float32, "X")
    _dev(amax0, torch.float32, "amax0")
    rows, cols = X.shape
    if amax0.numel() != (rows if axis == AXIS_ROW else cols):
        raise ValueError("amax0 must hold one maximum per scale group")
    shape = (rows, cols) if axis == AXIS_ROW else (cols, rows)
    codes = torch.empty(shape, dtype=torch.int8, device=X.device)
    amax = torch.empty_like(amax0)
    st = load_library().lrqmm_quantize_residual(_ptr(X), ldx, _ptr(amax0), rows, cols, axis, bits, round_mode,
                                                scale_mode, _ptr(codes), _ptr(amax), _stream())
    _check(st, "lrqmm_quantize_residual")
    return codes, amax


def lrqmm_residual_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load_library().lrqmm_residual_workspace_bytes(M, N, K))


def lrqmm_residual_matmul(A, B, D, bits: int, terms: int, round_mode: int = ROUND_FLOOR,
                          scale_mode: int = SCALE_VECTOR, alpha: float = 1.0, beta: float = 0.0,
                          workspace: Workspace | None = None):
    """Complete residual compensation: D <- alpha (first `terms` terms of Eq. (gemm_r_split)) + beta D."""
    import torch
    lda = _dev2d(A, torch.float32, "A")
    ldb = _dev2d(B, torch.float32, "B")
    ldd = _dev2d(D, torch.float32, "D")
    M, K = A.shape
    K2, N = B.shape
    if K != K2 or tuple(D.shape) != (M, N):
        raise ValueError("A is M x K, B is K x N, D is M x N")
    if workspace is None:
        workspace = Workspace(lrqmm_residual_workspace_bytes(M, N, K), A.device)
    st = load_library().lrqmm_residual_matmul(M, N, K, bits, terms, round_mode, scale_mode, _ptr(A), lda, _ptr(B),
                                              ldb, float(alpha), float(beta), _ptr(D), ldd,
                                              ctypes.c_void_p(workspace.ptr), workspace.nbytes, _stream())
    _check(st, "lrqmm_residual_matmul")
    return D


def lrqmm_fill_sketch(seed: int, stream_id: int, rows: int, cols: int, device="cuda"):
    import torch
    omega = torch.empty((rows, cols), dtype=torch.float32, device=device)
    st = load_library().lrqmm_fill_sketch(seed & 0xFFFFFFFFFFFFFFFF, stream_id, rows, cols, _ptr(omega),
                                          _stream())
    _check(st, "lrqmm_fill_sketch")
    return omega


def _rsvd_args(X, amax, omega, rank: int, oversample: int, workspace, strided: bool):
    """Checks shared by the two factorization entry points; allocates the outputs and, if none is given, a workspace."""
    import torch
    ldx = _dev2d(X, torch.float32, "X") if strided else None
    if not strided:
        _dev(X, torch.float32, "X")
    _dev(amax, torch.float32, "amax")
    _dev(omega, torch.float32, "omega")
    rows, cols = X.shape
    if omega is not None and tuple(omega.shape) != (cols, rank + oversample):
        raise ValueError("omega must be cols x (rank + oversample)")
    U = torch.empty((rows, rank), dtype=torch.float32, device=X.device)
    Sigma = torch.empty((rank,), dtype=torch.float32, device=X.device)
    Vt = torch.empty((rank, cols), dtype=torch.float32, device=X.device)
    if workspace is None:
        workspace = Workspace.for_problem(max(rows, cols), max(rows, cols), max(rows, cols), rank, oversample)
    return ldx, rows, cols, U, Sigma, Vt, workspace


def lrqmm_rsvd(X, amax, axis: int, bits: int, rank: int, oversample: int = 0, power_iters: int = 0,
               seed: int = 0, round_mode: int = ROUND_FLOOR, omega=None, workspace: Workspace | None = None):
    """U (rows x rank), Sigma (rank), Vt (rank x cols) of the residual of X."""
    _, rows, cols, U, Sigma, Vt, workspace = _rsvd_args(X, amax, omega, rank, oversample, workspace, False)
    st = load_library().lrqmm_rsvd(_ptr(X), _ptr(amax), rows, cols, axis, bits, round_mode, rank, oversample,
                                   power_iters, seed & 0xFFFFFFFFFFFFFFFF, _ptr(omega), _ptr(U), _ptr(Sigma),
                                   _ptr(Vt), ctypes.c_void_p(workspace.ptr), workspace.nbytes, _stream())
    _check(st, "lrqmm_rsvd")
    return U, Sigma, Vt


def lrqmm_rsvd_ex(X, amax, axis: int, bits: int, rank: int, oversample: int = 0, power_iters: int = 0,
                  seed: int = 0, round_mode: int = ROUND_FLOOR, omega=None, workspace: Workspace | None = None,
                  precision: int = PREC_FP32):
    """lrqmm_rsvd for a row-strided X, with a choice of arithmetic for the residual products."""
    ldx, rows, cols, U, Sigma, Vt, workspace = _rsvd_args(X, amax, omega, rank, oversample, workspace, True)
    st = load_library().lrqmm_rsvd_ex(_ptr(X), ldx, _ptr(amax), rows, cols, axis, bits, round_mode, rank,
                                      oversample, power_iters, seed & 0xFFFFFFFFFFFFFFFF, _ptr(omega),
                                      int(precision), _ptr(U), _ptr(Sigma), _ptr(Vt),
                                      ctypes.c_void_p(workspace.ptr), workspace.nbytes, _stream())
    _check(st, "lrqmm_rsvd_ex")
    return U, Sigma, Vt


def _gemm_args(Aq, amaxA, BqT, amaxB, factors_a, factors_b, want_cint: bool):
    """Checks shared by the three product entry points: shapes, the six factor tensors (or none), the optional
    int32 output.  Returns (M, N, K, rank, [U, Sig, Vt, W, Gam, Zt], Cint)."""
    import torch
    _dev(Aq, torch.int8, "Aq")
    _dev(BqT, torch.int8, "BqT")
    _dev(amaxA, torch.float32, "amaxA")
    _dev(amaxB, torch.float32, "amaxB")
    M, K = Aq.shape
    N, K2 = BqT.shape
    if K != K2:
        raise ValueError("Aq is M x K and BqT is N x K")
    rank = 0
    factors = [None] * 6
    if factors_a is not None:
        U, Sig, Vt = factors_a
        W, Gam, Zt = factors_b
        factors = [U, Sig, Vt, W, Gam, Zt]
        for n, t in zip(("U", "Sig", "Vt", "W", "Gam", "Zt"), factors):
            _dev(t, torch.float32, n)
        rank = Sig.numel()
        if tuple(U.shape) != (M, rank) or tuple(Vt.shape) != (rank, K) or tuple(W.shape) != (K, rank) \
                or tuple(Zt.shape) != (rank, N) or Gam.numel() != rank:
            raise ValueError("factor shapes")
    Cint = torch.empty((M, N), dtype=torch.int32, device=Aq.device) if want_cint else None
    return M, N, K, rank, factors, Cint


def _strided_output(D, M: int, N: int) -> int:
    import torch
    ldd = _dev2d(D, torch.float32, "D")
    if tuple(D.shape) != (M, N):
        raise ValueError("D must be M x N")
    return ldd


def lrqmm_gemm_ex(Aq, amaxA, BqT, amaxB, bits: int, D, alpha: float = 1.0, beta: float = 0.0, factors_a=None,
                  factors_b=None, want_cint: bool = False, workspace: Workspace | None = None):
    """D <- alpha (deq(Aq . Bq) + compensation) + beta D, in place in the (row-strided) tensor D."""
    M, N, K, rank, f, Cint = _gemm_args(Aq, amaxA, BqT, amaxB, factors_a, factors_b, want_cint)
    ldd = _strided_output(D, M, N)
    if workspace is None:
        workspace = Workspace.for_problem(M, N, K, rank, 0)
    st = load_library().lrqmm_gemm_ex(M, N, K, bits, rank, _ptr(Aq), _ptr(amaxA), _ptr(BqT), _ptr(amaxB),
                                      *map(_ptr, f), float(alpha), float(beta), _ptr(D), ldd, _ptr(Cint),
                                      ctypes.c_void_p(workspace.ptr), workspace.nbytes, _stream())
    _check(st, "lrqmm_gemm_ex")
    return (D, Cint) if want_cint else D


STATIC_SCRATCH_BYTES = 16 << 20
ERR_STATIC_LIMIT = -5


def lrqmm_gemm_static(Aq, amaxA, BqT, amaxB, bits: int, D, alpha: float = 1.0, beta: float = 0.0, factors_a=None,
                      factors_b=None, want_cint: bool = False):
    """lrqmm_gemm_ex on the library's static scratch buffer: no workspace, nothing allocated by the call
    itself (the optional int32 output is the caller's choice)."""
    M, N, K, rank, f, Cint = _gemm_args(Aq, amaxA, BqT, amaxB, factors_a, factors_b, want_cint)
    ldd = _strided_output(D, M, N)
    st = load_library().lrqmm_gemm_static(M, N, K, bits, rank, _ptr(Aq), _ptr(amaxA), _ptr(BqT), _ptr(amaxB),
                                          *map(_ptr, f), float(alpha), float(beta), _ptr(D), ldd, _ptr(Cint),
                                          _stream())
    _check(st, "lrqmm_gemm_static")
    return (D, Cint) if want_cint else D


def lrqmm_gemm(Aq, amaxA, BqT, amaxB, bits: int, factors_a=None, factors_b=None, want_cint: bool = False,
               workspace: Workspace | None = None, C=None):
    """C = deq(Aq . Bq) + compensation; factors_a = (U, Sig, Vt), factors_b = (W, Gam, Zt) or None."""
    import torch
    M, N, K, rank, f, Cint = _gemm_args(Aq, amaxA, BqT, amaxB, factors_a, factors_b, want_cint)
    if C is None:
        C = torch.empty((M, N), dtype=torch.float32, device=Aq.device)
    if workspace is None:
        workspace = Workspace.for_problem(M, N, K, rank, 0)
    st = load_library().lrqmm_gemm(M, N, K, bits, rank, _ptr(Aq), _ptr(amaxA), _ptr(BqT), _ptr(amaxB),
                                   *map(_ptr, f), _ptr(C), _ptr(Cint), ctypes.c_void_p(workspace.ptr),
                                   workspace.nbytes, _stream())
    _check(st, "lrqmm_gemm")
    return (C, Cint) if want_cint else C


def lrqmm_matmul(A, B, bits: int, rank: int, oversample: int = 0, power_iters: int = 0, seed: int = 0,
                 round_mode: int = ROUND_FLOOR, workspace: Workspace | None = None, C=None):
    """The whole hot path: C ~ A . B (all of Algorithm 2 except its final alpha/beta update)."""
    import torch
    _dev(A, torch.float32, "A")
    _dev(B, torch.float32, "B")
    M, K = A.shape
    K2, N = B.shape
    if K != K2:
        raise ValueError("A is M x K and B is K x N")
    if C is None:
        C = torch.empty((M, N), dtype=torch.float32, device=A.device)
    if workspace is None:
        workspace = Workspace.for_problem(M, N, K, rank, oversample)
    st = load_library().lrqmm_matmul(M, N, K, bits, rank, oversample, power_iters, seed & 0xFFFFFFFFFFFFFFFF,
                                     round_mode, _ptr(A), _ptr(B), _ptr(C), ctypes.c_void_p(workspace.ptr),
                                     workspace.nbytes, _stream())
    _check(st, "lrqmm_matmul")
    return C


def lrqmm_matmul_ex(A, B, D, bits: int, rank: int, oversample: int = 0, power_iters: int = 0, seed: int = 0,
                    round_mode: int = ROUND_FLOOR, scale_mode: int = SCALE_VECTOR, alpha: float = 1.0,
                    beta: float = 0.0, workspace: Workspace | None = None, precision: int = PREC_FP32):
    """All of Algorithm 2: D <- alpha C_F + beta D in place; A, B, D may be row-strided windows."""
    import torch
    lda = _dev2d(A, torch.float32, "A")
    ldb = _dev2d(B, torch.float32, "B")
    ldd = _dev2d(D, torch.float32, "D")
    M, K = A.shape
    K2, N = B.shape
    if K != K2 or tuple(D.shape) != (M, N):
        raise ValueError("A is M x K, B is K x N, D is M x N")
    if workspace is None:
        workspace = Workspace.for_problem(M, N, K, rank, oversample)
    st = load_library().lrqmm_matmul_ex(M, N, K, bits, rank, oversample, power_iters, seed & 0xFFFFFFFFFFFFFFFF,
                                        round_mode, scale_mode, int(precision), _ptr(A), lda, _ptr(B), ldb, float(alpha),
                                        float(beta), _ptr(D), ldd, ctypes.c_void_p(workspace.ptr),
                                        workspace.nbytes, _stream())
    _check(st, "lrqmm_matmul_ex")
    return D


PROF_GEMM_ONLY = 2


def lrqmm_profile_enable(on):
    """False/0 off, True/1 all stages, PROF_GEMM_ONLY: only the events around the integer GEMM."""
    _check(load_library().lrqmm_profile_enable(int(on)), "lrqmm_profile_enable")


def lrqmm_profile_read():
    """Mean per-stage milliseconds of the lrqmm_matmul calls since the last read: (dict, ncalls)."""
    ms = (ctypes.c_float * len(PROF_STAGES))()
    n = ctypes.c_int(0)
    _check(load_library().lrqmm_profile_read(ctypes.cast(ms, ctypes.c_void_p),
                                              ctypes.cast(ctypes.byref(n), ctypes.c_void_p)),
           "lrqmm_profile_read")
    return dict(zip(PROF_STAGES, [float(x) for x in ms])), int(n.value)
