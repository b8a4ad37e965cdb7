"""Accuracy sweeps of the paper's Evaluation section on the GPU path, with synthetic inputs.

    python -m paper_2409_18772_amd.accuracy --sweep tables|rank|size|all [--size 2000] [--rank 10]

  tables  relative Frobenius error of direct quantization and of LRQMM for the six input
          distributions of Tables 3-4 (matrix size 2000, approximate rank 10, one scale per
          matrix), at 4 and 8 bits and at the 3- and 5-bit widths of Table 5, carried in int8
  rank    error against the approximate rank at size 200 (Evaluation, "Precision test", Fig. 3)
  size    error against the matrix size at rank 10 (same figure)

Every product runs through lrqmm_matmul_ex (rank 0 = direct quantization, the first term of
Eq. (gemm_r_split)).  torch only holds the device memory; the float64 reference product
C_ref = A.B and the two norms of the error metric |C_ref - X|_F / |C_ref|_F are numpy on the host;
nothing of the method itself is computed outside the library.  One JSON line per measurement.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

DISTRIBUTIONS = ("normal", "uniform01", "uniform_pm1", "exponential", "chisquare", "poisson")


def _workloads():
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    if root not in sys.path:
        sys.path.insert(0, root)
    import lrqmm_workloads
    return lrqmm_workloads


def measure(A, B, bits: int, rank: int, oversample: int = 0, power_iters: int = 1, seed: int = 1,
            per_tensor: bool = True, round_mode: int = 0, rows=None, precision: int = 0) -> dict:
    """Errors of direct quantization and of LRQMM for host arrays A (M x K), B (K x N).

    rows: optional row indices of C on which the errors are evaluated (all rows if None).
    """
    import numpy as np
    import torch
    from . import binding as L
    dA = torch.from_numpy(A).cuda()
    dB = torch.from_numpy(B).cuda()
    M, K = A.shape
    N = B.shape[1]
    mode = L.SCALE_TENSOR if per_tensor else L.SCALE_VECTOR
    ws = L.Workspace.for_problem(M, N, K, rank, oversample)
    sel = slice(None) if rows is None else np.asarray(rows, dtype=np.int64)
    ref = A[sel].astype(np.float64) @ B.astype(np.float64)
    den = np.linalg.norm(ref)

    def err(rk):
        D = torch.empty((M, N), dtype=torch.float32, device="cuda")
        L.lrqmm_matmul_ex(dA, dB, D, bits, rk, oversample if rk else 0, power_iters if rk else 0, seed=seed,
                          round_mode=round_mode, scale_mode=mode, workspace=ws, precision=precision)
        torch.cuda.synchronize()
        return float(np.linalg.norm(ref - D.cpu().numpy()[sel].astype(np.float64)) / den)

    e_dq = err(0)
    e_lr = err(rank) if rank > 0 else e_dq
    return {"err_direct_quant": e_dq, "err_lrqmm": e_lr, "gain": e_dq / e_lr if e_lr > 0 else float("inf")}


def sweep_tables(size: int, rank: int, oversample: int, power_iters: int, bits_list=(4, 8, 3, 5)):
    wl = _workloads()
    for kind in DISTRIBUTIONS:
        A = wl.random_matrix(kind, size, size, seed=0)
        B = wl.random_matrix(kind, size, size, seed=1)
        for bits in bits_list:
            r = measure(A, B, bits, rank, oversample, power_iters)
            yield {"sweep": "tables", "distribution": kind, "size": size, "bits": bits, "rank": rank,
                   "oversample": oversample, "power_iters": power_iters, "scale": "per-matrix", **r}


def sweep_rank(size: int, oversample: int, power_iters: int, kind: str = "uniform01", bits: int = 8):
    wl = _workloads()
    A = wl.random_matrix(kind, size, size, seed=0)
    B = wl.random_matrix(kind, size, size, seed=1)
    for rank in (1, 2, 5, 10, 20, 40, 80):
        if rank + oversample > min(size, 80):
            continue
        r = measure(A, B, bits, rank, oversample, power_iters)
        yield {"sweep": "rank", "distribution": kind, "size": size, "bits": bits, "rank": rank,
               "oversample": oversample, "power_iters": power_iters, "scale": "per-matrix", **r}


def sweep_size(rank: int, oversample: int, power_iters: int, kind: str = "uniform01", bits: int = 8):
    wl = _workloads()
    for size in (200, 500, 1000, 2000, 4000):
        A = wl.random_matrix(kind, size, size, seed=0)
        B = wl.random_matrix(kind, size, size, seed=1)
        r = measure(A, B, bits, rank, oversample, power_iters)
        yield {"sweep": "size", "distribution": kind, "size": size, "bits": bits, "rank": rank,
               "oversample": oversample, "power_iters": power_iters, "scale": "per-matrix", **r}


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--sweep", choices=("tables", "rank", "size", "all"), default="tables")
    ap.add_argument("--size", type=int, default=2000)
    ap.add_argument("--rank", type=int, default=10)
    ap.add_argument("--oversample", type=int, default=0)
    ap.add_argument("--power-iters", type=int, default=1)
    a = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        raise SystemExit("accuracy sweeps run the HIP library and need a GPU")
    if a.sweep in ("tables", "all"):
        for rec in sweep_tables(a.size, a.rank, a.oversample, a.power_iters):
            print(json.dumps(rec), flush=True)
    if a.sweep in ("rank", "all"):
        for rec in sweep_rank(200, a.oversample, a.power_iters):
            print(json.dumps(rec), flush=True)
    if a.sweep in ("size", "all"):
        for rec in sweep_size(a.rank, a.oversample, a.power_iters):
            print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
