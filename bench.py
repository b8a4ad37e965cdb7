#!/usr/bin/env python3
"""Benchmark of the LRQMM hot path on one MI355X.

A step is one pass of the whole hot path (lrqmm_matmul: quantize A and B, factor
both residuals, integer GEMM with fused compensation) over one batch of synthetic
input already resident in HBM.  Prints ONE JSON line with the headline metric
(effective TOPS = 2MNK / t), a roofline object for the dominant kernel (the int8
MFMA GEMM), the per-stage split, relative errors against
the exact product, and the CPU oracle timed on the host cores as a baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0     # MI355X dense int8 MFMA, TOP/s
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, GB/s


def read_traffic(name: str, key: str = "traffic_bytes_per_launch"):
    """HBM bytes per launch measured offline with rocprofv3 --pmc (profiles/<name>, line `key: N`), or None."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        with open(path) as f:
            for line in f:
                if line.startswith(key + ":"):
                    return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


INPUT_TEXT = {
    "uniform_pm1": "U[-1,1]",
    "normal": "N(0,1)",
    "normal_outliers": "N(0,1) with 0.1% entries from N(0,20^2)",
    "relu_normal": "A = max(0, N(0,1)), B ~ N(0, 2/K)",
}
SHORT = {"c1_256_int8_r8": "c1", "c2_4096_int8_r16": "c2", "c3_4096_int4_r32_outliers": "c3",
         "c4_16384_int4_r64": "c4", "c5_resnet50_conv_int4_r8": "c5"}


def metric_text(w):
    shape = f"{w.M}^3" if w.M == w.N == w.K else f"{w.M}x{w.N}x{w.K}"
    return f"LRQMM effective TOPS (2MNK/t) at {shape} int{w.bits} r={w.rank}; rel. error vs direct quant"


def cpu_baseline(w, A, B, budget_rows: int):
    """Time the oracle (as it stands) on a bounded sample: all O(N^2) stages in full, the
    O(N^3) integer product / compensation / exact product on `budget_rows` rows of C."""
    import numpy as np
    from oracle import lrqmm_oracle as o
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    rows = np.arange(0, w.M, max(1, w.M // budget_rows))[:budget_rows]
    t0 = time.perf_counter()
    o.lrqmm(A, B, w.bits, w.rank, w.oversample, w.power_iters, seed=w.sketch_seed, row_sample=rows,
            want_cint=False)
    t_sample = time.perf_counter() - t0
    # second run with rank 0 on the same rows isolates the row-proportional part
    t0 = time.perf_counter()
    o.lrqmm(A, B, w.bits, 0, row_sample=rows, want_cint=False)
    t_rows = time.perf_counter() - t0
    t0 = time.perf_counter()
    o.lrqmm(A, B, w.bits, 0, row_sample=rows[:1], want_cint=False)
    t_fixed = time.perf_counter() - t0
    per_row = max(t_rows - t_fixed, 0.0) / max(len(rows) - 1, 1)
    t_full = (t_sample - per_row * len(rows)) + per_row * w.M
    ops = 2.0 * w.M * w.N * w.K
    return {
        "value": ops / t_full / 1e12, "unit": "TOPS", "cores": int(threads), "kind": "oracle",
        "sample": (f"oracle.lrqmm on the same inputs: quantization and both residual factorizations in full, "
                   f"integer GEMM/compensation on {len(rows)} of {w.M} rows of C ({t_sample:.1f} s measured); "
                   f"row-proportional time {per_row * 1e3:.1f} ms/row extrapolated to all rows "
                   f"({t_full:.0f} s).  Threads: the float64 stages (residual products, QR, SVD, compensation) "
                   f"run on the BLAS pool of {int(threads)} threads; the quantizer is single-threaded numpy and "
                   f"the int64 integer product, which is the row-proportional part, runs on 1 thread (numpy has "
                   f"no BLAS for integers)"),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3_4096_int4_r32_outliers")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=192)
    ap.add_argument("--precision-modes", action="store_true",
                    help="also time the reduced-precision compensation modes and report their errors")
    ap.add_argument("--no-baselines", action="store_true",
                    help="skip the complete-residual-compensation baselines (several extra full-size GEMMs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 64 MiB device copy (reference for rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU (one MI355X); run with --gpus 1")

    import numpy as np
    import torch
    import paper_2409_18772_amd as L
    import lrqmm_workloads as wl
    from oracle import lrqmm_oracle as o     # cpu_baseline leg and error check only

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    w = wl.CONFIGS[args.workload]
    A, B = wl.make_inputs(w)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    C = torch.empty((w.M, w.N), dtype=torch.float32, device="cuda")
    ws = L.Workspace.for_problem(w.M, w.N, w.K, w.rank, w.oversample)

    if args.calibrate_copy:
        src = torch.zeros(16 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)              # 64 MiB read + 64 MiB written by one copy kernel
        torch.cuda.synchronize()

    def step(rank=w.rank):
        L.lrqmm_matmul(dA, dB, w.bits, rank, w.oversample, w.power_iters, seed=w.sketch_seed, workspace=ws, C=C)

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    # headline: K steps of the whole path.  In the timed region only the integer GEMM is bracketed by
    # HIP events (on the stream it is launched on); the full stage split is taken in a second,
    # untimed pass, because its eleven event records per step lengthen a step by ~4 %.
    L.lrqmm_profile_enable(L.PROF_GEMM_ONLY)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    L.lrqmm_profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / args.steps
    gemm_stages, ncalls = L.lrqmm_profile_read()
    L.lrqmm_profile_enable(True)
    for _ in range(min(args.steps, 20)):
        step()
    torch.cuda.synchronize()
    stages, _ = L.lrqmm_profile_read()
    L.lrqmm_profile_enable(False)
    early = gemm_stages.get("int_gemm", 0.0) > 1e-3
    # the GEMM's launch time is the one measured inside the timed region
    stages["int_gemm" if early else "gemm"] = gemm_stages["int_gemm" if early else "gemm"]

    # direct-quantization pipeline alone (rank 0) for the overhead figure
    t_dq = timed(lambda: step(0), max(5, args.steps // 2), 2)
    # the integer product alone on the idle chip (codes resident, fused dequantizing store, no compensation):
    # context for the in-schedule figure of the roofline object
    cA, mA = L.lrqmm_quantize(dA, L.AXIS_ROW, w.bits)
    cB, mB = L.lrqmm_quantize(dB, L.AXIS_COL, w.bits)
    t_gemm_alone = timed(lambda: L.lrqmm_gemm(cA, mA, cB, mB, w.bits, workspace=ws, C=C), max(5, args.steps // 2), 2)
    del cA, cB
    step()
    torch.cuda.synchronize()
    Cn = C.cpu().numpy()

    ops = 2.0 * w.M * w.N * w.K
    tops = ops / t_step / 1e12
    # dominant kernel: the int8 MFMA GEMM.  For large problems lrqmm_matmul runs it early on its
    # third stream (stage "int_gemm", raw int32 sums) and the epilogue separately (stage "gemm");
    # otherwise stage "gemm" is the GEMM with its fused epilogue.
    gemm_key = "int_gemm" if early else "gemm"
    gemm_s = stages[gemm_key] * 1e-3
    achieved = ops / gemm_s / 1e12 if gemm_s > 0 else 0.0
    fp32_bytes = 4.0 * (w.M * w.K + w.K * w.N)
    passes = 2 + 2 * w.power_iters           # residual passes per operand
    stage_info = {
        k: {"ms": round(v, 4)} for k, v in stages.items()
    }
    # Quantization + factorization of one operand as one streaming job.  Algorithmic bytes: one read for the
    # group maxima, one per residual product (the first of them also writes the codes), 4 B per element each,
    # plus 1 B per element of codes.  (Shapes off the guard-free kernels read B once more: maxima, codes,
    # products.)  With rank 0 only the maxima and the codes remain.  Short rows of A (K <= 576, a sketch of at most
    # 16 columns) are the one case that gets by with fewer reads than this count: maxima, codes and the first
    # product come from a single read there ("reads_performed").
    one_read_a = (w.rank > 0 and w.K % 16 == 0 and 16 <= w.K <= 576 and w.rank + w.oversample <= 16)
    for op, elems in (("a", w.M * w.K), ("b", w.K * w.N)):
        n_reads = (1 + passes) if w.rank > 0 else (1 if op == "a" else 2)
        job_ms = stages["quantize_" + op] + stages["rsvd_" + op]
        gbs = (4.0 * n_reads + 1.0) * elems / (job_ms * 1e-3) / 1e9
        stage_info["rsvd_" + op].update(passes=passes)
        stage_info["quantize_and_factor_" + op] = {
            "ms": round(job_ms, 4), "operand_reads": n_reads,
            "reads_performed": n_reads - 1 if (op == "a" and one_read_a) else n_reads,
            "algorithmic_GBs": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)}
    stage_info[gemm_key].update(TOPs=round(achieved, 1), frac_int8_mfma=round(achieved / PEAK_INT8_TOPS, 4))
    # which roof bounds the product: its algorithmic bytes (codes read once, 4-byte results written once, panels)
    # against its operations; below peak_ops / peak_bytes operations per byte the kernel is bound by memory
    gemm_bytes = float(w.M * w.K + w.K * w.N + 4 * w.M * w.N + (0 if early else 8 * w.rank * (w.M + w.N)))
    large_tiles = w.M >= 256 and w.N >= 256 and -(-w.M // 256) * -(-w.N // 256) >= 128
    if ops / gemm_bytes >= PEAK_INT8_TOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        roof = {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                "frac": round(achieved / PEAK_INT8_TOPS, 4)}
    else:
        gbs_gemm = gemm_bytes / gemm_s / 1e9 if gemm_s > 0 else 0.0
        roof = {"bound": "hbm", "achieved": round(gbs_gemm, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(gbs_gemm / PEAK_HBM_GBS, 4), "algorithmic_bytes_per_launch": gemm_bytes}
    if early:   # the dequantizing rank-2r update alone: reads and rewrites C
        gbs = 8.0 * w.M * w.N / (stages["gemm"] * 1e-3) / 1e9
        stage_info["gemm"].update(kernel="rank_update_kernel", algorithmic_GBs=round(gbs, 1),
                                  frac_hbm=round(gbs / PEAK_HBM_GBS, 4))

    # accuracy on sampled rows against the exact float64 product
    rows = np.random.default_rng(0).choice(w.M, size=min(64, w.M), replace=False)
    exact = o.exact_product(A[rows], B)
    step(0)
    torch.cuda.synchronize()
    C0n = C.cpu().numpy()
    err_lr = o.rel_err(exact, Cn[rows])
    err_dq = o.rel_err(exact, C0n[rows])
    near = o.lrqmm(A, B, w.bits, 0, round_mode=o.NEAREST, row_sample=rows, want_cint=False)
    err_dq_near = o.rel_err(exact, near["C"])

    # complete residual compensation (Eq. (gemm_r_split) with three / four full-size integer GEMMs): the
    # alternative that the low-rank terms replace, on the same inputs and by the same library
    full_residual = {}
    rws = None if args.no_baselines else L.Workspace(L.lrqmm_residual_workspace_bytes(w.M, w.N, w.K))
    for terms, name in (() if args.no_baselines else ((3, "three_terms_QT110"), (4, "four_terms_QT111"))):
        fn = lambda: L.lrqmm_residual_matmul(dA, dB, C, w.bits, terms, workspace=rws)
        t_r = timed(fn, max(5, args.steps // 2), 2)
        full_residual[name] = {"ms": round(t_r * 1e3, 4), "rel_error": o.rel_err(exact, C.cpu().numpy()[rows])}
    del rws

    # reduced-precision compensation modes (lrqmm.h, LRQMM_PREC_*): step time, error against the exact product
    # and distance from the default mode's output, on the same sampled rows
    precision_modes = {}
    if args.precision_modes and w.rank > 0:
        for pname, mode in (("bf16x2_subspace_only", L.PREC_SUBSPACE_BF16X2), ("bf16x2", L.PREC_BF16X2),
                            ("bf16", L.PREC_BF16)):
            fn = lambda: L.lrqmm_matmul_ex(dA, dB, C, w.bits, w.rank, w.oversample, w.power_iters,
                                           seed=w.sketch_seed, workspace=ws, precision=mode)
            t_m = timed(fn, args.steps, 3)
            Cm = C.cpu().numpy()[rows]
            precision_modes[pname] = {
                "ms_per_step": round(t_m * 1e3, 4), "rel_error": o.rel_err(exact, Cm),
                "distance_from_default": float(np.linalg.norm(Cm.astype(np.float64) - Cn[rows])
                                               / np.linalg.norm(Cn[rows].astype(np.float64)))}

    out = {
        "metric": metric_text(w),
        "value": round(tops, 3), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(t_step * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": w.name, "M": w.M, "N": w.N, "K": w.K, "bits": w.bits, "rank": w.rank,
                   "oversample": w.oversample, "power_iters": w.power_iters, "sketch_seed": w.sketch_seed,
                   "inputs": f"{INPUT_TEXT.get(w.kind, w.kind)}, seeds {w.seed_a}/{w.seed_b}"},
        "roofline": {"kernel": ("int8_gemm256_kernel (int8 MFMA GEMM, raw int32 sums; on the library's third "
                                "stream beside the single-workgroup SVD kernels)") if early else
                               (("int8_gemm256_kernel" if large_tiles else ("int8_gemm_kernel (128 x 64 tiles)" if w.N <= 64 else "int8_gemm_kernel (128 x 128 tiles)"))
                                + " (int8 MFMA GEMM + fused dequant and rank-2r epilogue)"),
                     **roof,
                     # counter bytes of this kernel on this workload, or null when no summary is tracked for it
                     "traffic": read_traffic(f"int8_gemm_{SHORT.get(w.name, w.name)}_pmc.txt"),
                     "launch_ms": round(stages[gemm_key], 4), "ops_per_launch": ops,
                     "alone": {"ms": round(t_gemm_alone * 1e3, 4), "achieved": round(ops / t_gemm_alone / 1e12, 2),
                               "frac": round(ops / t_gemm_alone / 1e12 / PEAK_INT8_TOPS, 4),
                               "note": "lrqmm_gemm at rank 0 on the idle chip: the same product with its "
                                       "dequantizing float32 store, wall time per call"}},
        "stages": stage_info,
        "stages_note": "GEMM launch time from HIP events inside the timed region; the other stages from a "
                       "separate fully instrumented pass of the same step",
        "direct_quant_ms": round(t_dq * 1e3, 4),
        "overhead_vs_direct_quant": round((t_step - t_dq) / t_dq, 4),
        "rel_error": {"lrqmm": err_lr, "direct_quant_floor": err_dq, "direct_quant_nearest": err_dq_near,
                      "gain_vs_floor": err_dq / err_lr, "rows_sampled": int(len(rows))},
        "full_residual_baselines": full_residual,
    }
    if precision_modes:
        out["precision_modes"] = precision_modes
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, A, B, args.cpu_rows)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
