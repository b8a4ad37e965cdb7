"""Helpers for the GPU parity tests: tensors in, numpy out, loud progress lines."""
import sys

import numpy as np


def say(*a):
    print("[gpu-test]", *a, flush=True)
    sys.stdout.flush()


def to_dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def to_np(t):
    import torch
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def rel_fro(ref, x):
    ref = np.asarray(ref, dtype=np.float64)
    d = np.linalg.norm(ref)
    n = np.linalg.norm(ref - np.asarray(x, dtype=np.float64))
    return n / d if d > 0 else n


EPS32 = 2.0 ** -24


def elementwise_budget(ref, rank, rows=None):
    """Per-element bound on |C_gpu - C_oracle| for the compensated product, from the oracle's own
    intermediates (all float64).

    The epilogue forms, per output element, fl32(C_int s_i s_j) (at most three roundings of a value of
    size |C0|) and then adds the 2r products Lp[i,t] Rp[j,t] of the rank-2r update one after the other in
    float32, every partial sum being at most  S = |C0| + sum_t |Lp[i,t] Rp[j,t]|  in size: (2r + 3)
    roundings of at most 2^-24 S each.  The panel entries Lp = [U Sigma | A~ W], Rp = [V^T B~ + (V^T W)
    Gamma Z^T ; Gamma Z^T] are themselves length-K (or length-l) float32 sums and carry the float32
    factorization; their error enters through the same 2r products and is covered by a factor 4:
        budget = 4 (2r + 3) 2^-24 S.
    S is evaluated with the oracle's factors (the regrouping the kernel uses).  Unlike |C0| + |C - C0| it
    cannot vanish by cancellation, so no element has an empty budget.  A wrong element (a dropped tile,
    a wrong row of a panel, a missing scale) is off by O(S), five orders of magnitude above the budget.
    Returns (budget, S) for the sampled rows (all rows when rows is None).
    """
    sel = slice(None) if rows is None else np.asarray(rows)
    C0 = np.abs(np.asarray(ref["C0"], dtype=np.float64))
    if rank == 0:
        return 4 * 3 * EPS32 * C0, C0
    Ut = np.asarray(ref["U"], np.float64) * np.asarray(ref["Sig"], np.float64).reshape(1, -1)
    Ztp = np.asarray(ref["Gam"], np.float64).reshape(-1, 1) * np.asarray(ref["Zt"], np.float64)
    W = np.asarray(ref["W"], np.float64)
    Vt = np.asarray(ref["Vt"], np.float64)
    P = Vt @ ref["Bf"] + (Vt @ W) @ Ztp                   # r x N : right panel, first half
    S_left = ref["Af"][sel] @ W                           # rows x r : left panel, second half
    S = C0 + np.abs(Ut[sel]) @ np.abs(P) + np.abs(S_left) @ np.abs(Ztp)
    return 4 * (2 * rank + 3) * EPS32 * S, S


def check_elementwise(got, ref, rank, rows=None, what=""):
    """Every sampled element of C within its budget; prints the worst ratio error / (2^-24 S)."""
    budget, S = elementwise_budget(ref, rank, rows)
    err = np.abs(np.asarray(got, dtype=np.float64) - np.asarray(ref["C"], dtype=np.float64))
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(S > 0, err / (EPS32 * S), np.where(err > 0, np.inf, 0.0))
    worst = float(ratio.max()) if ratio.size else 0.0
    say(what, "element-wise: worst |err| / (2^-24 S) =", round(worst, 2), "allowed", 4 * (2 * rank + 3))
    bad = np.argwhere(err > budget)
    assert bad.size == 0, f"{what}: {len(bad)} elements beyond their budget, first at {bad[:5].tolist()}"
