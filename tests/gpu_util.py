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
