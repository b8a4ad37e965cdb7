"""Compile the HIP sources into paper_2409_18772_amd/liblrqmm.so for gfx950 (in-tree)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblrqmm.so")
SOURCES = ["api.hip", "quantize.hip", "sketch.hip", "passes.hip", "orth.hip", "gemm.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                  # no implicit FMA: quantizer and sketch must round as written
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fvisibility=hidden", "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines()
                    if "packed-fp32-ops" not in l)   # host pass does not know the device feature
    if out.strip() and verbose:
        print(out)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
