"""Build and run the roofline microbenchmarks (csrc/microbench/peaks.hip) on the current GPU:

    python -m paper_2409_18772_amd.microbench

int8 matrix-core rates with constant and with refreshed operands, LDS read/write rates in the GEMM's access
patterns, and a streaming copy.  The figures behind the ceilings quoted for the GEMM and the streaming kernels.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "microbench", "peaks.hip")
OUT = os.path.join(HERE, "_build", "peaks")


def build() -> str:
    os.makedirs(os.path.dirname(OUT), exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                    "-packed-fp32-ops", SRC, "-o", OUT], check=True)
    return OUT


def main() -> int:
    exe = OUT if os.path.exists(OUT) and os.path.getmtime(OUT) > os.path.getmtime(SRC) else build()
    return subprocess.run([exe]).returncode


if __name__ == "__main__":
    sys.exit(main())
