"""Compile the HIP sources into paper_2409_18772_amd/liblrqmm.so for gfx950 (in-tree).

Each source is compiled to an object file of its own (in parallel), then linked.  `build()` always
recompiles everything; `python -m paper_2409_18772_amd.build --incremental` recompiles only the
sources that are newer than their objects (or older than a header), for quick edit/run cycles.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "liblrqmm.so")
SOURCES = ["api.hip", "quantize.hip", "sketch.hip", "passes.hip", "orth.hip", "gemm.hip"]
HEADERS = [os.path.join(CSRC, "common.h"), os.path.join(CSRC, "kernels.h"),
           os.path.join(HERE, "..", "include", "lrqmm.h")]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                  # no implicit FMA: quantizer and sketch must round as written
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fvisibility=hidden", "-Wall", "-Wno-unused-function",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines()
                    if "packed-fp32-ops" not in l)   # host pass does not know the device feature
    if out.strip() and verbose:
        print(out, flush=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)


def build(verbose: bool = True, incremental: bool = False, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in HEADERS)
    jobs, objs = [], []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s.replace(".hip", ".o"))
        objs.append(obj)
        fresh = (incremental and os.path.exists(obj)
                 and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header))
        if not fresh:
            jobs.append([hipcc] + FLAGS + list(extra_flags) + ["-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=min(6, max(1, len(jobs)))) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], verbose)
    return LIB


def build_host_check(verbose: bool = False) -> str:
    """Checked host build: every source with -DLRQMM_CHECK and the host pass under AddressSanitizer and
    UndefinedBehaviorSanitizer (device code as usual), linked with csrc/host_check/host_check.cpp into the
    executable _build/host_check.  Running it needs no GPU: it exercises argument validation and workspace
    carving only (see the driver's header)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    obj_dir = os.path.join(OBJ, "checked")
    os.makedirs(obj_dir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-DLRQMM_CHECK", "-g"]
    flags = [f for f in FLAGS if f != "-O3"] + ["-O1"] + san
    jobs, objs = [], []
    for s in SOURCES:
        obj = os.path.join(obj_dir, s.replace(".hip", ".o"))
        objs.append(obj)
        jobs.append([hipcc] + flags + ["-c", os.path.join(CSRC, s), "-o", obj])
    drv = os.path.join(obj_dir, "host_check.o")
    jobs.append([hipcc, "-x", "c++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
                 "-fno-sanitize-recover=undefined", "-I", os.path.join(HERE, "..", "include"), "-c",
                 os.path.join(CSRC, "host_check", "host_check.cpp"), "-o", drv])
    with ThreadPoolExecutor(max_workers=min(7, len(jobs))) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    exe = os.path.join(OBJ, "host_check")
    _run([hipcc, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize"] + objs + [drv, "-o", exe],
         verbose)
    return exe


if __name__ == "__main__":
    build(incremental="--incremental" in sys.argv)
    print("built", LIB)
