"""Host-side checked build (no GPU): the library's host code compiled with -DLRQMM_CHECK under AddressSanitizer and
UndefinedBehaviorSanitizer, driven through the C ABI by csrc/host_check/host_check.cpp.

The driver makes only calls that return before the first HIP call: size queries, calls with a rejected
argument, and calls whose workspace is one byte short (those run the whole workspace carving).  It sweeps every
combination of 14 extents from 1 to LRQMM_MAX_DIM for M, N, K with ranks 0..80, and checks the error code of
every rejected argument.  A sanitizer report, a failed LRQMM_CHECK assertion or a wrong status fails the test.
"""
import subprocess


def test_checked_host_build_runs_clean():
    from paper_2409_18772_amd.build import build_host_check
    exe = build_host_check(verbose=False)
    proc = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    tail = "\n".join(proc.stdout.splitlines()[-15:])
    assert proc.returncode == 0, tail
    assert "runtime error" not in proc.stdout and "AddressSanitizer" not in proc.stdout, tail
    assert "0 failures" in proc.stdout, tail
