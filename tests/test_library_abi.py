"""No-GPU checks of the boundary: the library loads and exports what include/lrqmm.h declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    with open(os.path.join(ROOT, "include", "lrqmm.h")) as f:
        text = f.read()
    return sorted(set(re.findall(r"LRQMM_API[^;(]*?\b(lrqmm_\w+)\s*\(", text)))


def test_header_declares_the_three_named_calls():
    names = _declared()
    for n in ("lrqmm_quantize", "lrqmm_rsvd", "lrqmm_gemm", "lrqmm_matmul", "lrqmm_fill_sketch",
              "lrqmm_workspace_bytes", "lrqmm_status_string", "lrqmm_profile_enable", "lrqmm_profile_read"):
        assert n in names


def test_library_exports_every_declared_symbol():
    import paper_2409_18772_amd as L
    if not os.path.exists(L.lib_path()):
        pytest.skip("library not built (run __graft_entry__.build())")
    lib = ctypes.CDLL(L.lib_path())
    for n in _declared():
        assert hasattr(lib, n), n
    assert set(_declared()) == set(L.binding.EXPORTS)


def test_host_side_validation_without_a_gpu():
    import paper_2409_18772_amd as L
    if not os.path.exists(L.lib_path()):
        pytest.skip("library not built")
    lib = L.load_library()
    assert L.lrqmm_status_string(0) == "ok"
    assert "workspace" in L.lrqmm_status_string(-3)
    assert L.lrqmm_workspace_bytes(-1, 4, 4, 0, 0) == 0
    assert L.lrqmm_workspace_bytes(64, 64, 64, 70, 20) == 0
    small, big = L.lrqmm_workspace_bytes(256, 256, 256, 8, 0), L.lrqmm_workspace_bytes(4096, 4096, 4096, 32, 8)
    assert 0 < small < big
    assert big % 1 == 0 and big >= 2 * 4096 * 4096
    # argument checks return before anything touches a device
    assert lib.lrqmm_quantize(None, 4, 4, 0, 1, 0, None, None, None) == -2
    assert lib.lrqmm_quantize(None, 4, 4, 5, 8, 0, None, None, None) == -1
    assert lib.lrqmm_quantize(None, 4, 4, 0, 8, 0, None, None, None) == -1
    assert lib.lrqmm_rsvd(None, None, 8, 8, 0, 8, 0, 0, 0, 0, 0, None, None, None, None, None, 0, None) == -1
    assert lib.lrqmm_rsvd(None, None, 8, 8, 0, 8, 0, 9, 0, 0, 0, None, None, None, None, None, 0, None) == -1
    assert lib.lrqmm_rsvd(None, None, 200, 200, 0, 8, 0, 81, 0, 0, 0, None, None, None, None, None, 0, None) == -2
    assert lib.lrqmm_gemm(4, 4, 1 << 20, 8, 0, *([None] * 12), None, 0, None) == -2
    assert lib.lrqmm_matmul(4, 4, 4, 8, 5, 0, 0, 0, 0, None, None, None, None, 0, None) == -1
    assert lib.lrqmm_fill_sketch(1, -1, 4, 4, None, None) == -1
    # strides below the row length, unknown scale granularity
    assert lib.lrqmm_quantize_ex(None, 3, 4, 4, 0, 8, 0, 0, None, None, None) == -1
    assert lib.lrqmm_quantize_ex(None, 4, 4, 4, 0, 8, 0, 7, None, None, None) == -1
    assert lib.lrqmm_rsvd_ex(None, 7, None, 8, 8, 0, 8, 0, 2, 0, 0, 0, None, 0, None, None, None, None, 0, None) == -1
    assert lib.lrqmm_rsvd_ex(None, 8, None, 8, 8, 0, 8, 0, 2, 0, 0, 0, None, 3, None, None, None, None, 0, None) == -1     # unknown precision
    assert lib.lrqmm_gemm_ex(4, 4, 4, 8, 0, *([None] * 10), 1.0, 0.0, None, 3, None, None, 0, None) == -1
    assert lib.lrqmm_matmul_ex(4, 4, 4, 8, 0, 0, 0, 0, 0, 0, 0, None, 3, None, 4, 1.0, 0.0, None, 4, None, 0, None) == -1
    assert lib.lrqmm_matmul_ex(4, 4, 4, 8, 0, 0, 0, 0, 0, 3, 0, None, 4, None, 4, 1.0, 0.0, None, 4, None, 0, None) == -1
    assert lib.lrqmm_matmul_ex(4, 4, 4, 8, 0, 0, 0, 0, 0, 0, 5, None, 4, None, 4, 1.0, 0.0, None, 4, None, 0, None) == -1     # unknown precision


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_2409_18772_amd.binding as b
    monkeypatch.setattr(b, "_LIB", None)
    monkeypatch.setattr(b, "_HERE", str(tmp_path))
    with pytest.raises(ImportError):
        b.load_library()
