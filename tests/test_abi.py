"""Host-side checks that need no GPU: the built library exports what include/ac.h declares, and
argument validation rejects bad calls before any launch."""
import os
import re

import pytest

from paper_2505_18574_amd import ops

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ac.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ac_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    L = ops.lib()
    names = declared_symbols()
    assert set(names) == set(ops.EXPORTS)
    for name in names:
        assert getattr(L, name) is not None


def test_version_and_status_strings():
    assert ops.ac_version() >= 100
    seen = set()
    for code in range(0, -9, -1):
        s = ops.status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert ops.status_string(-1234) == "unknown status"


def test_validation_without_gpu():
    # every call below fails validation (or is empty), so nothing is launched
    L = ops.lib()
    p = 0x1000  # never dereferenced
    assert L.ac_gemm_i8(p, 8, p + 256, 8, None, 0, p + 512, 8, 8, 8, 8, -1, 0, None, 0, None) == ops.AC_ERR_SHIFT
    assert L.ac_gemm_i8(p, 8, p + 256, 8, None, 0, p + 512, 8, 8, 8, 8, 0, 7, None, 0, None) == ops.AC_ERR_ACT
    assert L.ac_gemm_i8(p, 7, p + 256, 8, None, 0, p + 512, 8, 8, 8, 8, 0, 0, None, 0, None) == ops.AC_ERR_STRIDE
    assert L.ac_gemm_i8(p, 8, p + 256, 8, p + 768, 4, p + 512, 8, 8, 8, 8, 0, 0, None, 0, None) == ops.AC_ERR_STRIDE
    assert L.ac_gemm_i8(p, 8, p + 256, 8, None, 0, p + 512, 8, 8, 8, 8, 0, 0, None, 64, None) == ops.AC_ERR_WORKSPACE
    assert L.ac_gemm_i8(p, 8, p + 256, 8, None, 0, p + 512, 8, 8, 8, 8, 0, 0, p + 1, 64, None) == ops.AC_ERR_WORKSPACE
    assert L.ac_gemm_i8(p, 8, p + 256, 8, None, 0, None, 8, 8, 8, 8, 0, 0, None, 0, None) == ops.AC_ERR_NULL
    assert L.ac_gemm_i8(None, 8, None, 8, None, 0, None, 8, 0, 8, 8, 0, 0, None, 0, None) == ops.AC_OK
    assert L.ac_conv2d_i8(p, p + 256, None, p + 512, 1, 4, 4, 16, 16, 3, 3, 1, -1, 0, 0, None, 0, None) == ops.AC_ERR_SHAPE
    assert L.ac_conv2d_i8(p, p + 256, None, p + 512, 1, 40000, 4, 16, 16, 3, 3, 1, 1, 0, 0, None, 0, None) == ops.AC_ERR_SHAPE
    assert L.ac_conv2d_i8(p, p + 256, None, p + 512, 1, 4, 4, 16, 0, 3, 3, 1, 1, 0, 0, None, 0, None) == ops.AC_OK
    assert L.ac_gemm_bf16(p, 8, p + 256, 8, p + 512, 4, 8, 8, 8, 1.0, 0.0, None) == ops.AC_ERR_STRIDE
    assert L.ac_gemm_bf16(p, 8, p + 256, 8, p + 512, 8, 8, 0, 8, 1.0, 0.0, None) == ops.AC_OK
    assert L.ac_batched_gemm_f32(p, p + 256, p + 512, None, None, None, 33, 4, None) == ops.AC_ERR_SHAPE
    assert L.ac_batched_gemm_f32(p, p + 256, p + 512, None, None, None, 12, -1, None) == ops.AC_ERR_SHAPE
    assert ops.ac_gemm_i8_workspace_bytes(0, 8, 8) == 0


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(ops, "_lib", None)
    monkeypatch.setattr(ops, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libac_mi355x.so"))
    with pytest.raises(ImportError):
        ops.lib()
