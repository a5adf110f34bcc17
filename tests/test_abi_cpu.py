"""The C-ABI library loads without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "h3d.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(h3d_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    import paper_2007_12856_amd as h3d
    if not os.path.exists(h3d.LIB_PATH):
        from paper_2007_12856_amd import build
        build.build()
    lib = ctypes.CDLL(h3d.LIB_PATH)
    names = declared_symbols()
    assert len(names) >= 20
    for name in names:
        assert hasattr(lib, name), f"{name} declared in include/h3d.h but not exported"
        assert name in h3d._SIGNATURES, f"{name} has no Python binding"
        assert callable(getattr(h3d, name)), name


def test_descriptor_layout_matches_header():
    import paper_2007_12856_amd as h3d
    # void* + 8 x int32 + 2 x int64 with natural alignment
    assert ctypes.sizeof(h3d.h3d_tensor) == 8 + 8 * 4 + 4 * 8
    assert h3d.h3d_tensor.d_offset.offset == 40 and h3d.h3d_tensor.dtype.offset == 8 and h3d.h3d_tensor.c_stride.offset == 56


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2007_12856_amd as h3d
    monkeypatch.setattr(h3d, "_lib", None)
    monkeypatch.setattr(h3d, "LIB_PATH", "/nonexistent/libh3d.so")
    with pytest.raises(RuntimeError):
        h3d.lib()
