"""The C-ABI library loads and exports every symbol include/ggnn.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ggnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ggnn_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = _declared()
    for must in ("ggnn_build", "ggnn_query", "ggnn_graph_import", "ggnn_graph_export", "ggnn_free"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_1912_01059_amd import binding
    path = os.path.join(ROOT, "paper_1912_01059_amd", "libggnn.so")
    if not os.path.exists(path):
        from paper_1912_01059_amd import hipbuild
        hipbuild.build()
    lib = ctypes.CDLL(path)
    for name in _declared():
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == _declared()


def test_argument_errors_are_reported_without_a_gpu():
    from paper_1912_01059_amd import binding
    L = binding.lib()
    out = ctypes.c_void_p()
    rc = L.ggnn_graph_create(None, 100, 128, 24, 3, 1, None, ctypes.byref(out))
    assert rc == -1 and b"NULL" in L.ggnn_last_error()
    rc = L.ggnn_query(None, None, 1, 10, 10, 0.5, None, None)
    assert rc == -1
    rc = L.ggnn_merge(None, 0, 0)
    assert rc == -1
    # row lengths: float32 up to 1024 elements, multiples of 16 bytes (a non-null dummy address is
    # enough: arguments are checked before anything touches the device)
    dummy = ctypes.c_void_p(4096)
    assert L.ggnn_graph_create(dummy, 1000, 1028, 24, 3, 1, None, ctypes.byref(out)) == -1
    assert b"too large" in L.ggnn_last_error()
    assert L.ggnn_graph_create(dummy, 1000, 130, 24, 3, 1, None, ctypes.byref(out)) == -1
    assert b"multiple of 16" in L.ggnn_last_error()


def test_missing_library_fails_loudly(monkeypatch):
    from paper_1912_01059_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libggnn.so")
    with pytest.raises(binding.GgnnError):
        binding.lib()
