"""The C-ABI library loads and exports every function include/fastcache.h
declares (no compute calls: this runs without a GPU)."""

import ctypes
import os
import re

from conftest import ROOT


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "fastcache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(fc_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_header_declares_the_named_entry_points():
    names = _declared_functions()
    for must in ("fc_pool_create", "fc_pool_alloc", "fc_compress_batch", "fc_pool_free"):
        assert must in names


def test_library_exports_every_declared_symbol():
    import torch  # noqa: F401  (its HIP runtime first, as the binding does: one runtime per process)
    from paper_2503_08461_amd import _build, fastcache
    if not os.path.exists(_build.LIB_PATH):
        _build.build_library()
    lib = ctypes.CDLL(_build.LIB_PATH)
    for name in _declared_functions():
        assert hasattr(lib, name), name
    assert sorted(fastcache.EXPORTS) == _declared_functions()
    # entry points that need no device answer sensibly
    lib.fc_last_error.restype = ctypes.c_char_p
    lib.fc_kernel_name.restype = ctypes.c_char_p
    assert lib.fc_kernel_name(1) == b"snapkv_score"
    assert lib.fc_pool_num_free(None) == -1
    out = ctypes.c_void_p()
    rc = lib.fc_pool_create(ctypes.byref(out), None, ctypes.c_size_t(0), 4, 16, 1, 1, 64, 0)
    assert rc == -1 and b"kv_base" in lib.fc_last_error()


def test_binding_fails_loudly_without_the_library(monkeypatch):
    from paper_2503_08461_amd import fastcache
    import pytest
    monkeypatch.setattr(fastcache, "_lib", None)
    monkeypatch.setattr(fastcache, "LIB_PATH", "/nonexistent/libfastcache.so")
    with pytest.raises(FileNotFoundError):
        fastcache.load_library()
