"""The C-ABI library loads and exports every symbol include/ginex.h declares (no GPU)."""
import ctypes
import os
import re

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ginex.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ginex_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    from paper_2208_09151_amd import _lib
    lib = _lib.load()
    names = declared_symbols()
    assert len(names) == 9
    assert sorted(_lib.SIGNATURES) == names
    for n in names:
        assert getattr(lib, n) is not None
    assert lib.ginex_version() >= 100


def test_host_side_argument_checks_need_no_gpu():
    from paper_2208_09151_amd import _lib
    lib = _lib.load()
    fan = np.array([10, 10, 10], dtype=np.int32)
    p = ctypes.c_void_p(fan.ctypes.data)
    # workspace queries are pure host arithmetic
    a = lib.ginex_sample_workspace_bytes(1 << 20, 20, 1000, p, 3)
    b = lib.ginex_sample_workspace_bytes(1 << 20, 40, 1000, p, 3)
    assert 0 < a < b
    assert lib.ginex_sample_workspace_bytes(1 << 20, 0, 1000, p, 3) == 0
    assert b"S=0" in lib.ginex_last_error()
    bad = np.array([10, 65], dtype=np.int32)
    assert lib.ginex_sample_workspace_bytes(100, 1, 10, ctypes.c_void_p(bad.ctypes.data), 2) == 0
    assert b"fanout[1]=65" in lib.ginex_last_error()
    c = lib.ginex_changeset_workspace_bytes(1 << 20, 5_000_000, 20, 100_000)
    assert c > 2 * 8 * 5_000_000
    assert lib.ginex_changeset_workspace_bytes(1 << 20, 5_000_000, 9000, 100_000) == 0
    # null descriptors are rejected before anything touches the GPU
    assert lib.ginex_cache_init(None, None, 0, None) == -1
    assert lib.ginex_gather(None, None, 0, None, None, None, None, 0, None) == -1
    desc = _lib.CacheDesc(0, 4, 24, 0, 10, 0)
    assert lib.ginex_cache_init(ctypes.byref(desc), None, 0, None) == -1
    assert b"multiple of 16" in lib.ginex_last_error()
