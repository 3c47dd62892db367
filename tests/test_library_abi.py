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
    assert len(names) == 20
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


def test_precondition_and_workspace_errors_are_reported_before_any_launch():
    """Host-side validation: every error below is returned before the first HIP call, so
    fake device addresses are never touched."""
    from paper_2208_09151_amd import _lib
    lib = _lib.load()
    fake = ctypes.c_void_p(0x1000)
    fan = np.array([10, 10], dtype=np.int32)
    so = np.array([0, 5, 12], dtype=np.int64)
    host = lambda n: np.zeros(n, dtype=np.int64)
    ids_off, hops, ro, co, tot = host(3), host(6), host(5), host(5), host(3)
    g = _lib.CsrDesc(100, 1000, 0x1000, 0, 0x1000, None, None)
    P = lambda a: ctypes.c_void_p(a.ctypes.data)

    def sample(seed_offsets=so, S=2, ws_bytes=16, fanout=fan, ws=fake):
        return lib.ginex_sample_superbatch(
            ctypes.byref(g), fake, P(seed_offsets), S, P(fanout), len(fanout), 0, 0,
            fake, 1000, P(ids_off), P(hops), fake, 1000, fake, 1000, P(ro), P(co), P(tot),
            ws, ws_bytes, None)

    assert sample() == -3 and b"workspace" in lib.ginex_last_error()
    assert sample(seed_offsets=np.array([0, 7, 3], dtype=np.int64)) == -4
    assert b"not monotone" in lib.ginex_last_error()
    assert sample(seed_offsets=np.array([1, 5, 12], dtype=np.int64)) == -4
    assert sample(fanout=np.array([10, 0], dtype=np.int32)) == -1
    assert sample(ws=None) == -1
    need = lib.ginex_sample_workspace_bytes(100, 2, 7, P(fan), 2)
    assert sample(ws=ctypes.c_void_p(0x1010), ws_bytes=need) == -1   # misaligned workspace
    assert b"aligned" in lib.ginex_last_error()

    io = np.array([0, 4, 9], dtype=np.int64)
    ic, tc = host(1), host(1)

    def changeset(ids_offsets=io, S=2, cap=3, ws_bytes=16, n=100):
        return lib.ginex_changeset(n, fake, P(ids_offsets), S, cap, fake, P(ic), fake, fake, fake,
                                   100, fake, fake, None, P(tc), None, fake, ws_bytes, None)

    assert changeset() == -3
    assert changeset(ids_offsets=np.array([0, 9, 4], dtype=np.int64)) == -4
    assert changeset(ids_offsets=np.array([0, 200, 300], dtype=np.int64)) == -4   # > nodes
    assert b"more ids than nodes" in lib.ginex_last_error()
    assert changeset(cap=-1) == -1
    assert changeset(S=0) == -1

    c = _lib.CacheDesc(0x1000, 4, 64, 0x1000, 10, 0x1000)
    assert lib.ginex_cache_init(ctypes.byref(c), fake, 5, None) == -1      # more rows than lines
    assert lib.ginex_cache_init_part(ctypes.byref(c), fake, 2, 5, None) == -1
    assert lib.ginex_cache_init_part(ctypes.byref(c), fake, 3, 2, None) == -1
    assert lib.ginex_gather(ctypes.byref(c), fake, 2, fake, fake, fake, fake, 3, None) == -1
    # warm initialization: the two caches must front the same slow tier and share no array
    other = _lib.CacheDesc(0x2000, 4, 64, 0x2000, 10, 0x3000)
    assert lib.ginex_cache_init_warm(ctypes.byref(c), ctypes.byref(other), fake, 0, 2, None) == -1
    assert b"same slow tier" in lib.ginex_last_error()
    assert lib.ginex_cache_init_warm(ctypes.byref(c), ctypes.byref(c), fake, 0, 2, None) == -1
    assert b"share" in lib.ginex_last_error()
    # a carried cache needs a start state, and at least one line
    assert lib.ginex_changeset_resume(100, fake, P(io), 2, 3, None, fake, fake, fake, fake, 100,
                                      fake, fake, None, P(tc), fake, 16, None) == -1
    assert lib.ginex_changeset_resume(100, fake, P(io), 2, 0, fake, fake, fake, fake, fake, 100,
                                      fake, fake, None, P(tc), fake, 1 << 40, None) == -1
    assert b"cap >= 1" in lib.ginex_last_error()
    # neighbour cache: half a cache in the graph descriptor, missing outputs, small workspace
    half = _lib.CsrDesc(100, 1000, 0x1000, 0, 0x1000, 0x1000, None)
    assert lib.ginex_sample_superbatch(
        ctypes.byref(half), fake, P(so), 2, P(fan), 2, 0, 0, fake, 1000, P(ids_off), P(hops),
        fake, 1000, fake, 1000, P(ro), P(co), P(tot), fake, 1 << 40, None) == -1
    assert b"neighbour cache" in lib.ginex_last_error()
    cn, ue = host(1), host(1)
    assert lib.ginex_neighbor_cache_build(ctypes.byref(g), 10, None, fake, P(cn), P(ue), fake,
                                          1 << 40, None) == -1
    assert lib.ginex_neighbor_cache_build(ctypes.byref(g), -1, fake, fake, P(cn), P(ue), fake,
                                          1 << 40, None) == -1
    assert lib.ginex_neighbor_cache_build(ctypes.byref(g), 10, fake, fake, P(cn), P(ue), fake,
                                          16, None) == -3
    assert lib.ginex_neighbor_cache_workspace_bytes(0) == 0
    assert lib.ginex_cache_update(ctypes.byref(c), fake, fake, fake, fake, 9, None) == -1
    assert lib.ginex_gather_lines(ctypes.byref(c), fake, None, 2, -1, fake, None, None, None, 0,
                                  None) == -1
    assert b"src_line" in lib.ginex_last_error()
    assert lib.ginex_gather_lines(ctypes.byref(c), fake, fake, 2, -1, fake, fake, fake, fake, 3,
                                  None) == -1
    assert lib.ginex_gather_lines(ctypes.byref(c), fake, fake, 2, 3, fake, None, None, None, 0,
                                  None) == -1
    assert b"n_slow" in lib.ginex_last_error()
    # the allocation-free changeset checks its shape against the built-in scratch on the host
    big = np.array([0, 1 << 22, 1 << 23], dtype=np.int64)
    assert lib.ginex_changeset_noalloc(1 << 24, fake, P(big), 2, 1000, fake, P(ic), fake, fake, fake,
                                       1 << 23, fake, fake, None, P(tc), None, None) == -3
    assert b"scratch" in lib.ginex_last_error()
    # static policy: descriptor, outputs and workspace are checked on the host
    assert lib.ginex_static_select_workspace_bytes(0) == 0
    assert lib.ginex_static_select_workspace_bytes(1000) > 2 * 8 * 1000
    assert lib.ginex_static_select(None, 3, fake, P(cn), fake, 1 << 40, None) == -1
    assert lib.ginex_static_select(ctypes.byref(g), 3, None, P(cn), fake, 1 << 40, None) == -1
    assert lib.ginex_static_select(ctypes.byref(g), -1, fake, P(cn), fake, 1 << 40, None) == -1
    assert lib.ginex_static_select(ctypes.byref(g), 3, fake, P(cn), fake, 16, None) == -3
    assert lib.ginex_cache_count_misses(None, fake, 3, fake, None) == -1
    assert lib.ginex_cache_count_misses(ctypes.byref(c), None, 3, fake, None) == -1
    assert lib.ginex_cache_count_misses(ctypes.byref(c), fake, 3, None, None) == -1
    assert lib.ginex_gather(ctypes.byref(c), fake, 2, ctypes.c_void_p(0x1008), None, None, None,
                            0, None) == -1                                   # out misaligned
