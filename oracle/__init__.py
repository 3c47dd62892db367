"""CPU oracle for the Ginex hot path: TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may
import this package.  It wraps ``ginex_oracle.cpp`` (plain single-threaded C++,
compiled with g++) through ctypes and takes/returns numpy arrays.  It shares no
code with the HIP library and never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ginex_oracle.cpp")
_LIB = os.path.join(_HERE, "libginex_oracle.so")

NEVER = 0x7FFFFFFF


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["g++", "-O2", "-std=c++17", "-Wall", "-shared", "-fPIC", _SRC, "-o", _LIB])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_draw64.restype = C.c_uint64
        _lib.oracle_draw64.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]
        _lib.oracle_floyd_picks.restype = C.c_int32
        _lib.oracle_floyd_picks.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32,
                                            C.c_int64, C.c_int32, C.c_void_p]
        _lib.oracle_lru_misses.restype = C.c_int64
        _lib.oracle_static_misses.restype = C.c_int64
        _lib.oracle_static_select.restype = C.c_int64
        _lib.oracle_gather_update.restype = C.c_int64
    return _lib


def _p(a):
    return C.c_void_p(a.ctypes.data) if a is not None else C.c_void_p(0)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_p(ctr), _p(key), _p(out))
    return out


def draw64(seed, node, batch, hop, i):
    return int(lib().oracle_draw64(seed, node, batch, hop, i))


def floyd_picks(seed, node, batch, hop, deg, k):
    out = np.zeros(max(k, 1), dtype=np.int64)
    n = lib().oracle_floyd_picks(seed, node, batch, hop, deg, k, _p(out))
    return out[:n].copy()


def neighbor_cache_build(offsets, indices, budget):
    """Section 3.2: returns (address_table int64 [N], cache_array int32 [used], cached node
    count)."""
    offsets = np.ascontiguousarray(offsets)
    assert offsets.dtype in (np.int32, np.int64)
    indices = _i32(indices)
    n = len(offsets) - 1
    address_table = np.zeros(max(n, 1), dtype=np.int64)
    cache_array = np.zeros(max(budget, 1), dtype=np.int32)
    cached, used = C.c_int64(0), C.c_int64(0)
    rc = lib().oracle_neighbor_cache_build(
        C.c_int64(n), _p(offsets), C.c_int32(offsets.dtype == np.int64), _p(indices),
        C.c_int64(budget), _p(address_table), _p(cache_array), C.byref(cached), C.byref(used))
    assert rc == 0
    return address_table[:n], cache_array[:used.value], cached.value


def neighbor_lookup(address_table, cache_array, v):
    """The neighbour list of ``v`` from the cache, or None on a miss (Figure 6b)."""
    address_table, cache_array = _i64(address_table), _i32(cache_array)
    deg = C.c_int64(0)
    lib().oracle_neighbor_lookup.restype = C.c_int64
    at = lib().oracle_neighbor_lookup(_p(address_table), _p(cache_array), C.c_int32(v),
                                      C.byref(deg))
    return None if at < 0 else cache_array[at:at + deg.value]


def sample_superbatch(offsets, indices, seeds, seed_offsets, fanout, rng_seed=0,
                      first_batch_index=0, neighbor_cache=None):
    """``neighbor_cache``: optional (address_table, cache_array); the result then also holds
    ``lookups`` = (hits, misses).
    Returns a dict with flat ``ids``, ``ids_offsets``, ``hop_sizes`` [S, H+1] and the
    per-(batch, hop) adjacency as flat ``adj_rowptr``/``adj_col`` with
    ``adj_row_offsets``/``adj_col_offsets`` of length S*H+1 (batch-major)."""
    offsets = np.ascontiguousarray(offsets)
    assert offsets.dtype in (np.int32, np.int64)
    indices = _i32(indices)
    seeds = _i32(seeds)
    seed_offsets = _i64(seed_offsets)
    fanout = _i32(fanout)
    S, H = len(seed_offsets) - 1, len(fanout)
    n = len(offsets) - 1
    ids_offsets = np.zeros(S + 1, dtype=np.int64)
    hop_sizes = np.zeros(S * (H + 1), dtype=np.int64)
    row_off = np.zeros(S * H + 1, dtype=np.int64)
    col_off = np.zeros(S * H + 1, dtype=np.int64)
    need = np.zeros(3, dtype=np.int64)
    # upper bounds: a list grows by at most (1 + fanout) per hop and never beyond n
    caps = [0, 0, 0]
    for b in range(S):
        cur = min(int(seed_offsets[b + 1] - seed_offsets[b]), n)
        for k in fanout:
            caps[1] += cur + 1
            caps[2] += cur * int(k)
            cur = min(cur * (1 + int(k)), n)
        caps[0] += cur
    ids = np.zeros(max(caps[0], 1), dtype=np.int32)
    rowptr = np.zeros(max(caps[1], 1), dtype=np.int64)
    col = np.zeros(max(caps[2], 1), dtype=np.int32)
    if neighbor_cache is not None:
        at, ca = _i64(neighbor_cache[0]), _i32(neighbor_cache[1])
        if len(ca) == 0:
            ca = np.zeros(1, dtype=np.int32)
        lookups = np.zeros(2, dtype=np.int64)
        rc = lib().oracle_sample_superbatch_cached(
            C.c_int64(n), _p(offsets), C.c_int32(offsets.dtype == np.int64), _p(indices),
            _p(at), _p(ca),
            _p(seeds), _p(seed_offsets), C.c_int32(S), _p(fanout), C.c_int32(H),
            C.c_uint64(rng_seed), C.c_uint32(first_batch_index),
            _p(ids), C.c_int64(caps[0]), _p(ids_offsets), _p(hop_sizes),
            _p(rowptr), C.c_int64(caps[1]), _p(col), C.c_int64(caps[2]),
            _p(row_off), _p(col_off), _p(need), _p(lookups))
    else:
        lookups = None
        rc = lib().oracle_sample_superbatch(
            C.c_int64(n), _p(offsets), C.c_int32(offsets.dtype == np.int64), _p(indices),
            _p(seeds), _p(seed_offsets), C.c_int32(S), _p(fanout), C.c_int32(H),
            C.c_uint64(rng_seed), C.c_uint32(first_batch_index),
            _p(ids), C.c_int64(caps[0]), _p(ids_offsets), _p(hop_sizes),
            _p(rowptr), C.c_int64(caps[1]), _p(col), C.c_int64(caps[2]),
            _p(row_off), _p(col_off), _p(need))
    assert rc == 0
    return dict(lookups=lookups, ids=ids[:need[0]], ids_offsets=ids_offsets,
                hop_sizes=hop_sizes.reshape(S, H + 1),
                adj_rowptr=rowptr[:need[1]], adj_col=col[:need[2]],
                adj_row_offsets=row_off, adj_col_offsets=col_off)


def next_use(num_nodes, ids, ids_offsets):
    ids = _i32(ids)
    ids_offsets = _i64(ids_offsets)
    S = len(ids_offsets) - 1
    nxt = np.zeros(max(len(ids), 1), dtype=np.int32)
    first = np.zeros(num_nodes, dtype=np.int32)
    lib().oracle_next_use(C.c_int64(num_nodes), _p(ids), _p(ids_offsets), C.c_int32(S),
                          _p(nxt), _p(first))
    return nxt[:len(ids)], first


def _changeset(fn, num_nodes, ids, ids_offsets, cap):
    ids = _i32(ids)
    ids_offsets = _i64(ids_offsets)
    S = len(ids_offsets) - 1
    init_ids = np.zeros(max(cap, 1), dtype=np.int32)
    init_count = np.zeros(1, dtype=np.int64)
    cs_offsets = np.zeros(S + 1, dtype=np.int64)
    miss = np.zeros(max(S, 1), dtype=np.int64)
    capacity = max(len(ids), 1)     # every changeset record is a miss, so this suffices
    a = np.zeros(capacity, dtype=np.int32)
    b = np.zeros(capacity, dtype=np.int32)
    c = np.zeros(capacity, dtype=np.int32)
    rc = fn(C.c_int64(num_nodes), _p(ids), _p(ids_offsets), C.c_int32(S), C.c_int64(cap),
            _p(init_ids), _p(init_count), _p(a), _p(b), _p(c), C.c_int64(capacity),
            _p(cs_offsets), _p(miss))
    assert rc == 0
    n = int(cs_offsets[S])
    return dict(init_ids=init_ids[:int(init_count[0])], in_ids=a[:n], out_ids=b[:n],
                in_positions=c[:n], cs_offsets=cs_offsets, miss_count=miss[:S])


def _changeset_resume(fn, num_nodes, ids, ids_offsets, cap, start_ids):
    ids, ids_offsets, start_ids = _i32(ids), _i64(ids_offsets), _i32(start_ids)
    assert len(start_ids) <= cap
    S = len(ids_offsets) - 1
    init_ids = np.zeros(max(cap, 1), dtype=np.int32)
    final_ids = np.zeros(max(cap, 1), dtype=np.int32)
    init_count = np.zeros(1, dtype=np.int64)
    cs_offsets = np.zeros(S + 1, dtype=np.int64)
    miss = np.zeros(max(S, 1), dtype=np.int64)
    capacity = max(len(ids), 1)
    a, b, c = (np.zeros(capacity, dtype=np.int32) for _ in range(3))
    st = start_ids if len(start_ids) else np.zeros(1, dtype=np.int32)
    rc = fn(C.c_int64(num_nodes), _p(ids), _p(ids_offsets), C.c_int32(S), C.c_int64(cap),
            _p(st), C.c_int64(len(start_ids)), _p(final_ids), _p(init_ids), _p(init_count),
            _p(a), _p(b), _p(c), C.c_int64(capacity), _p(cs_offsets), _p(miss))
    assert rc == 0
    n = int(cs_offsets[S])
    return dict(init_ids=init_ids[:int(init_count[0])], in_ids=a[:n], out_ids=b[:n],
                in_positions=c[:n], cs_offsets=cs_offsets, miss_count=miss[:S],
                final_ids=final_ids[:cap])


def changeset_resume(num_nodes, ids, ids_offsets, cap, start_ids):
    """Belady changesets from a given cache state (line r holds start_ids[r]); the result also
    holds ``final_ids``, the row of every line after the last iteration (-1 = empty)."""
    return _changeset_resume(lib().oracle_changeset_resume, num_nodes, ids, ids_offsets, cap,
                             start_ids)


def changeset_resume_by_sorting(num_nodes, ids, ids_offsets, cap, start_ids):
    return _changeset_resume(lib().oracle_changeset_resume_by_sorting, num_nodes, ids,
                             ids_offsets, cap, start_ids)


def changeset(num_nodes, ids, ids_offsets, cap):
    """Belady changesets with a priority queue (the variant used at scale)."""
    return _changeset(lib().oracle_changeset, num_nodes, ids, ids_offsets, cap)


def changeset_by_sorting(num_nodes, ids, ids_offsets, cap):
    """The same, straight from the definition (sort all candidates every iteration)."""
    return _changeset(lib().oracle_changeset_by_sorting, num_nodes, ids, ids_offsets, cap)


def changeset_lru(num_nodes, ids, ids_offsets, cap):
    """The same lists under the LRU policy (heap variant)."""
    return _changeset(lib().oracle_changeset_lru, num_nodes, ids, ids_offsets, cap)


def changeset_lru_by_sorting(num_nodes, ids, ids_offsets, cap):
    """LRU straight from the definition."""
    return _changeset(lib().oracle_changeset_lru_by_sorting, num_nodes, ids, ids_offsets, cap)


def lru_misses(num_nodes, ids, ids_offsets, cap, init_ids):
    ids, ids_offsets, init_ids = _i32(ids), _i64(ids_offsets), _i32(init_ids)
    return int(lib().oracle_lru_misses(
        C.c_int64(num_nodes), _p(ids), _p(ids_offsets), C.c_int32(len(ids_offsets) - 1),
        C.c_int64(cap), _p(init_ids), C.c_int64(len(init_ids))))


def static_select(num_nodes, indices, cap):
    """The ``cap`` nodes of highest out-degree (occurrences in ``indices``), larger degree
    first, smaller id first among equals."""
    indices = _i32(indices)
    out = np.zeros(max(min(cap, num_nodes), 1), dtype=np.int32)
    n = int(lib().oracle_static_select(C.c_int64(num_nodes), _p(indices),
                                       C.c_int64(len(indices)), C.c_int64(cap), _p(out)))
    return out[:n].copy()


def static_misses(num_nodes, ids, members):
    ids, members = _i32(ids), _i32(members)
    return int(lib().oracle_static_misses(C.c_int64(num_nodes), _p(ids), C.c_int64(len(ids)),
                                          _p(members), C.c_int64(len(members))))


def resolve_lines(num_nodes, ids, ids_offsets, init_ids, in_ids, out_ids, cs_offsets):
    """Address-table lookup result (cache line or -1) of every access, the table being set up
    from ``init_ids`` and patched with each iteration's update after that iteration's
    lookups."""
    ids, ids_offsets, init_ids = _i32(ids), _i64(ids_offsets), _i32(init_ids)
    in_ids, out_ids, cs_offsets = _i32(in_ids), _i32(out_ids), _i64(cs_offsets)
    lines = np.zeros(max(len(ids), 1), dtype=np.int32)
    lib().oracle_resolve_lines(C.c_int64(num_nodes), _p(ids), _p(ids_offsets),
                               C.c_int32(len(ids_offsets) - 1), _p(init_ids),
                               C.c_int64(len(init_ids)), _p(in_ids), _p(out_ids), _p(cs_offsets),
                               _p(lines))
    return lines[:len(ids)]


def _bytes2d(a):
    a = np.ascontiguousarray(a)
    return a.view(np.uint8).reshape(a.shape[0], -1)


def gather(slow, ids):
    """out[p] = slow[ids[p]] (rows compared as bytes)."""
    s = _bytes2d(slow)
    ids = _i32(ids)
    out = np.zeros((len(ids), s.shape[1]), dtype=np.uint8)
    lib().oracle_gather(_p(s), C.c_int64(s.shape[1]), _p(ids), C.c_int64(len(ids)), _p(out))
    return out


class Cache:
    """The executor's cache replayed on the CPU: 2-D cache array + address table."""

    def __init__(self, slow, cap):
        self.slow = _bytes2d(slow)
        self.row_bytes = self.slow.shape[1]
        self.rows = np.zeros((max(cap, 1), self.row_bytes), dtype=np.uint8)
        self.addr = np.full(self.slow.shape[0], -1, dtype=np.int32)

    def init(self, init_ids):
        init_ids = _i32(init_ids)
        lib().oracle_cache_init(_p(self.rows), _p(self.addr), C.c_int64(len(self.addr)),
                                _p(self.slow), C.c_int64(self.row_bytes), _p(init_ids),
                                C.c_int64(len(init_ids)))

    def gather_update(self, ids, in_ids, out_ids, in_positions):
        ids, in_ids, out_ids, in_positions = map(_i32, (ids, in_ids, out_ids, in_positions))
        out = np.zeros((len(ids), self.row_bytes), dtype=np.uint8)
        hits = lib().oracle_gather_update(
            _p(self.rows), _p(self.addr), _p(self.slow), C.c_int64(self.row_bytes), _p(ids),
            C.c_int64(len(ids)), _p(out), _p(in_ids), _p(out_ids), _p(in_positions),
            C.c_int64(len(in_ids)))
        return out, int(hits)
