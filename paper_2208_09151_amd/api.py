"""Python names for the C entry points: tensors in, tensors out, nothing computed here."""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass

import numpy as np
import torch

from . import _lib
from ._lib import CacheDesc, CsrDesc


class GinexError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"ginex error {code}: {msg}")
        self.code = code


def library_path() -> str:
    return _lib.LIB_PATH


def version() -> int:
    return int(_lib.load().ginex_version())


def _check(rc):
    if rc != 0:
        raise GinexError(rc, _lib.load().ginex_last_error().decode())


def _dev(t: torch.Tensor, dtype=None) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError("expected a tensor in GPU memory")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    return t


def _readable(t: torch.Tensor, dtype=None) -> torch.Tensor:
    """Memory the GPU can read: device memory or pinned host memory."""
    if not (t.is_cuda or t.is_pinned()):
        raise ValueError("expected a tensor in GPU memory or in pinned host memory")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    return t


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _np_ptr(a):
    return C.c_void_p(a.ctypes.data)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


@dataclass
class SampleResult:
    ids: torch.Tensor               # flat int32, device
    ids_offsets: np.ndarray         # [S+1] int64, host
    hop_sizes: np.ndarray           # [S, H+1] int64, host
    adj_rowptr: torch.Tensor | None  # flat int64, device
    adj_col: torch.Tensor | None    # flat int32, device
    adj_row_offsets: np.ndarray     # [S*H+1], segment h*S+b (hop-major)
    adj_col_offsets: np.ndarray
    totals: np.ndarray              # ids, rowptr entries, col entries (= sampled edges)

    def adj_segment(self, b: int, h: int):
        S = len(self.ids_offsets) - 1
        g = h * S + b
        return (self.adj_rowptr[self.adj_row_offsets[g]:self.adj_row_offsets[g + 1]],
                self.adj_col[self.adj_col_offsets[g]:self.adj_col_offsets[g + 1]])


def sample_capacity(num_nodes, seed_offsets, fanout):
    """Upper bounds (ids, rowptr entries, col entries) for a superbatch."""
    ids = rows = cols = 0
    for b in range(len(seed_offsets) - 1):
        n = min(int(seed_offsets[b + 1] - seed_offsets[b]), num_nodes)
        for k in fanout:
            rows += n + 1
            cols += n * k
            n = min(n * (1 + k), num_nodes)
        ids += n
    return ids, rows, cols


@dataclass
class NeighborCache:
    address_table: torch.Tensor     # int64 [num_nodes], device
    cache_array: torch.Tensor       # int32 [budget], device
    cached_nodes: int
    used_entries: int


def neighbor_cache_build(offsets, indices, budget, device="cuda"):
    """ginex_neighbor_cache_build.  ``offsets``/``indices`` in device or pinned host memory;
    ``budget`` = entries of the cache array."""
    lib = _lib.load()
    _readable(offsets)
    _readable(indices, torch.int32)
    if offsets.dtype not in (torch.int32, torch.int64):
        raise ValueError("offsets must be int32 or int64")
    n = offsets.numel() - 1
    need = lib.ginex_neighbor_cache_workspace_bytes(n)
    if need == 0:
        raise GinexError(-1, lib.ginex_last_error().decode())
    ws = torch.empty(need, dtype=torch.uint8, device=device)
    address_table = torch.empty(n, dtype=torch.int64, device=device)
    cache_array = torch.empty(max(budget, 1), dtype=torch.int32, device=device)
    cached = np.zeros(1, dtype=np.int64)
    used = np.zeros(1, dtype=np.int64)
    g = CsrDesc(n, indices.numel(), offsets.data_ptr(), int(offsets.dtype == torch.int64),
                indices.data_ptr(), None, None)
    _check(lib.ginex_neighbor_cache_build(C.byref(g), budget, _ptr(address_table),
                                          _ptr(cache_array), _np_ptr(cached), _np_ptr(used),
                                          _ptr(ws), ws.numel(), _stream()))
    return NeighborCache(address_table, cache_array, int(cached[0]), int(used[0]))


def static_select(num_nodes, indices, cap, device="cuda"):
    """ginex_static_select: the ``cap`` nodes of highest out-degree (occurrences in
    ``indices``, device or pinned host int32), as a device int32 tensor in rank order."""
    lib = _lib.load()
    _readable(indices, torch.int32)
    need = lib.ginex_static_select_workspace_bytes(num_nodes)
    if need == 0:
        raise GinexError(-1, lib.ginex_last_error().decode())
    ws = torch.empty(need, dtype=torch.uint8, device=device)
    out = torch.empty(max(min(cap, num_nodes), 1), dtype=torch.int32, device=device)
    count = np.zeros(1, dtype=np.int64)
    g = CsrDesc(num_nodes, indices.numel(), None, 0, indices.data_ptr(), None, None)
    _check(lib.ginex_static_select(C.byref(g), cap, _ptr(out), _np_ptr(count), _ptr(ws),
                                   ws.numel(), _stream()))
    return out[:int(count[0])]


def sample_superbatch(offsets, indices, seeds, seed_offsets, fanout, rng_seed=0,
                      first_batch_index=0, with_adj=True, workspace=None, out=None,
                      neighbor_cache=None):
    """ginex_sample_superbatch.  ``seeds`` is a device tensor, ``offsets``/``indices`` device
    tensors or, for a graph that does not fit into HBM, pinned host tensors (then a
    ``neighbor_cache`` keeps the hot rows in HBM); ``seed_offsets`` and ``fanout`` are host
    sequences.  ``out`` may carry preallocated (ids, adj_rowptr, adj_col) device tensors."""
    lib = _lib.load()
    _readable(offsets)
    _readable(indices, torch.int32)
    _dev(seeds, torch.int32)
    if offsets.dtype not in (torch.int32, torch.int64):
        raise ValueError("offsets must be int32 or int64")
    so = np.ascontiguousarray(np.asarray(seed_offsets), dtype=np.int64)
    fo = np.ascontiguousarray(np.asarray(fanout), dtype=np.int32)
    S, H = len(so) - 1, len(fo)
    n = offsets.numel() - 1
    dev = seeds.device
    max_batch = int(np.max(np.diff(so))) if S > 0 else 0
    need = lib.ginex_sample_workspace_bytes(n, S, max_batch, _np_ptr(fo), H)
    if need == 0:
        raise GinexError(-1, lib.ginex_last_error().decode())
    ws = workspace if workspace is not None and workspace.numel() >= need else _workspace(need, dev)
    cap_ids, cap_rows, cap_cols = sample_capacity(n, so, fo)
    if out is not None:
        ids, rowptr, col = out
    else:
        ids = torch.empty(max(cap_ids, 1), dtype=torch.int32, device=dev)
        rowptr = torch.empty(max(cap_rows, 1), dtype=torch.int64, device=dev) if with_adj else None
        col = torch.empty(max(cap_cols, 1), dtype=torch.int32, device=dev) if with_adj else None
    ids_offsets = np.zeros(S + 1, dtype=np.int64)
    hop_sizes = np.zeros(S * (H + 1), dtype=np.int64)
    row_off = np.zeros(S * H + 1, dtype=np.int64)
    col_off = np.zeros(S * H + 1, dtype=np.int64)
    totals = np.zeros(3, dtype=np.int64)
    nc = neighbor_cache
    g = CsrDesc(n, indices.numel(), offsets.data_ptr(), int(offsets.dtype == torch.int64),
                indices.data_ptr(), nc.address_table.data_ptr() if nc else None,
                nc.cache_array.data_ptr() if nc else None)
    rc = lib.ginex_sample_superbatch(
        C.byref(g), _ptr(seeds), _np_ptr(so), S, _np_ptr(fo), H, rng_seed, first_batch_index,
        _ptr(ids), ids.numel(), _np_ptr(ids_offsets), _np_ptr(hop_sizes),
        _ptr(rowptr), rowptr.numel() if rowptr is not None else 0,
        _ptr(col), col.numel() if col is not None else 0,
        _np_ptr(row_off), _np_ptr(col_off), _np_ptr(totals), _ptr(ws), ws.numel(), _stream())
    _check(rc)
    return SampleResult(ids[:totals[0]], ids_offsets, hop_sizes.reshape(S, H + 1),
                        rowptr[:totals[1]] if with_adj else None,
                        col[:totals[2]] if with_adj else None, row_off, col_off, totals)


@dataclass
class ChangesetResult:
    init_ids: torch.Tensor      # int32 device, line r holds init_ids[r]
    in_ids: torch.Tensor
    out_ids: torch.Tensor
    in_positions: torch.Tensor
    cs_offsets: np.ndarray      # [S+1] host
    miss_count: np.ndarray      # [S] host
    init_ready: np.ndarray = None   # [S] host: rows of C_0 first accessed in iterations 0..i
    final_ids: torch.Tensor = None  # resumed superbatches: row of every line after the last iteration
    src_line: torch.Tensor = None   # int32 device [total ids]: cache line of every access, -1 = miss


def changeset(num_nodes, ids, ids_offsets, cap, workspace=None, policy="belady",
              builtin_scratch=False, with_lines=True):
    """ginex_changeset (``policy="belady"``) or ginex_changeset_lru (``policy="lru"``).
    ``ids`` is a device int32 tensor, ``ids_offsets`` a host array.  ``builtin_scratch``:
    ginex_changeset_noalloc, which takes no workspace (small shapes only); the outputs are
    still allocated here, by the caller.  ``with_lines``: also ask for ``src_line``."""
    lib = _lib.load()
    if policy not in ("belady", "lru"):
        raise ValueError(f"unknown policy {policy!r}")
    if builtin_scratch and policy != "belady":
        raise ValueError("the allocation-free entry point exists for Belady changesets only")
    entry = lib.ginex_changeset if policy == "belady" else lib.ginex_changeset_lru
    _dev(ids, torch.int32)
    io = np.ascontiguousarray(np.asarray(ids_offsets), dtype=np.int64)
    S = len(io) - 1
    total = int(io[-1]) if S >= 0 else 0
    dev = ids.device
    if not builtin_scratch:
        need = lib.ginex_changeset_workspace_bytes(num_nodes, total, S, cap)
        if need == 0:
            raise GinexError(-1, lib.ginex_last_error().decode())
        ws = workspace if workspace is not None and workspace.numel() >= need \
            else _workspace(need, dev)
    init_ids = torch.empty(max(cap, 1), dtype=torch.int32, device=dev)
    cs_cap = max(total, 1)
    in_ids = torch.empty(cs_cap, dtype=torch.int32, device=dev)
    out_ids = torch.empty(cs_cap, dtype=torch.int32, device=dev)
    in_pos = torch.empty(cs_cap, dtype=torch.int32, device=dev)
    cs_off = torch.empty(S + 1, dtype=torch.int64, device=dev)
    miss = torch.empty(max(S, 1), dtype=torch.int64, device=dev)
    init_count = np.zeros(1, dtype=np.int64)
    total_changes = np.zeros(1, dtype=np.int64)
    init_ready = np.zeros(max(S, 1), dtype=np.int64)
    lines = torch.empty(cs_cap, dtype=torch.int32, device=dev) if with_lines else None
    if builtin_scratch:
        rc = lib.ginex_changeset_noalloc(
            num_nodes, _ptr(ids), _np_ptr(io), S, cap, _ptr(init_ids), _np_ptr(init_count),
            _ptr(in_ids), _ptr(out_ids), _ptr(in_pos), cs_cap, _ptr(cs_off), _ptr(miss),
            _ptr(lines), _np_ptr(total_changes), _np_ptr(init_ready), _stream())
    else:
        rc = entry(num_nodes, _ptr(ids), _np_ptr(io), S, cap, _ptr(init_ids),
                   _np_ptr(init_count), _ptr(in_ids), _ptr(out_ids), _ptr(in_pos), cs_cap,
                   _ptr(cs_off), _ptr(miss), _ptr(lines), _np_ptr(total_changes),
                   _np_ptr(init_ready), _ptr(ws), ws.numel(), _stream())
    _check(rc)
    n = int(total_changes[0])
    return ChangesetResult(init_ids[:int(init_count[0])], in_ids[:n], out_ids[:n], in_pos[:n],
                           cs_off.cpu().numpy(), miss[:S].cpu().numpy(), init_ready[:S],
                           src_line=lines[:total] if with_lines else None)


def changeset_resume(num_nodes, ids, ids_offsets, start_ids, workspace=None, with_lines=True):
    """ginex_changeset_resume: Belady changesets from the cache state ``start_ids`` (device
    int32 [cap], line r holds start_ids[r]).  ``init_ids`` of the result echoes the start state,
    ``final_ids`` is the start state of the next superbatch."""
    lib = _lib.load()
    _dev(ids, torch.int32)
    _dev(start_ids, torch.int32)
    io = np.ascontiguousarray(np.asarray(ids_offsets), dtype=np.int64)
    S = len(io) - 1
    total = int(io[-1]) if S >= 0 else 0
    cap = start_ids.numel()
    dev = ids.device
    need = lib.ginex_changeset_workspace_bytes(num_nodes, total, S, cap)
    if need == 0:
        raise GinexError(-1, lib.ginex_last_error().decode())
    ws = workspace if workspace is not None and workspace.numel() >= need else _workspace(need, dev)
    final_ids = torch.empty(cap, dtype=torch.int32, device=dev)
    cs_cap = max(total, 1)
    in_ids = torch.empty(cs_cap, dtype=torch.int32, device=dev)
    out_ids = torch.empty(cs_cap, dtype=torch.int32, device=dev)
    in_pos = torch.empty(cs_cap, dtype=torch.int32, device=dev)
    cs_off = torch.empty(S + 1, dtype=torch.int64, device=dev)
    miss = torch.empty(max(S, 1), dtype=torch.int64, device=dev)
    total_changes = np.zeros(1, dtype=np.int64)
    lines = torch.empty(cs_cap, dtype=torch.int32, device=dev) if with_lines else None
    rc = lib.ginex_changeset_resume(num_nodes, _ptr(ids), _np_ptr(io), S, cap, _ptr(start_ids),
                                    _ptr(final_ids), _ptr(in_ids), _ptr(out_ids), _ptr(in_pos),
                                    cs_cap, _ptr(cs_off), _ptr(miss), _ptr(lines),
                                    _np_ptr(total_changes), _ptr(ws), ws.numel(), _stream())
    _check(rc)
    n = int(total_changes[0])
    return ChangesetResult(start_ids, in_ids[:n], out_ids[:n], in_pos[:n], cs_off.cpu().numpy(),
                           miss[:S].cpu().numpy(), np.full(S, cap, dtype=np.int64), final_ids,
                           src_line=lines[:total] if with_lines else None)


class FeatureCache:
    """The HBM feature cache: ``cap`` rows plus an address table, over a slow tier."""

    def __init__(self, slow: torch.Tensor, cap: int, device="cuda"):
        if slow.dim() != 2 or not slow.is_contiguous():
            raise ValueError("slow tier must be a contiguous 2-D tensor")
        if not (slow.is_cuda or slow.is_pinned()):
            raise ValueError("slow tier must be pinned host memory or device memory")
        self.slow = slow
        self.num_nodes = slow.shape[0]
        self.row_bytes = slow.shape[1] * slow.element_size()
        self.cap = cap
        self.rows = torch.empty((max(cap, 1), slow.shape[1]), dtype=slow.dtype, device=device)
        self.addr = torch.empty(self.num_nodes, dtype=torch.int32, device=device)
        self._desc = CacheDesc(self.rows.data_ptr(), cap, self.row_bytes, self.addr.data_ptr(),
                               self.num_nodes, slow.data_ptr())
        self._desc_ref = C.byref(self._desc)
        self._gather = _lib.load().ginex_gather
        self._gather_lines = _lib.load().ginex_gather_lines
        self._update = _lib.load().ginex_cache_update
        self._init_part = _lib.load().ginex_cache_init_part
        self._init_warm = _lib.load().ginex_cache_init_warm

    def init(self, init_ids: torch.Tensor):
        _dev(init_ids, torch.int32)
        _check(_lib.load().ginex_cache_init(C.byref(self._desc), _ptr(init_ids),
                                            init_ids.numel(), _stream()))

    def init_part_raw(self, init_ptr: int, begin: int, end: int, stream_ptr: int):
        """ginex_cache_init_part on raw device addresses: lines begin..end-1 of C_0."""
        rc = self._init_part(self._desc_ref, init_ptr, begin, end, stream_ptr)
        if rc:
            _check(rc)

    def init_warm_raw(self, prev: "FeatureCache", init_ptr: int, begin: int, end: int,
                      stream_ptr: int):
        """ginex_cache_init_warm: like init_part_raw, rows that ``prev`` holds come from it."""
        rc = self._init_warm(self._desc_ref, prev._desc_ref, init_ptr, begin, end, stream_ptr)
        if rc:
            _check(rc)

    def gather(self, ids, out=None, in_ids=None, out_ids=None, in_positions=None, src_line=None,
               n_slow=-1):
        """One executor iteration: gather the rows of ``ids`` then apply the changeset.  With
        ``src_line`` (the slice of ``ChangesetResult.src_line`` for this iteration) the gather
        is ginex_gather_lines and does not probe the address table; ``n_slow`` (the iteration's
        miss count, if known) lets it pick a launch shape that suits the host link."""
        _dev(ids, torch.int32)
        n = ids.numel()
        if out is None:
            out = torch.empty((n, self.slow.shape[1]), dtype=self.slow.dtype,
                              device=self.rows.device)
        nc = in_ids.numel() if in_ids is not None else 0
        lists = (_ptr(in_ids) if nc else None, _ptr(out_ids) if nc else None,
                 _ptr(in_positions) if nc else None, nc, _stream())
        if src_line is not None:
            _dev(src_line, torch.int32)
            if src_line.numel() != n:
                raise ValueError("src_line must have one entry per id")
            _check(self._gather_lines(C.byref(self._desc), _ptr(ids), _ptr(src_line), n, int(n_slow),
                                      _ptr(out), *lists))
        else:
            _check(self._gather(C.byref(self._desc), _ptr(ids), n, _ptr(out), *lists))
        return out

    def gather_raw(self, ids_ptr: int, n: int, out_ptr: int, stream_ptr: int):
        """ginex_gather with an empty changeset, on raw device addresses (for tight loops)."""
        rc = self._gather(self._desc_ref, ids_ptr, n, out_ptr, None, None, None, 0, stream_ptr)
        if rc:
            _check(rc)

    def gather_lines_raw(self, ids_ptr: int, lines_ptr: int, n: int, n_slow: int, out_ptr: int,
                         stream_ptr: int):
        """ginex_gather_lines with an empty changeset, on raw device addresses."""
        rc = self._gather_lines(self._desc_ref, ids_ptr, lines_ptr, n, n_slow, out_ptr, None, None,
                                None, 0, stream_ptr)
        if rc:
            _check(rc)

    def update_raw(self, out_ptr: int, in_ptr: int, outids_ptr: int, pos_ptr: int,
                   n_change: int, stream_ptr: int):
        """ginex_cache_update on raw device addresses (for tight loops)."""
        rc = self._update(self._desc_ref, out_ptr, in_ptr, outids_ptr, pos_ptr, n_change,
                          stream_ptr)
        if rc:
            _check(rc)

    def count_misses(self, ids, counter: torch.Tensor):
        """ginex_cache_count_misses: adds the number of ``ids`` not resident right now to
        ``counter`` (device int64, one element, zeroed by the caller)."""
        _dev(ids, torch.int32)
        _dev(counter, torch.int64)
        _check(_lib.load().ginex_cache_count_misses(C.byref(self._desc), _ptr(ids), ids.numel(),
                                                    _ptr(counter), _stream()))

    def update(self, out, in_ids, out_ids, in_positions):
        """The cache update alone, for a gather that was issued without a changeset."""
        nc = in_ids.numel() if in_ids is not None else 0
        _check(_lib.load().ginex_cache_update(C.byref(self._desc), _ptr(out),
                                              _ptr(in_ids) if nc else None,
                                              _ptr(out_ids) if nc else None,
                                              _ptr(in_positions) if nc else None, nc, _stream()))
