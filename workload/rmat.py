"""R-MAT graphs (Chakrabarti, Zhan, Faloutsos, SDM 2004) as CSR, from integer hashing only.

Every random word is a SplitMix64-style hash of (seed, edge index, attempt, level), computed
with wrapping int64 torch ops, so a given seed yields the same graph on any device.  The
quadrant of each level is chosen by comparing a 32-bit word with integer thresholds.
Multi-edges and self-loops are kept, so the edge count is exact.
"""
from __future__ import annotations

import math
import sys

import torch

_MASK64 = (1 << 64) - 1


def _s64(x: int) -> int:
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


_GOLD = _s64(0x9E3779B97F4A7C15)
_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    return (z >> s) & ((1 << (64 - s)) - 1)


def mix64(z: torch.Tensor) -> torch.Tensor:
    """SplitMix64 finaliser on an int64 tensor (bit pattern of the unsigned arithmetic)."""
    z = z + _GOLD
    z = (z ^ _lsr(z, 30)) * _C1
    z = (z ^ _lsr(z, 27)) * _C2
    return z ^ _lsr(z, 31)


def mix64_int(x: int) -> int:
    z = (x + 0x9E3779B97F4A7C15) & _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def _rmat_endpoints(e: torch.Tensor, attempt: int, scale: int, thr, key: int):
    """(src, dst) in [0, 2**scale) for the edge indices ``e`` (int64 tensor)."""
    base = mix64(e ^ _s64(key))
    base = mix64(base + _s64(attempt * 0xD1B54A32D192ED03))
    src = torch.zeros_like(e)
    dst = torch.zeros_like(e)
    a, ab, abc = thr
    for pair in range((scale + 1) // 2):
        w = mix64(base + pair)
        for half in range(2):
            level = 2 * pair + half
            if level >= scale:
                break
            w32 = _lsr(w, 32) if half else (w & 0xFFFFFFFF)
            q = (w32 >= a).to(torch.int64) + (w32 >= ab).to(torch.int64) \
                + (w32 >= abc).to(torch.int64)
            src = (src << 1) | (q >> 1)
            dst = (dst << 1) | (q & 1)
    return src, dst


def _coprime_multiplier(n: int, key: int) -> int:
    m = (mix64_int(key) % n) | 1
    while math.gcd(m, n) != 1:
        m += 2
    return m % n if n > 1 else 0


def _say(verbose, *a):
    if verbose:
        print("[workload]", *a, file=sys.stderr, flush=True)


def _edge_chunks(num_nodes: int, num_edges: int, abc, seed: int, device, chunk: int,
                 verbose: bool):
    """Yields (src, dst) int64 tensors, `chunk` edges at a time, endpoints < num_nodes,
    ids relabelled by a seeded affine bijection so that hubs are spread over the id range."""
    scale = max(1, math.ceil(math.log2(num_nodes)))
    a, b, c = abc
    thr = (int(a * 2 ** 32), int((a + b) * 2 ** 32), int((a + b + c) * 2 ** 32))
    key = mix64_int(seed ^ 0x52D4A7)
    mul = _coprime_multiplier(num_nodes, key ^ 1)
    add = mix64_int(key ^ 2) % num_nodes
    for lo in range(0, num_edges, chunk):
        e = torch.arange(lo, min(lo + chunk, num_edges), dtype=torch.int64, device=device)
        src, dst = _rmat_endpoints(e, 0, scale, thr, key)
        for attempt in range(1, 64):
            bad = (src >= num_nodes) | (dst >= num_nodes)
            if not bool(bad.any()):
                break
            s2, d2 = _rmat_endpoints(e[bad], attempt, scale, thr, key)
            src[bad] = s2
            dst[bad] = d2
        src %= num_nodes
        dst %= num_nodes
        if (lo // chunk) % 8 == 7:
            _say(verbose, f"edges {lo + chunk} / {num_edges}")
        # num_nodes < 2**28 and mul < num_nodes: the product stays below 2**56
        yield (src * mul + add) % num_nodes, (dst * mul + add) % num_nodes


def rmat_edges(num_nodes: int, num_edges: int, abc, seed: int, device="cpu",
               chunk: int = 1 << 25, verbose: bool = False):
    """All ``num_edges`` directed edges as two int64 tensors (src, dst)."""
    parts = list(_edge_chunks(num_nodes, num_edges, abc, seed, device, chunk, verbose))
    return torch.cat([p[0] for p in parts]), torch.cat([p[1] for p in parts])


def rmat_csr(num_nodes: int, num_edges: int, abc, seed: int, device="cpu",
             symmetrise: bool = False, offsets_64: bool | None = None,
             verbose: bool = False, chunk: int = 1 << 25):
    """CSR whose row v lists the sources of the edges that end in v (its in-neighbours),
    sorted by (row, column).  With ``symmetrise`` the reverse of every edge is added, so
    the result holds 2*num_edges entries.  Returns (offsets, indices) on ``device``.

    Edges are binned by row range while they are drawn and every bin is sorted on its own,
    so no single sort exceeds 2**28 keys; the result does not depend on the binning."""
    total = num_edges * (2 if symmetrise else 1)
    bins = max(1, -(-total // (1 << 28)))
    rows_per_bin = -(-num_nodes // bins)
    binned = [[] for _ in range(bins)]
    for src, dst in _edge_chunks(num_nodes, num_edges, abc, seed, device, chunk, verbose):
        pairs = [(src, dst), (dst, src)] if symmetrise else [(src, dst)]
        for col, row in pairs:
            key = row * num_nodes + col
            if bins == 1:
                binned[0].append(key)
                continue
            which = row // rows_per_bin
            order = torch.argsort(which)
            key = key[order]
            cuts = torch.cumsum(torch.bincount(which, minlength=bins), 0).tolist()
            lo = 0
            for b in range(bins):
                if cuts[b] > lo:
                    binned[b].append(key[lo:cuts[b]].clone())
                lo = cuts[b]
    _say(verbose, f"edges drawn; sorting {bins} row bins into CSR")
    index_parts = []
    counts = torch.zeros(num_nodes, dtype=torch.int64, device=device)
    for b in range(bins):
        if not binned[b]:
            continue
        key = torch.sort(torch.cat(binned[b]))[0]
        binned[b] = None
        index_parts.append((key % num_nodes).to(torch.int32))
        row = key // num_nodes
        del key
        lo = b * rows_per_bin
        hi = min(lo + rows_per_bin, num_nodes)
        counts[lo:hi] = torch.bincount(row - lo, minlength=hi - lo)
        del row
    indices = torch.cat(index_parts) if index_parts else torch.zeros(0, dtype=torch.int32,
                                                                       device=device)
    del index_parts
    _say(verbose, "sorted")
    if offsets_64 is None:
        offsets_64 = total >= 2 ** 31
    offsets = torch.zeros(num_nodes + 1, dtype=torch.int64, device=indices.device)
    torch.cumsum(counts, 0, out=offsets[1:])
    if not offsets_64:
        offsets = offsets.to(torch.int32)
    return offsets, indices
