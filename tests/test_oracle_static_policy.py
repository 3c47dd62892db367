"""Pins for the oracle's static highest-out-degree cache (CPU only).

Section 2.3 "Challenge 1": the policy the paper compares Belady's with keeps the nodes of
highest out-degree in memory and never changes the cache.  The paper prints no worked
example of it, so the pins are graphs whose ranking is known in closed form, invariants
checked against library histograms, and hand-counted traces.
"""
import numpy as np

import oracle
from workload import make_workload


def test_select_on_graphs_whose_ranking_is_known():
    # star: every row lists node 5 only -> 5 first, then all others tie at 0 in id order
    n = 9
    star = np.full(n, 5, dtype=np.int32)
    assert oracle.static_select(n, star, 4).tolist() == [5, 0, 1, 2]
    # ladder: node v occurs v times -> descending ids
    ladder = np.concatenate([np.full(v, v, dtype=np.int32) for v in range(n)])
    assert oracle.static_select(n, ladder, n).tolist() == list(range(n - 1, -1, -1))
    assert oracle.static_select(n, ladder, 3).tolist() == [8, 7, 6]
    # order of the occurrences does not matter
    rng = np.random.default_rng(1)
    assert oracle.static_select(n, rng.permutation(ladder), 3).tolist() == [8, 7, 6]
    # all equal (each node once): id order; no edges at all: id order too
    assert oracle.static_select(n, np.arange(n, dtype=np.int32)[::-1].copy(), 5).tolist() == [0, 1, 2, 3, 4]
    assert oracle.static_select(n, np.zeros(0, dtype=np.int32), 3).tolist() == [0, 1, 2]
    # two tie groups: degrees 3,3,1,1,1,0 for nodes 4,2,5,1,0,3
    idx = np.array([4, 2, 4, 2, 5, 1, 0, 4, 2], dtype=np.int32)
    assert oracle.static_select(6, idx, 6).tolist() == [2, 4, 0, 1, 5, 3]
    # cap beyond the node count returns every node once; cap 0 returns nothing
    assert sorted(oracle.static_select(6, idx, 100).tolist()) == list(range(6))
    assert len(oracle.static_select(6, idx, 0)) == 0


def test_select_invariants_on_the_tiny_workload():
    w = make_workload(1, features=False)
    n = w.cfg.num_nodes
    indices = w.indices.numpy()
    deg = np.bincount(indices, minlength=n)          # library histogram, not the oracle's loop
    for cap in (1, 100, 2048, n):
        sel = oracle.static_select(n, indices, cap)
        assert len(sel) == cap and len(set(sel.tolist())) == cap
        d = deg[sel]
        assert np.all(d[:-1] >= d[1:])               # larger degree first
        same = d[:-1] == d[1:]
        assert np.all(sel[:-1][same] < sel[1:][same])  # smaller id first among equals
        rest = np.ones(n, dtype=bool)
        rest[sel] = False
        if rest.any():
            # nothing left out beats the last one taken, and a left-out node of the same
            # degree has a larger id
            assert deg[rest].max() <= d[-1]
            tied = np.flatnonzero(rest & (deg == d[-1]))
            assert tied.size == 0 or tied.min() > sel[d == d[-1]].max()
    # a smaller cache is a prefix of a larger one
    assert np.array_equal(oracle.static_select(n, indices, 100),
                          oracle.static_select(n, indices, 2048)[:100])


def test_static_misses_on_a_hand_counted_trace():
    # cache {1, 4}; accesses 1 2 4 | 4 4 0 | 3 1: the hits are 1, 4, 4, 4, 1 -> 3 misses of 8
    ids = np.array([1, 2, 4, 4, 4, 0, 3, 1], dtype=np.int32)
    assert oracle.static_misses(5, ids, np.array([1, 4], dtype=np.int32)) == 3
    assert oracle.static_misses(5, ids, np.array([4, 1], dtype=np.int32)) == 3
    assert oracle.static_misses(5, ids, np.zeros(0, dtype=np.int32)) == 8       # no cache
    assert oracle.static_misses(5, ids, np.arange(5, dtype=np.int32)) == 0      # everything cached
    assert oracle.static_misses(5, ids, np.array([2], dtype=np.int32)) == 7


def test_static_misses_equal_total_minus_the_members_access_counts():
    rng = np.random.default_rng(7)
    for _ in range(50):
        n = int(rng.integers(1, 60))
        ids = rng.integers(0, n, size=int(rng.integers(0, 400))).astype(np.int32)
        members = rng.choice(n, size=int(rng.integers(0, n + 1)), replace=False).astype(np.int32)
        counts = np.bincount(ids, minlength=n)
        assert oracle.static_misses(n, ids, members) == len(ids) - int(counts[members].sum())


def test_static_cache_replayed_through_the_executor_oracle_counts_the_same_misses():
    # the cache replay (init + gathers with empty changesets) must see exactly the misses the
    # counter reports, and return the slow tier's rows whatever the cache holds
    w = make_workload(1)
    cfg = w.cfg
    r = oracle.sample_superbatch(w.offsets.numpy(), w.indices.numpy(), w.seeds.numpy(),
                                 w.seed_offsets.numpy(), cfg.fanout)
    sel = oracle.static_select(cfg.num_nodes, w.indices.numpy(), cfg.cap)
    cache = oracle.Cache(w.features.numpy(), cfg.cap)
    cache.init(sel)
    none = np.zeros(0, dtype=np.int32)
    hits = 0
    for i in range(cfg.S):
        ids_i = r["ids"][r["ids_offsets"][i]:r["ids_offsets"][i + 1]]
        out, h = cache.gather_update(ids_i, none, none, none)
        hits += h
        assert np.array_equal(out, oracle.gather(w.features.numpy(), ids_i))
    assert len(r["ids"]) - hits == oracle.static_misses(cfg.num_nodes, r["ids"], sel)
