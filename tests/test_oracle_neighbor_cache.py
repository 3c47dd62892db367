"""Pins for the oracle's neighbour cache (CPU only): Section 3.2, policy and structure."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from workload import make_workload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def random_csr(rng, n, e):
    dst = rng.integers(0, n, size=e)
    src = rng.integers(0, n, size=e)
    order = np.argsort(dst, kind="stable")
    offsets = np.zeros(n + 1, dtype=np.int64)
    np.add.at(offsets, dst + 1, 1)
    return np.cumsum(offsets), src[order].astype(np.int32)


def test_lookup_on_the_layout_the_paper_describes():
    kv = {}
    for line in open(os.path.join(GOLDEN, "neighbor_cache_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        kv[key] = [int(x) for x in vals]
    at = np.array(kv["address_table"], dtype=np.int64)
    ca = np.array(kv["cache_array"], dtype=np.int32)
    v = kv["stated_node"][0]
    assert at[v] == kv["stated_address"][0] and ca[at[v]] == kv["stated_count"][0]
    got = oracle.neighbor_lookup(at, ca, v)
    lo, hi = kv["stated_first_neighbor_index"][0], kv["stated_last_neighbor_index"][0]
    assert np.array_equal(got, ca[lo:hi + 1]) and len(got) == kv["stated_count"][0]
    for u in range(kv["num_nodes"][0]):
        res = oracle.neighbor_lookup(at, ca, u)
        assert (res is not None) == (u in kv["cached_nodes"])
    assert list(oracle.neighbor_lookup(at, ca, 5)) == [0, 7]
    assert list(oracle.neighbor_lookup(at, ca, 9)) == [1, 4, 5]


def test_selection_is_the_exact_ratio_ranking_and_the_layout_is_dense():
    rng = np.random.default_rng(3)
    for trial in range(120):
        n = int(rng.integers(1, 60))
        e = int(rng.integers(0, 400))
        off, ind = random_csr(rng, n, e)
        if trial % 2:
            off = off.astype(np.int32)
        in_deg = np.diff(off)
        out_deg = np.bincount(ind, minlength=n)
        # exact rationals: with degrees this small the 2^-32 quantisation cannot reorder
        rank = sorted((v for v in range(n) if in_deg[v] > 0),
                      key=lambda v: (-Fraction(int(out_deg[v]), int(in_deg[v])), v))
        for budget in (0, 1, 2, int(rng.integers(0, e + n + 2)), e + n):
            at, ca, cached = oracle.neighbor_cache_build(off, ind, budget)
            want, used = [], 0
            for v in rank:
                if used + 1 + in_deg[v] > budget:
                    break
                want.append(v)
                used += 1 + int(in_deg[v])
            assert cached == len(want) and len(ca) == used <= budget
            assert sorted(np.nonzero(at >= 0)[0].tolist()) == sorted(want)
            pos = 0
            for v in want:                      # records in rank order, back to back
                assert at[v] == pos and ca[pos] == in_deg[v]
                assert np.array_equal(ca[pos + 1:pos + 1 + in_deg[v]], ind[off[v]:off[v + 1]])
                assert np.array_equal(oracle.neighbor_lookup(at, ca, v), ind[off[v]:off[v + 1]])
                pos += 1 + int(in_deg[v])
            for v in set(range(n)) - set(want):
                assert at[v] == -1 and oracle.neighbor_lookup(at, ca, v) is None
        # a budget for everything caches every node that has neighbours
        at, ca, cached = oracle.neighbor_cache_build(off, ind, e + n)
        assert cached == int((in_deg > 0).sum()) and len(ca) == e + cached


def test_a_hub_that_is_cheap_to_keep_ranks_first():
    # node 0 is everyone's neighbour and has one neighbour itself; node 1 has many
    # neighbours and is nobody's: 0 must be cached first, 1 last
    n = 8
    rows = {0: [2], 1: [0, 2, 3, 4, 5, 6, 7], 2: [0], 3: [0, 2], 4: [0], 5: [0, 3], 6: [0], 7: [0]}
    off = np.cumsum([0] + [len(rows[v]) for v in range(n)]).astype(np.int64)
    ind = np.array([u for v in range(n) for u in rows[v]], dtype=np.int32)
    at, ca, cached = oracle.neighbor_cache_build(off, ind, 2)
    assert cached == 1 and at[0] == 0 and list(ca) == [1, 2]
    at, ca, cached = oracle.neighbor_cache_build(off, ind, len(ind) + n - 1)
    assert cached == n - 1 and at[1] == -1      # everything but the costly, useless row


@pytest.fixture(scope="module")
def tiny():
    return make_workload(1, features=False)


def test_sampling_through_the_cache_equals_sampling_without_it(tiny):
    w = tiny
    off, ind = w.offsets.numpy(), w.indices.numpy()
    args = (off, ind, w.seeds.numpy(), w.seed_offsets.numpy(), w.cfg.fanout)
    plain = oracle.sample_superbatch(*args)
    lookups = plain["hop_sizes"][:, :-1].sum()          # one row fetch per frontier node
    previous_hits = -1
    for budget in (0, 1000, len(ind) // 10, len(ind) // 2, len(ind) + len(off)):
        at, ca, cached = oracle.neighbor_cache_build(off, ind, budget)
        got = oracle.sample_superbatch(*args, neighbor_cache=(at, ca))
        for k in plain:
            if k != "lookups":
                assert np.array_equal(plain[k], got[k]), k
        hits, misses = got["lookups"]
        assert hits + misses == lookups
        assert hits >= previous_hits                      # a larger cache never hits less
        previous_hits = hits
        # hits counted independently from the sampled lists
        want_hits = 0
        for b in range(w.cfg.S):
            lo = got["ids_offsets"][b]
            for h in range(len(w.cfg.fanout)):
                front = got["ids"][lo:lo + got["hop_sizes"][b, h]]
                want_hits += int((at[front] >= 0).sum())
        assert hits == want_hits
    assert misses == (np.diff(off)[np.concatenate(
        [got["ids"][got["ids_offsets"][b]:got["ids_offsets"][b] + got["hop_sizes"][b, h]]
         for b in range(w.cfg.S) for h in range(len(w.cfg.fanout))])] == 0).sum()
