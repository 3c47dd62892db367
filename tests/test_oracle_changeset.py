"""Pins for the oracle's next-use computation and Belady changesets (CPU only).

Section 3.3 (cache policy, update lists) and Section 3.4 (recurrence, tracking).
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle.tracker import NextAccessTracker
from workload import make_workload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
NEVER = oracle.NEVER


def flat(ids_list):
    off = np.cumsum([0] + [len(x) for x in ids_list]).astype(np.int64)
    ids = np.array([v for x in ids_list for v in x], dtype=np.int32)
    return ids, off


def random_trace(rng, n, S, max_len):
    return [list(rng.choice(n, size=rng.integers(0, min(max_len, n) + 1), replace=False))
            for _ in range(S)]


def naive_next_use(ids_list):
    """The O(S^2) forward scan the paper rejects (Section 3.4), as a cross-check."""
    out = []
    for i, ids in enumerate(ids_list):
        for v in ids:
            nxt = NEVER
            for j in range(i + 1, len(ids_list)):
                if v in ids_list[j]:
                    nxt = j
                    break
            out.append(nxt)
    return out


def test_next_use_against_forward_scan_and_tracker():
    rng = np.random.default_rng(0)
    for _ in range(200):
        n, S = int(rng.integers(1, 12)), int(rng.integers(1, 9))
        tr = random_trace(rng, n, S, 6)
        ids, off = flat(tr)
        nxt, first = oracle.next_use(n, ids, off)
        assert list(nxt) == naive_next_use(tr)
        t = NextAccessTracker(n, tr)
        for v in range(n):
            if t.count[v]:
                assert t.next_access(v) == first[v]
            else:
                assert first[v] == NEVER
        p = 0
        for i, cur in enumerate(tr):
            t.advance(cur)
            for v in cur:
                assert t.next_access(v) == nxt[p]
                p += 1


def test_tracker_reproduces_the_values_the_paper_states():
    kv, trace = {}, []
    for line in open(os.path.join(GOLDEN, "next_access_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        if k == "ids":
            trace.append([int(x) for x in v])
        else:
            kv[k] = [int(x) for x in v]
    n = kv["num_nodes"][0]
    t = NextAccessTracker(n, trace)
    assert t.ptr[3] == kv["ptr3"][0] and t.ptr[4] == kv["ptr4"][0]
    assert [x & 0x7FFFFFFF for x in t.iters[t.ptr[3]:t.ptr[3] + 3]] == kv["node3_iters"]
    assert t.dummy_index == kv["dummy_index"][0]
    assert t.iters[t.ptr[3]] >> 31 == 1            # head of node 3's run is marked
    t.advance(trace[0])
    assert t.ptr[3] == 5 and t.ptr[4] == 8         # both advanced by one
    t.advance(trace[1])
    assert t.ptr[2] == kv["ptr2_after_iteration1"][0]
    ids, off = flat(trace)
    nxt, first = oracle.next_use(n, ids, off)
    assert list(first) == [1, 2, 1, 0, 0]
    assert list(nxt) == [2, 3, NEVER, 3, 4, NEVER, 4, NEVER, NEVER, NEVER]


def replay(n, cap, tr, cs):
    """Replays the changesets, checking every structural invariant; returns the states."""
    cache = {int(v): s for s, v in enumerate(cs["init_ids"])}
    assert len(cache) == len(cs["init_ids"]) <= cap
    states, total_miss = [set(cache)], 0
    for i, cur in enumerate(tr):
        lo, hi = cs["cs_offsets"][i], cs["cs_offsets"][i + 1]
        ins, outs, pos = cs["in_ids"][lo:hi], cs["out_ids"][lo:hi], cs["in_positions"][lo:hi]
        misses = [v for v in cur if v not in cache]
        assert cs["miss_count"][i] == len(misses)
        total_miss += len(misses)
        assert set(ins) <= set(misses) and len(set(ins)) == len(ins)
        assert set(outs) <= set(cache) and len(set(outs)) == len(outs)
        assert not set(ins) & set(outs)
        assert all(cur[p] == v for p, v in zip(pos, ins))
        assert list(pos) == sorted(pos)
        slots = [cache[int(o)] for o in outs]
        assert slots == sorted(slots)
        for v, o in zip(ins, outs):
            cache[int(v)] = cache.pop(int(o))
        assert len(cache) <= cap and len(set(cache.values())) == len(cache)
        states.append(set(cache))
    return states, total_miss


def optimal_misses(tr, cap, c0=None):
    """Exhaustive search: every C_{i+1} that is a subset of C_i union ids_i with at most
    `cap` rows is tried.  With c0=None every initial state is tried as well."""
    S = len(tr)
    memo = {}

    def go(i, cache):
        if i == S:
            return 0
        key = (i, cache)
        if key not in memo:
            cur = frozenset(tr[i])
            miss = len(cur - cache)
            pool = sorted(cache | cur)
            best = None
            for r in range(min(cap, len(pool)) + 1):
                for nxt in itertools.combinations(pool, r):
                    c = go(i + 1, frozenset(nxt))
                    best = c if best is None else min(best, c)
            memo[key] = miss + best
        return memo[key]

    if c0 is not None:
        return go(0, frozenset(c0))
    nodes = sorted({v for x in tr for v in x})
    return min(go(0, frozenset(c)) for r in range(min(cap, len(nodes)) + 1)
               for c in itertools.combinations(nodes, r))


def test_belady_is_optimal_by_exhaustive_search():
    rng = np.random.default_rng(3)
    checked_pressure = 0
    for _ in range(300):
        n, S, cap = int(rng.integers(2, 7)), int(rng.integers(1, 6)), int(rng.integers(0, 4))
        tr = [[int(v) for v in x] for x in random_trace(rng, n, S, 3)]
        ids, off = flat(tr)
        cs = oracle.changeset(n, ids, off, cap)
        _, total = replay(n, cap, tr, cs)
        assert total == int(cs["miss_count"].sum())
        assert total == optimal_misses(tr, cap, [int(v) for v in cs["init_ids"]])
        assert total == optimal_misses(tr, cap)           # C_0 is an optimal start too
        checked_pressure += total > 0
    assert checked_pressure > 100


def test_heap_variant_equals_the_definition_and_the_recurrence():
    rng = np.random.default_rng(5)
    for _ in range(300):
        n, S, cap = int(rng.integers(1, 40)), int(rng.integers(1, 12)), int(rng.integers(0, 12))
        tr = [[int(v) for v in x] for x in random_trace(rng, n, S, 15)]
        ids, off = flat(tr)
        a = oracle.changeset(n, ids, off, cap)
        b = oracle.changeset_by_sorting(n, ids, off, cap)
        for k in a:
            assert np.array_equal(a[k], b[k]), k
        states, _ = replay(n, cap, tr, a)
        nxt, first = oracle.next_use(n, ids, off)
        # C_0: the cap smallest (first access, id); line r = rank
        order = sorted((first[v], v) for v in range(n) if first[v] != NEVER)[:cap]
        assert [v for _, v in order] == list(a["init_ids"])
        # C_{i+1} = the cap smallest of union(C_i, ids_i) by (next access, incoming, id)
        key = {v: first[v] for v in range(n)}
        p = 0
        for i, cur in enumerate(tr):
            for v in cur:
                key[v] = nxt[p]
                p += 1
            cand = sorted((key[v], v not in states[i], v) for v in states[i] | set(cur))
            assert {v for _, _, v in cand[:cap]} == states[i + 1]
            assert states[i + 1] <= states[i] | set(cur)


def test_last_record_is_empty_and_full_fit_never_changes():
    rng = np.random.default_rng(7)
    for _ in range(50):
        n, S = 20, 6
        tr = [[int(v) for v in x] for x in random_trace(rng, n, S, 8)]
        ids, off = flat(tr)
        cs = oracle.changeset(n, ids, off, 5)
        assert cs["cs_offsets"][S] == cs["cs_offsets"][S - 1]   # S records, the last is empty
        distinct = len(set(ids.tolist()))
        full = oracle.changeset(n, ids, off, distinct)
        assert len(full["init_ids"]) == distinct and full["cs_offsets"][S] == 0
        assert full["miss_count"].sum() == 0
        # init_count + misses >= distinct, with equality iff everything fits
        assert len(cs["init_ids"]) + cs["miss_count"].sum() >= distinct


@pytest.fixture(scope="module")
def tiny():
    w = make_workload(1, features=False)
    r = oracle.sample_superbatch(w.offsets.numpy(), w.indices.numpy(), w.seeds.numpy(),
                                 w.seed_offsets.numpy(), w.cfg.fanout)
    return w, r


def test_invariants_and_policy_bounds_on_tiny_config(tiny):
    w, r = tiny
    n, cap = w.cfg.num_nodes, w.cfg.cap
    cs = oracle.changeset(n, r["ids"], r["ids_offsets"], cap)
    tr = [r["ids"][r["ids_offsets"][i]:r["ids_offsets"][i + 1]].tolist()
          for i in range(w.cfg.S)]
    _, total = replay(n, cap, tr, cs)
    # the cache (2048 rows) is smaller than one iteration's ids: rows must bypass it
    assert cap < min(len(x) for x in tr)
    assert total <= oracle.lru_misses(n, r["ids"], r["ids_offsets"], cap, cs["init_ids"])
    deg = (w.offsets[1:] - w.offsets[:-1]).numpy()
    out_deg = np.bincount(w.indices.numpy(), minlength=n)
    for score in (deg, out_deg):
        top = np.argsort(-score, kind="stable")[:cap]
        assert total <= oracle.static_misses(n, r["ids"], top)
    b = oracle.changeset_by_sorting(n, r["ids"], r["ids_offsets"], cap)
    for k in cs:
        assert np.array_equal(cs[k], b[k]), k


def test_lru_helper_counts_misses_of_a_plain_lru():
    # 3 lines, one id per iteration: textbook LRU
    tr = [[1], [2], [3], [1], [4], [2], [1]]
    ids, off = flat(tr)
    # start empty: 1,2,3 miss; 1 hit; 4 miss (evicts 2); 2 miss (evicts 3); 1 hit
    assert oracle.lru_misses(5, ids, off, 3, np.array([], dtype=np.int32)) == 5


# ---- LRU changesets (Section 2.3: the policy Belady's is compared with) -----------------

def list_lru(cap, init, trace):
    """A textbook LRU list for one id per iteration: front = most recently used.  The
    prefetched rows have not been used: among them the larger id leaves first."""
    order = sorted(init)
    misses, states = 0, [set(order)]
    for v in trace:
        if v in order:
            order.remove(v)
        else:
            misses += 1
            if len(order) == cap:
                order.pop()
        order.insert(0, v)
        states.append(set(order))
    return misses, states


def test_lru_changesets_on_a_cyclic_trace_miss_every_access_after_the_prefetch():
    # cap rows, cap+1 ids accessed round-robin, one per iteration: after the cap prefetched
    # rows are used once, LRU always evicts the row needed next, Belady one row per cycle
    for cap in (1, 2, 3, 5):
        S = 6 * (cap + 1)
        tr = [[i % (cap + 1)] for i in range(S)]
        ids, off = flat(tr)
        lru = oracle.changeset_lru(cap + 1, ids, off, cap)
        assert list(lru["init_ids"]) == list(range(cap))
        assert list(lru["miss_count"]) == [0] * cap + [1] * (S - cap)
        # every miss is inserted and evicts the row that is accessed next
        assert list(lru["in_ids"]) == [i % (cap + 1) for i in range(cap, S)]
        assert list(lru["out_ids"]) == [(i + 1) % (cap + 1) for i in range(cap, S)]
        bel = oracle.changeset(cap + 1, ids, off, cap)
        assert bel["miss_count"].sum() < lru["miss_count"].sum() or cap == 1


def test_lru_changesets_equal_a_textbook_lru_list_for_single_accesses():
    rng = np.random.default_rng(21)
    for _ in range(300):
        n, S, cap = int(rng.integers(1, 12)), int(rng.integers(1, 40)), int(rng.integers(1, 8))
        trace = [int(v) for v in rng.integers(0, n, size=S)]
        tr = [[v] for v in trace]
        ids, off = flat(tr)
        cs = oracle.changeset_lru(n, ids, off, cap)
        states, total = replay(n, cap, tr, cs)
        misses, want = list_lru(cap, [int(v) for v in cs["init_ids"]], trace)
        assert total == misses
        assert states == want


def test_lru_heap_variant_equals_the_definition_and_the_miss_counter():
    rng = np.random.default_rng(22)
    for _ in range(300):
        n, S, cap = int(rng.integers(1, 40)), int(rng.integers(1, 12)), int(rng.integers(0, 12))
        tr = [[int(v) for v in x] for x in random_trace(rng, n, S, 15)]
        ids, off = flat(tr)
        a = oracle.changeset_lru(n, ids, off, cap)
        b = oracle.changeset_lru_by_sorting(n, ids, off, cap)
        for k in a:
            assert np.array_equal(a[k], b[k]), k
        bel = oracle.changeset(n, ids, off, cap)
        assert np.array_equal(a["init_ids"], bel["init_ids"])        # the same prefetch
        states, total = replay(n, cap, tr, a)
        assert bel["miss_count"].sum() <= total                       # Belady is optimal
        # the state after iteration i: the cap most recently used rows of union(C_i, ids_i);
        # never-used prefetched rows are the oldest; ties: resident first, then smaller id
        last = {int(v): -1 for v in a["init_ids"]}
        for i, cur in enumerate(tr):
            for v in cur:
                last[v] = i
            cand = sorted((-last[v], v not in states[i], v) for v in states[i] | set(cur))
            assert {v for _, _, v in cand[:cap]} == states[i + 1]
        # the stand-alone LRU miss counter knows no resident-before-incoming rule: the two
        # agree whenever no iteration is longer than the cache
        if cap > 0 and all(len(x) <= cap for x in tr):
            assert total == oracle.lru_misses(n, ids, off, cap, a["init_ids"])


def test_lru_on_tiny_config_sits_between_belady_and_all_miss(tiny):
    w, r = tiny
    n = w.cfg.num_nodes
    tr = [r["ids"][r["ids_offsets"][i]:r["ids_offsets"][i + 1]].tolist() for i in range(w.cfg.S)]
    for cap in (w.cfg.cap, 4 * max(len(x) for x in tr)):
        lru = oracle.changeset_lru(n, r["ids"], r["ids_offsets"], cap)
        _, total = replay(n, cap, tr, lru)
        bel = oracle.changeset(n, r["ids"], r["ids_offsets"], cap)
        assert bel["miss_count"].sum() <= total <= len(r["ids"])
        if cap >= max(len(x) for x in tr):
            assert total == oracle.lru_misses(n, r["ids"], r["ids_offsets"], cap, lru["init_ids"])


# ---- changesets from a carried cache state (an extension; Section 3.1 re-initializes) ------

def replay_lines(cap, start, tr, cs):
    """Replays changesets on explicit cache lines; rows beyond the evicted ones take the free
    lines in ascending order.  Returns the per-iteration states and the final line table."""
    lines = [-1] * cap
    for r, v in enumerate(start):
        lines[r] = int(v)
    where = {v: r for r, v in enumerate(lines) if v >= 0}
    states, total = [set(where)], 0
    for i, cur in enumerate(tr):
        lo, hi = cs["cs_offsets"][i], cs["cs_offsets"][i + 1]
        ins, outs, pos = cs["in_ids"][lo:hi], cs["out_ids"][lo:hi], cs["in_positions"][lo:hi]
        misses = [v for v in cur if v not in where]
        assert cs["miss_count"][i] == len(misses)
        total += len(misses)
        assert all(cur[p] == v for p, v in zip(pos, ins)) and list(pos) == sorted(pos)
        freed = []
        for o in outs:
            if o >= 0:
                freed.append(where.pop(int(o)))
                lines[freed[-1]] = -1
        assert freed == sorted(freed)
        for j, v in enumerate(ins):
            assert v in misses
            line = freed[j] if j < len(freed) else lines.index(-1)
            lines[line] = int(v)
            where[int(v)] = line
        assert len(where) <= cap
        states.append(set(where))
    return states, total, lines


def test_resume_from_the_standard_prefetch_is_the_standard_changeset():
    rng = np.random.default_rng(31)
    for _ in range(200):
        n, S, cap = int(rng.integers(1, 40)), int(rng.integers(1, 12)), int(rng.integers(0, 12))
        tr = [[int(v) for v in x] for x in random_trace(rng, n, S, 15)]
        ids, off = flat(tr)
        std = oracle.changeset(n, ids, off, cap)
        res = oracle.changeset_resume(n, ids, off, cap, std["init_ids"])
        for k in std:
            assert np.array_equal(std[k], res[k]), k
        _, _, lines = replay_lines(cap, std["init_ids"], tr, std)
        assert list(res["final_ids"]) == lines


def test_resume_heap_equals_definition_and_is_optimal_for_its_start_state():
    rng = np.random.default_rng(32)
    pressure = 0
    for trial in range(300):
        small = trial % 2 == 0          # small cases also go through the exhaustive search
        n = int(rng.integers(2, 7 if small else 40))
        S = int(rng.integers(1, 6 if small else 12))
        cap = int(rng.integers(0, 4 if small else 12))
        tr = [[int(v) for v in x] for x in random_trace(rng, n, S, 3 if small else 15)]
        ids, off = flat(tr)
        start = rng.permutation(n)[:int(rng.integers(0, min(cap, n) + 1))].astype(np.int32)
        a = oracle.changeset_resume(n, ids, off, cap, start)
        b = oracle.changeset_resume_by_sorting(n, ids, off, cap, start)
        for k in a:
            assert np.array_equal(a[k], b[k]), k
        assert np.array_equal(a["init_ids"], start)
        states, total, lines = replay_lines(cap, start, tr, a)
        assert list(a["final_ids"]) == lines
        # the recurrence, with rows that are never accessed ranked last
        nxt, first = oracle.next_use(n, ids, off)
        key = {v: first[v] for v in range(n)}
        p = 0
        for i, cur in enumerate(tr):
            for v in cur:
                key[v] = nxt[p]
                p += 1
            cand = sorted((key[v], v not in states[i], v) for v in states[i] | set(cur))
            assert {v for _, _, v in cand[:cap]} == states[i + 1]
        if small:
            assert total == optimal_misses(tr, cap, [int(v) for v in start])
            pressure += total > 0
    assert pressure > 50


def test_resumed_superbatches_chain_through_their_final_states():
    rng = np.random.default_rng(33)
    for _ in range(50):
        n, cap = 30, int(rng.integers(1, 12))
        state = rng.permutation(n)[:cap].astype(np.int32)
        for k in range(4):
            tr = [[int(v) for v in x] for x in random_trace(rng, n, 6, 10)]
            ids, off = flat(tr)
            cs = oracle.changeset_resume(n, ids, off, cap, state)
            _, _, lines = replay_lines(cap, state, tr, cs)
            assert list(cs["final_ids"]) == lines and -1 not in lines   # a full cache stays full
            # rows that both superbatches use and the cache kept are hits from the start
            assert cs["miss_count"][0] == len(set(tr[0]) - set(state.tolist()))
            state = cs["final_ids"]
