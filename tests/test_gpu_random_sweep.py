"""Randomised parity sweeps: many small random cases per entry point, shapes and switches drawn
at random from a fixed seed, every result compared with the oracle element by element."""
import numpy as np
import pytest
import torch

import oracle
from test_gpu_parity import check_changeset, check_resumed, check_sample, dev, ginex  # noqa: F401

pytestmark = pytest.mark.gpu


def _trace(rng, n, S, max_len, skew):
    tr = []
    for _ in range(S):
        m = int(rng.integers(0, min(max_len, n) + 1))
        if skew and m:                       # a few hot rows that come back in most iterations
            w = 1.0 / (1.0 + np.arange(n)) ** skew
            tr.append(rng.choice(n, size=m, replace=False, p=w / w.sum()))
        else:
            tr.append(rng.choice(n, size=m, replace=False))
    off = np.cumsum([0] + [len(x) for x in tr]).astype(np.int64)
    ids = np.concatenate(tr).astype(np.int32) if off[-1] else np.zeros(0, dtype=np.int32)
    return ids, off


def _ids(ids):
    return dev(ids) if len(ids) else torch.zeros(1, dtype=torch.int32, device="cuda")[:0]


def test_changeset_entry_points_on_random_traces(ginex, monkeypatch):
    """Belady, LRU, resumed (a cache that holds the trace and one that does not) and chains of
    resumed calls that hand final_ids on, 1 600 cases."""
    rng = np.random.default_rng(20261127)
    for trial in range(1600):
        big = rng.random() < 0.25
        n = int(rng.integers(2, 60000 if big else 600))
        S = int(rng.integers(1, 300 if rng.random() < 0.2 else 20))
        max_len = int(rng.integers(1, 4000 if big else 200))
        skew = 0.0 if n > 5000 else float(rng.choice([0.0, 0.0, 0.7, 1.2]))
        ids, off = _trace(rng, n, S, max_len, skew)
        distinct = max(len(np.unique(ids)), 1)
        kind = rng.choice(["belady", "lru", "resume", "chain"])
        try:
            monkeypatch.setenv("GINEX_STATIC_THRESHOLDS", "1" if rng.random() < 0.7 else "0")
            if kind in ("belady", "lru"):
                cap = int(rng.integers(0, n + 2)) if rng.random() < 0.5 else int(rng.integers(0, distinct + 1))
                ref = (oracle.changeset if kind == "belady" else oracle.changeset_lru)(n, ids, off, cap)
                res = ginex.changeset(n, _ids(ids), off, cap,
                                      **({"policy": "lru"} if kind == "lru" else {}))
                check_changeset(res, ref, (n, ids, off))
                continue
            holds = rng.random() < 0.6      # a line for every distinct row: no loop over the state
            cap = int(rng.integers(min(distinct, n), n + 1)) if holds else int(rng.integers(1, n + 1))
            way = str(rng.choice(["", "", "2", "0"]))   # as the library chooses, stepped, loop
            if way:
                monkeypatch.setenv("GINEX_PLANNED", way)
            else:
                monkeypatch.delenv("GINEX_PLANNED", raising=False)
            start = rng.permutation(n)[:cap].astype(np.int32)
            for _ in range(1 if kind == "resume" else int(rng.integers(2, 5))):
                ref = oracle.changeset_resume(n, ids, off, cap, start)
                res = ginex.changeset_resume(n, _ids(ids), off, dev(start))
                check_resumed(res, ref, (n, ids, off))
                start = ref["final_ids"].astype(np.int32)
                ids, off = _trace(rng, n, S, max_len, skew)
        except AssertionError:
            print("failing trial", trial, kind, n, S, max_len, skew, flush=True)
            raise


def test_sampler_on_random_graphs_batches_and_switches(ginex, monkeypatch):
    """Random R-MAT graphs (both offset widths), 1-3 hops with fanouts up to 64, batches from
    empty to 1 100 seeds with and without repeats, the hash sets in LDS or in HBM, several
    launch shapes; every fourth case feeds the sampled ids into ginex_changeset.  1 500 cases."""
    from workload import rmat_csr
    rng = np.random.default_rng(4242)
    graphs = []
    for g in range(10):
        n = int(rng.integers(10, 20000))
        off, ind = rmat_csr(n, int(n * rng.integers(1, 30)),
                            (0.5, 0.2, 0.2) if g % 2 else (0.45, 0.22, 0.22),
                            int(rng.integers(1, 1000)), "cpu", offsets_64=bool(g & 2))
        graphs.append((n, off.numpy(), ind.numpy(), off.cuda(), ind.cuda()))
    for trial in range(1500):
        n, off, ind, off_d, ind_d = graphs[int(rng.integers(0, len(graphs)))]
        H = int(rng.integers(1, 4))
        fanout = tuple(int(rng.integers(1, 26)) if rng.random() < 0.9 else int(rng.integers(26, 65))
                       for _ in range(H))
        S = int(rng.integers(1, 12))
        most = min(n, 1100 if rng.random() < 0.3 else 80)
        sizes = [int(rng.integers(0, most + 1)) for _ in range(S)]
        batches = [rng.choice(n, size=s, replace=bool(rng.random() < 0.1)) for s in sizes]
        seeds = np.concatenate(batches).astype(np.int32)
        so = np.cumsum([0] + sizes)
        rs, fb = int(rng.integers(0, 2**31)), int(rng.integers(0, 1000))
        monkeypatch.setenv("GINEX_SAMPLER_LDS", "1" if rng.random() < 0.7 else "0")
        tiles = str(rng.choice(["", "1", "3", "64"]))
        if tiles:
            monkeypatch.setenv("GINEX_SAMPLER_TILES", tiles)
        else:
            monkeypatch.delenv("GINEX_SAMPLER_TILES", raising=False)
        try:
            ref = oracle.sample_superbatch(off, ind, seeds, so, fanout, rng_seed=rs,
                                           first_batch_index=fb)
            res = ginex.sample_superbatch(off_d, ind_d, _ids(seeds), so, fanout, rng_seed=rs,
                                          first_batch_index=fb)
            check_sample(res, ref, S, H)
            if trial % 4 == 0 and len(ref["ids"]):
                cap = int(rng.integers(0, n + 1))
                cref = oracle.changeset(n, ref["ids"], ref["ids_offsets"], cap)
                cres = ginex.changeset(n, res.ids[:res.totals[0]], res.ids_offsets, cap)
                check_changeset(cres, cref, (n, ref["ids"], ref["ids_offsets"]))
        except AssertionError:
            print("failing trial", trial, n, fanout, sizes, rs, fb, flush=True)
            raise


def test_executor_on_random_traces_and_row_sizes(ginex):
    """Cache initialization, gather (through the resolved lines or through the address table)
    and update on random traces: every iteration's bytes, the address table and the cache rows
    against the oracle's replay, for Belady and LRU changesets and resumed ones (where the cache
    starts from the given rows), row sizes from 16 bytes to 3 KB.  1 500 cases."""
    rng = np.random.default_rng(9091)
    for trial in range(1500):
        n = int(rng.integers(2, 3000))
        S = int(rng.integers(1, 16))
        ids, off = _trace(rng, n, S, int(rng.integers(1, 400)), float(rng.choice([0.0, 0.0, 1.0])))
        row_words = int(rng.choice([4, 8, 12, 32, 36, 128, 200, 768]))
        slow = torch.from_numpy(rng.integers(-2**31, 2**31, size=(n, row_words), dtype=np.int64)
                                .astype(np.int32)).view(torch.float32).pin_memory()
        sb = slow.numpy().view(np.uint8).reshape(n, -1)
        kind = str(rng.choice(["belady", "lru", "resume"]))
        ids_d = _ids(ids)
        try:
            if kind == "resume":
                cap = int(rng.integers(1, n + 1))
                start = rng.permutation(n)[:cap].astype(np.int32)
                ref_cs = oracle.changeset_resume(n, ids, off, cap, start)
                cs = ginex.changeset_resume(n, ids_d, off, dev(start))
                check_resumed(cs, ref_cs, (n, ids, off))
                first = start
            else:
                cap = int(rng.integers(0, n + 1))
                ref_cs = (oracle.changeset if kind == "belady" else oracle.changeset_lru)(n, ids, off, cap)
                cs = ginex.changeset(n, ids_d, off, cap, **({"policy": "lru"} if kind == "lru" else {}))
                check_changeset(cs, ref_cs, (n, ids, off))
                first = ref_cs["init_ids"]
            cache = ginex.FeatureCache(slow, cap)
            cache.init(dev(first))
            ref = oracle.Cache(slow.numpy(), cap)
            ref.init(first)
            through_lines = bool(rng.random() < 0.6)
            co = cs.cs_offsets
            for i in range(S):
                sl, a, b = slice(co[i], co[i + 1]), off[i], off[i + 1]
                out = cache.gather(ids_d[a:b], None, cs.in_ids[sl], cs.out_ids[sl], cs.in_positions[sl],
                                   **({"src_line": cs.src_line[a:b]} if through_lines else {}))
                ref.gather_update(ids[a:b], ref_cs["in_ids"][sl], ref_cs["out_ids"][sl],
                                  ref_cs["in_positions"][sl])
                got = out.cpu().numpy().view(np.uint8).reshape(out.shape[0], row_words * 4)
                assert np.array_equal(got, sb[ids[a:b]]), i
            assert np.array_equal(cache.addr.cpu().numpy(), ref.addr)
            held = np.nonzero(ref.addr >= 0)[0]
            rows = cache.rows.cpu().numpy().view(np.uint8).reshape(cache.rows.shape[0], row_words * 4)
            assert np.array_equal(rows[ref.addr[held]], sb[held])
        except AssertionError:
            print("failing trial", trial, kind, n, S, row_words, flush=True)
            raise


def test_static_selection_and_neighbour_cache_on_random_graphs(ginex):
    """The highest-out-degree selection and the neighbour cache (build, then sampling through
    it with `indices` in HBM or in pinned host memory) on random R-MAT graphs of both offset
    widths, random capacities and budgets.  300 cases."""
    from test_gpu_parity import check_neighbor_cache
    from workload import rmat_csr
    rng = np.random.default_rng(777)
    for trial in range(300):
        n = int(rng.integers(1, 8000))
        e = int(rng.integers(0, 25 * n + 1))
        off, ind = rmat_csr(n, e, (0.5, 0.2, 0.2) if trial % 2 else (0.57, 0.19, 0.19),
                            int(rng.integers(1, 10**6)), "cpu", offsets_64=bool(trial & 2))
        e = int(off[-1])
        off_np, ind_np = off.numpy(), ind.numpy()
        ind_d = ind.cuda() if e else torch.zeros(1, dtype=torch.int32, device="cuda")[:0]
        try:
            cap = int(rng.integers(0, n + 3))
            assert np.array_equal(ginex.static_select(n, ind_d, cap).cpu().numpy(),
                                  oracle.static_select(n, ind_np, cap)), "static"
            budget = int(rng.integers(0, e + n + 2))
            nc = ginex.neighbor_cache_build(off.cuda(), ind_d, budget)
            check_neighbor_cache(nc, oracle.neighbor_cache_build(off_np, ind_np, budget))
            if e == 0:
                continue
            H = int(rng.integers(1, 4))
            fanout = tuple(int(rng.integers(1, 20)) for _ in range(H))
            S = int(rng.integers(1, 6))
            sizes = [int(rng.integers(0, min(n, 200) + 1)) for _ in range(S)]
            seeds = np.concatenate([rng.choice(n, size=s, replace=False) for s in sizes]).astype(np.int32)
            so = np.cumsum([0] + sizes)
            rs = int(rng.integers(0, 2**31))
            ref = oracle.sample_superbatch(off_np, ind_np, seeds, so, fanout, rng_seed=rs)
            where = ind.pin_memory() if trial % 3 == 0 else ind_d
            res = ginex.sample_superbatch(off.cuda(), where, _ids(seeds), so, fanout, rng_seed=rs,
                                          neighbor_cache=nc)
            check_sample(res, ref, S, H)
        except AssertionError:
            print("failing trial", trial, n, e, flush=True)
            raise
