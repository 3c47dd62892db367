"""Parity of the HIP path with the CPU oracle, element by element, through the C ABI.

Tolerance is zero: everything on this path is integer work or byte copies.
"""
import numpy as np
import pytest
import torch

import oracle
from workload import make_workload

pytestmark = pytest.mark.gpu


def dev(a, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


@pytest.fixture(scope="module")
def ginex():
    import paper_2208_09151_amd as g
    assert torch.cuda.is_available()
    print("library:", g.library_path(), "version", g.version(), flush=True)
    return g


class Case:
    """A workload plus the oracle's results for it."""

    def __init__(self, index, S=None):
        print(f"[case] building workload {index}", flush=True)
        w = make_workload(index, device="cuda", S=S)
        self.w, self.cfg = w, w.cfg
        self.off = w.offsets.cpu().numpy()
        self.ind = w.indices.cpu().numpy()
        self.seeds = w.seeds.numpy()
        self.seed_off = w.seed_offsets.numpy()
        print(f"[case] oracle sampling {index}", flush=True)
        self.samp = oracle.sample_superbatch(self.off, self.ind, self.seeds, self.seed_off,
                                             self.cfg.fanout, rng_seed=0)
        print(f"[case] oracle changeset {index}", flush=True)
        self.cs = oracle.changeset(self.cfg.num_nodes, self.samp["ids"],
                                   self.samp["ids_offsets"], self.cfg.cap)


@pytest.fixture(scope="module")
def case1():
    return Case(1)


@pytest.fixture(scope="module")
def case2():
    return Case(2)


def check_sample(res, ref, S, H):
    assert np.array_equal(res.ids_offsets, ref["ids_offsets"])
    assert np.array_equal(res.hop_sizes, ref["hop_sizes"])
    assert np.array_equal(res.ids.cpu().numpy(), ref["ids"])
    assert res.totals[0] == len(ref["ids"])
    assert res.totals[1] == len(ref["adj_rowptr"]) and res.totals[2] == len(ref["adj_col"])
    rp, col = res.adj_rowptr.cpu().numpy(), res.adj_col.cpu().numpy()
    for b in range(S):
        for h in range(H):
            g_ref, g = b * H + h, h * S + b
            a = ref["adj_rowptr"][ref["adj_row_offsets"][g_ref]:ref["adj_row_offsets"][g_ref + 1]]
            c = ref["adj_col"][ref["adj_col_offsets"][g_ref]:ref["adj_col_offsets"][g_ref + 1]]
            assert np.array_equal(rp[res.adj_row_offsets[g]:res.adj_row_offsets[g + 1]], a), (b, h)
            assert np.array_equal(col[res.adj_col_offsets[g]:res.adj_col_offsets[g + 1]], c), (b, h)


def run_sample(ginex, c, **kw):
    return ginex.sample_superbatch(c.w.offsets, c.w.indices, c.w.seeds.cuda(), c.seed_off,
                                   c.cfg.fanout, rng_seed=0, **kw)


@pytest.mark.parametrize("which", ["case1", "case2"])
def test_sampler_matches_oracle(ginex, which, request):
    c = request.getfixturevalue(which)
    res = run_sample(ginex, c)
    check_sample(res, c.samp, c.cfg.S, len(c.cfg.fanout))
    again = run_sample(ginex, c)          # atomics must not make the result order-dependent
    assert torch.equal(res.ids, again.ids) and torch.equal(res.adj_col, again.adj_col)
    no_adj = run_sample(ginex, c, with_adj=False)
    assert torch.equal(res.ids, no_adj.ids)
    assert np.array_equal(res.adj_col_offsets, no_adj.adj_col_offsets)


def check_changeset(res, ref, trace=None):
    """``trace`` = (num_nodes, ids, ids_offsets): also compares the resolved cache line of
    every access with the oracle's address-table replay of ITS lists."""
    if trace is not None:
        n, ids, off = trace
        want = oracle.resolve_lines(n, ids, off, ref["init_ids"], ref["in_ids"], ref["out_ids"],
                                    ref["cs_offsets"])
        assert res.src_line is not None and res.src_line.numel() == len(ids)
        assert np.array_equal(res.src_line.cpu().numpy(), want)
    assert np.array_equal(res.miss_count, ref["miss_count"])
    assert np.array_equal(res.cs_offsets, ref["cs_offsets"])
    assert np.array_equal(res.init_ids.cpu().numpy(), ref["init_ids"])
    assert np.array_equal(res.in_ids.cpu().numpy(), ref["in_ids"])
    assert np.array_equal(res.out_ids.cpu().numpy(), ref["out_ids"])
    assert np.array_equal(res.in_positions.cpu().numpy(), ref["in_positions"])


@pytest.mark.parametrize("which", ["case1", "case2"])
def test_changeset_matches_oracle(ginex, which, request):
    c = request.getfixturevalue(which)
    trace = (c.cfg.num_nodes, c.samp["ids"], c.samp["ids_offsets"])
    res = ginex.changeset(c.cfg.num_nodes, dev(c.samp["ids"]), c.samp["ids_offsets"], c.cfg.cap)
    check_changeset(res, c.cs, trace)
    # a small cache puts every iteration under pressure
    ref = oracle.changeset(c.cfg.num_nodes, c.samp["ids"], c.samp["ids_offsets"], 1000)
    check_changeset(ginex.changeset(c.cfg.num_nodes, dev(c.samp["ids"]),
                                    c.samp["ids_offsets"], 1000), ref, trace)
    # the lists do not depend on whether the lines are asked for
    bare = ginex.changeset(c.cfg.num_nodes, dev(c.samp["ids"]), c.samp["ids_offsets"], 1000,
                           with_lines=False)
    assert bare.src_line is None
    check_changeset(bare, ref)


@pytest.mark.parametrize("which", ["case1", "case2"])
def test_gather_and_cache_update_match_oracle(ginex, which, request):
    c = request.getfixturevalue(which)
    slow = c.w.features
    assert slow.is_pinned()
    sb = slow.numpy().view(np.uint8).reshape(slow.shape[0], -1)
    cache = ginex.FeatureCache(slow, c.cfg.cap)
    ids_d = dev(c.samp["ids"])
    cs = {k: dev(c.cs[k]) for k in ("init_ids", "in_ids", "out_ids", "in_positions")}
    cache.init(cs["init_ids"])
    ref = oracle.Cache(slow.numpy(), c.cfg.cap)
    ref.init(c.cs["init_ids"])
    assert np.array_equal(cache.addr.cpu().numpy(), ref.addr)
    io, co = c.samp["ids_offsets"], c.cs["cs_offsets"]
    for i in range(c.cfg.S):
        out = cache.gather(ids_d[io[i]:io[i + 1]], None, cs["in_ids"][co[i]:co[i + 1]],
                           cs["out_ids"][co[i]:co[i + 1]], cs["in_positions"][co[i]:co[i + 1]])
        got = out.cpu().numpy().view(np.uint8).reshape(out.shape[0], -1)
        assert np.array_equal(got, sb[c.samp["ids"][io[i]:io[i + 1]]]), i
        ref.gather_update(c.samp["ids"][io[i]:io[i + 1]], c.cs["in_ids"][co[i]:co[i + 1]],
                          c.cs["out_ids"][co[i]:co[i + 1]], c.cs["in_positions"][co[i]:co[i + 1]])
        if i % 5 == 0 or i == c.cfg.S - 1:
            assert np.array_equal(cache.addr.cpu().numpy(), ref.addr), i
    rows = cache.rows.cpu().numpy().view(np.uint8).reshape(cache.rows.shape[0], -1)
    res = np.nonzero(ref.addr >= 0)[0]
    assert np.array_equal(rows[ref.addr[res]], sb[res])
    assert np.array_equal(rows[:c.cfg.cap], ref.rows[:c.cfg.cap])


def test_whole_path_end_to_end(ginex, case1):
    """sample -> changeset -> init -> gather chained on device data only."""
    c = case1
    res = run_sample(ginex, c)
    cs = ginex.changeset(c.cfg.num_nodes, res.ids, res.ids_offsets, c.cfg.cap)
    check_changeset(cs, c.cs)
    cache = ginex.FeatureCache(c.w.features, c.cfg.cap)
    cache.init(cs.init_ids)
    sb = c.w.features.numpy().view(np.uint8).reshape(c.cfg.num_nodes, -1)
    io, co = res.ids_offsets, cs.cs_offsets
    for i in range(c.cfg.S):
        out = cache.gather(res.ids[io[i]:io[i + 1]], None, cs.in_ids[co[i]:co[i + 1]],
                           cs.out_ids[co[i]:co[i + 1]], cs.in_positions[co[i]:co[i + 1]])
        got = out.cpu().numpy().view(np.uint8).reshape(out.shape[0], -1)
        assert np.array_equal(got, sb[c.samp["ids"][io[i]:io[i + 1]]])


# ---- edge cases ------------------------------------------------------------------------

def small_graph(n=300, e=6000, seed=5, offsets_64=False):
    from workload import rmat_csr
    off, ind = rmat_csr(n, e, (0.5, 0.2, 0.2), seed, "cpu", offsets_64=offsets_64)
    return off, ind


@pytest.mark.parametrize("fanout", [(1,), (3, 2), (16, 16), (25, 10), (40, 2), (64,)])
@pytest.mark.parametrize("offsets_64", [False, True])
def test_sampler_fanouts_and_offset_widths(ginex, fanout, offsets_64):
    off, ind = small_graph(offsets_64=offsets_64)
    rng = np.random.default_rng(len(fanout) + fanout[0])
    batches = [rng.choice(300, size=s, replace=False) for s in (7, 0, 64, 1, 33)]
    seeds = np.concatenate(batches).astype(np.int32)
    so = np.cumsum([0] + [len(b) for b in batches])
    ref = oracle.sample_superbatch(off.numpy(), ind.numpy(), seeds, so, fanout, rng_seed=77,
                                   first_batch_index=9)
    res = ginex.sample_superbatch(off.cuda(), ind.cuda(), dev(seeds), so, fanout, rng_seed=77,
                                  first_batch_index=9)
    check_sample(res, ref, len(batches), len(fanout))


def test_sampler_repeated_seeds_and_partition_independence(ginex):
    off, ind = small_graph()
    seeds = np.array([5, 9, 5, 5, 100, 9, 17], dtype=np.int32)
    so = np.array([0, 7])
    ref = oracle.sample_superbatch(off.numpy(), ind.numpy(), seeds, so, (4, 4))
    res = ginex.sample_superbatch(off.cuda(), ind.cuda(), dev(seeds), so, (4, 4))
    check_sample(res, ref, 1, 2)
    assert res.hop_sizes[0][0] == 4
    # batch b sampled alone, under its global index, equals batch b inside a superbatch
    rng = np.random.default_rng(0)
    batches = [rng.choice(300, size=20, replace=False).astype(np.int32) for _ in range(6)]
    allb = ginex.sample_superbatch(off.cuda(), ind.cuda(), dev(np.concatenate(batches)),
                                   np.arange(7) * 20, (5, 5, 5), rng_seed=3, first_batch_index=100)
    for b in (0, 3, 5):
        one = ginex.sample_superbatch(off.cuda(), ind.cuda(), dev(batches[b]), [0, 20], (5, 5, 5),
                                      rng_seed=3, first_batch_index=100 + b)
        lo, hi = allb.ids_offsets[b], allb.ids_offsets[b + 1]
        assert torch.equal(one.ids, allb.ids[lo:hi])


def test_sampler_reports_required_capacity(ginex):
    off, ind = small_graph()
    seeds = dev(np.arange(50, dtype=np.int32))
    full = ginex.sample_superbatch(off.cuda(), ind.cuda(), seeds, [0, 50], (5, 5))
    tiny = (torch.empty(10, dtype=torch.int32, device="cuda"),
            torch.empty(10, dtype=torch.int64, device="cuda"),
            torch.empty(10, dtype=torch.int32, device="cuda"))
    with pytest.raises(ginex.GinexError) as e:
        ginex.sample_superbatch(off.cuda(), ind.cuda(), seeds, [0, 50], (5, 5), out=tiny)
    assert e.value.code == -2 and str(full.totals[0]) in str(e.value)


def random_trace(rng, n, S, max_len):
    tr = [rng.choice(n, size=rng.integers(0, min(max_len, n) + 1), replace=False)
          for _ in range(S)]
    off = np.cumsum([0] + [len(x) for x in tr]).astype(np.int64)
    ids = np.concatenate(tr).astype(np.int32) if off[-1] else np.zeros(0, dtype=np.int32)
    return ids, off


def test_changeset_random_small_traces(ginex):
    rng = np.random.default_rng(11)
    for trial in range(60):
        n = int(rng.integers(1, 400))
        S = int(rng.integers(1, 14))
        cap = int(rng.integers(0, n + 2))
        ids, off = random_trace(rng, n, S, int(rng.integers(1, 200)))
        ref = oracle.changeset(n, ids, off, cap)
        ids_d = dev(ids) if len(ids) else torch.zeros(1, dtype=torch.int32, device="cuda")[:0]
        res = ginex.changeset(n, ids_d, off, cap)
        try:
            check_changeset(res, ref, (n, ids, off))
        except AssertionError:
            print("failing trial", trial, n, S, cap, flush=True)
            raise


def test_changeset_degenerate_capacities(ginex, case1):
    c = case1
    ids, io = c.samp["ids"], c.samp["ids_offsets"]
    distinct = len(np.unique(ids))
    for cap in (0, 1, 7, distinct - 1, distinct, distinct + 5):
        ref = oracle.changeset(c.cfg.num_nodes, ids, io, cap)
        res = ginex.changeset(c.cfg.num_nodes, dev(ids), io, cap)
        check_changeset(res, ref, (c.cfg.num_nodes, ids, io))
    # one iteration only, and a trace whose ties all fall into one bucket
    one = oracle.changeset(c.cfg.num_nodes, ids[:io[1]], io[:2], 100)
    check_changeset(ginex.changeset(c.cfg.num_nodes, dev(ids[:io[1]]), io[:2], 100), one)


@pytest.mark.parametrize("row_bytes", [16, 48, 256, 1024, 3072])
def test_gather_row_sizes_and_empty_changesets(ginex, row_bytes):
    rng = np.random.default_rng(row_bytes)
    n, cap = 500, 60
    slow = torch.from_numpy(rng.integers(0, 255, size=(n, row_bytes), dtype=np.uint8)).pin_memory()
    ids, off = random_trace(rng, n, 6, 200)
    ref_cs = oracle.changeset(n, ids, off, cap)
    cache = ginex.FeatureCache(slow, cap)
    cache.init(dev(ref_cs["init_ids"]))
    ref = oracle.Cache(slow.numpy(), cap)
    ref.init(ref_cs["init_ids"])
    co = ref_cs["cs_offsets"]
    for i in range(6):
        cur = ids[off[i]:off[i + 1]]
        sl = slice(co[i], co[i + 1])
        out = cache.gather(dev(cur) if len(cur) else torch.zeros(0, dtype=torch.int32, device="cuda"),
                           None, dev(ref_cs["in_ids"][sl]) if co[i + 1] > co[i] else None,
                           dev(ref_cs["out_ids"][sl]) if co[i + 1] > co[i] else None,
                           dev(ref_cs["in_positions"][sl]) if co[i + 1] > co[i] else None)
        want, _ = ref.gather_update(cur, ref_cs["in_ids"][sl], ref_cs["out_ids"][sl],
                                    ref_cs["in_positions"][sl])
        assert np.array_equal(out.cpu().numpy(), want)
        assert np.array_equal(out.cpu().numpy(), slow.numpy()[cur])
    assert np.array_equal(cache.addr.cpu().numpy(), ref.addr)
    assert np.array_equal(cache.rows.cpu().numpy()[:cap], ref.rows[:cap])


def test_separate_update_equals_fused_gather_update(ginex, case1):
    c = case1
    cs = {k: dev(c.cs[k]) for k in ("init_ids", "in_ids", "out_ids", "in_positions")}
    a, b = ginex.FeatureCache(c.w.features, c.cfg.cap), ginex.FeatureCache(c.w.features, c.cfg.cap)
    a.init(cs["init_ids"])
    b.init(cs["init_ids"])
    ids_d, io, co = dev(c.samp["ids"]), c.samp["ids_offsets"], c.cs["cs_offsets"]
    for i in range(c.cfg.S):
        sl = slice(co[i], co[i + 1])
        oa = a.gather(ids_d[io[i]:io[i + 1]], None, cs["in_ids"][sl], cs["out_ids"][sl],
                      cs["in_positions"][sl])
        ob = b.gather(ids_d[io[i]:io[i + 1]])
        b.update(ob, cs["in_ids"][sl], cs["out_ids"][sl], cs["in_positions"][sl])
        assert torch.equal(oa, ob)
    assert torch.equal(a.addr, b.addr) and torch.equal(a.rows, b.rows)


def test_gather_reads_a_device_resident_slow_tier_too(ginex):
    rng = np.random.default_rng(2)
    slow = torch.from_numpy(rng.standard_normal((1000, 32)).astype(np.float32)).cuda()
    cache = ginex.FeatureCache(slow, 10)
    cache.init(dev(np.arange(10, dtype=np.int32)))
    ids = rng.permutation(1000)[:300].astype(np.int32)
    out = cache.gather(dev(ids))
    assert torch.equal(out, slow[torch.from_numpy(ids).long().cuda()])


def test_pipelined_inspector_equals_sequential(ginex, case2):
    """Superbatch-level pipeline: changeset(k) under sample(k+1), on two streams and two
    host threads, must give exactly what the oracle gives for every superbatch."""
    from workload.configs import seed_batches, train_nodes
    c = case2
    cfg, S = c.cfg, 6
    train = train_nodes(cfg.num_nodes, cfg.train_frac, cfg.seed)
    sbs, refs = [], []
    for k in range(4):
        seeds, so = seed_batches(train, cfg.batch, S, cfg.seed, first_batch=k * S)
        sbs.append((seeds.cuda(), so.numpy(), k * S))
        r = oracle.sample_superbatch(c.off, c.ind, seeds.numpy(), so.numpy(), cfg.fanout,
                                     rng_seed=0, first_batch_index=k * S)
        refs.append((r, oracle.changeset(cfg.num_nodes, r["ids"], r["ids_offsets"], 20000)))
    pipe = ginex.InspectorPipeline(c.w.offsets, c.w.indices, cfg.num_nodes, cfg.fanout, 20000,
                                   cfg.batch, S)
    for mode in ("overlap", "sequential"):
        seen = []

        def consume(k, samp, cs):
            assert np.array_equal(samp.ids.cpu().numpy(), refs[k][0]["ids"]), (mode, k)
            check_changeset(cs, refs[k][1])
            seen.append(k)

        pipe.run(sbs, rng_seed=0, mode=mode, consume=consume)
        assert seen == [0, 1, 2, 3]


def test_validation_mode_rejects_bad_traces(ginex, monkeypatch):
    monkeypatch.setenv("GINEX_VALIDATE", "1")
    good = np.array([3, 4, 2, 0, 3, 1], dtype=np.int32)
    off = np.array([0, 2, 4, 6])
    check_changeset(ginex.changeset(5, dev(good), off, 2), oracle.changeset(5, good, off, 2))
    off_g, ind_g = small_graph()
    with pytest.raises(ginex.GinexError) as e:
        ginex.sample_superbatch(off_g.cuda(), ind_g.cuda(), dev(np.array([1, 300], dtype=np.int32)),
                                [0, 2], (3,))
    assert e.value.code == -4 and "seeds outside" in str(e.value)
    # a broken CSR: an index out of range, offsets that decrease, offsets that do not end at E
    good_seeds = dev(np.array([1, 2], dtype=np.int32))
    ginex.sample_superbatch(off_g.cuda(), ind_g.cuda(), good_seeds, [0, 2], (3,))
    for breakage in ("index", "decrease", "end"):
        o, i = off_g.clone(), ind_g.clone()
        if breakage == "index":
            i[5] = 300
        elif breakage == "decrease":
            o[10] = o[11] + 1
        else:
            o[-1] += 1
        with pytest.raises(ginex.GinexError) as e:
            ginex.sample_superbatch(o.cuda(), i.cuda(), good_seeds, [0, 2], (3,))
        assert e.value.code == -4 and "CSR" in str(e.value), breakage
    for bad in ([3, 3, 2, 0, 3, 1], [3, 4, 2, 0, 9, 1]):     # a repeat / an id >= num_nodes
        with pytest.raises(ginex.GinexError) as e:
            ginex.changeset(5, dev(np.array(bad, dtype=np.int32)), off, 2)
        assert e.value.code == -4


@pytest.mark.parametrize("fanout,batch,S", [((10, 10, 10), 8, 1500), ((15, 10, 5), 64, 300),
                                            ((25, 10), 128, 100)])
def test_many_small_batches_whole_path(ginex, case1, fanout, batch, S):
    """Superbatches of the size the paper uses (thousands of batches), other popular
    sampling sizes, with the cache under pressure in every iteration."""
    from workload.configs import seed_batches, train_nodes
    c = case1
    cfg = c.cfg
    train = train_nodes(cfg.num_nodes, cfg.train_frac, cfg.seed)
    seeds, so = seed_batches(train, batch, S, cfg.seed)
    ref = oracle.sample_superbatch(c.off, c.ind, seeds.numpy(), so.numpy(), fanout, rng_seed=5)
    res = ginex.sample_superbatch(c.w.offsets, c.w.indices, seeds.cuda(), so.numpy(), fanout,
                                  rng_seed=5)
    check_sample(res, ref, S, len(fanout))
    for cap in (300, 3000):
        rcs = oracle.changeset(cfg.num_nodes, ref["ids"], ref["ids_offsets"], cap)
        cs = ginex.changeset(cfg.num_nodes, res.ids, res.ids_offsets, cap)
        check_changeset(cs, rcs)


def test_executor_under_next_inspector_gathers_the_right_bytes(ginex, case2):
    """Executor of superbatch k while superbatch k+1 is inspected on other streams: every
    gathered batch input must still be slow[ids]."""
    from workload.configs import seed_batches, train_nodes
    c = case2
    cfg, S, cap = c.cfg, 5, 15000
    train = train_nodes(cfg.num_nodes, cfg.train_frac, cfg.seed)
    sbs, refs = [], []
    for k in range(3):
        seeds, so = seed_batches(train, cfg.batch, S, cfg.seed, first_batch=k * S)
        sbs.append((seeds.cuda(), so.numpy(), k * S))
        refs.append(oracle.sample_superbatch(c.off, c.ind, seeds.numpy(), so.numpy(), cfg.fanout,
                                             rng_seed=0, first_batch_index=k * S))
    pipe = ginex.InspectorPipeline(c.w.offsets, c.w.indices, cfg.num_nodes, cfg.fanout, cap,
                                   cfg.batch, S)
    cache = ginex.FeatureCache(c.w.features, cap)
    feats = c.w.features.numpy()
    done = []

    def execute(k, samp, cs):
        assert np.array_equal(samp.ids.cpu().numpy(), refs[k]["ids"])
        check_changeset(cs, oracle.changeset(cfg.num_nodes, refs[k]["ids"],
                                             refs[k]["ids_offsets"], cap))
        cache.init(cs.init_ids)
        io, co = samp.ids_offsets, cs.cs_offsets
        for i in range(S):
            sl = slice(co[i], co[i + 1])
            out = cache.gather(samp.ids[io[i]:io[i + 1]], None, cs.in_ids[sl], cs.out_ids[sl],
                               cs.in_positions[sl])
            want = oracle.gather(feats, refs[k]["ids"][io[i]:io[i + 1]])
            got = out.cpu().numpy().view(np.uint8).reshape(out.shape[0], -1)
            assert np.array_equal(got, want), (k, i)
        done.append(k)

    for overlap in (True, False):
        del done[:]
        pipe.run_with_executor(sbs, execute, overlap=overlap)
        assert done == [0, 1, 2]
    # three stages in flight (sampling of k+2, changesets of k+1, executor of k), five
    # superbatches so that every buffer set is reused
    for k in range(3, 5):
        seeds, so = seed_batches(train, cfg.batch, S, cfg.seed, first_batch=k * S)
        sbs.append((seeds.cuda(), so.numpy(), k * S))
        refs.append(oracle.sample_superbatch(c.off, c.ind, seeds.numpy(), so.numpy(), cfg.fanout,
                                             rng_seed=0, first_batch_index=k * S))
    del done[:]
    pipe.run_three_stage(sbs, execute)
    assert done == [0, 1, 2, 3, 4]

    # an error in a stage reaches the caller and leaves no thread behind
    def failing(k, samp, cs):
        raise RuntimeError("executor failed")
    with pytest.raises(RuntimeError, match="executor failed"):
        pipe.run_three_stage(sbs, failing)
    del done[:]
    pipe.run_three_stage(sbs[:2], execute)
    assert done == [0, 1]


# ---- LRU changesets through the same kernels (Section 2.3) -------------------------------

def test_lru_changeset_random_small_traces(ginex):
    rng = np.random.default_rng(31)
    for trial in range(60):
        n = int(rng.integers(1, 400))
        S = int(rng.integers(1, 14))
        cap = int(rng.integers(0, n + 2))
        ids, off = random_trace(rng, n, S, int(rng.integers(1, 200)))
        ref = oracle.changeset_lru(n, ids, off, cap)
        ids_d = dev(ids) if len(ids) else torch.zeros(1, dtype=torch.int32, device="cuda")[:0]
        res = ginex.changeset(n, ids_d, off, cap, policy="lru")
        try:
            check_changeset(res, ref, (n, ids, off))
        except AssertionError:
            print("failing trial", trial, n, S, cap, flush=True)
            raise


@pytest.mark.parametrize("which", ["case1", "case2"])
def test_lru_changeset_matches_oracle_and_feeds_the_executor(ginex, which, request):
    c = request.getfixturevalue(which)
    ids, io = c.samp["ids"], c.samp["ids_offsets"]
    n, S = c.cfg.num_nodes, c.cfg.S
    distinct = len(np.unique(ids))
    longest = int(np.diff(io).max())
    ids_d = dev(ids)
    sb = c.w.features.numpy().view(np.uint8).reshape(n, -1)
    for cap in (1, 1000, c.cfg.cap, longest + 1, distinct // 2, distinct - 1, distinct):
        ref = oracle.changeset_lru(n, ids, io, cap)
        res = ginex.changeset(n, ids_d, io, cap, policy="lru")
        check_changeset(res, ref, (n, ids, io))
        bel = ginex.changeset(n, ids_d, io, cap)
        assert bel.miss_count.sum() <= res.miss_count.sum()
    # the executor runs an LRU changeset like any other
    cap = max(1000, distinct // 8)
    res = ginex.changeset(n, ids_d, io, cap, policy="lru")
    cache = ginex.FeatureCache(c.w.features, cap)
    cache.init(res.init_ids)
    co = res.cs_offsets
    for i in range(S):
        sl = slice(co[i], co[i + 1])
        out = cache.gather(ids_d[io[i]:io[i + 1]], None, res.in_ids[sl], res.out_ids[sl],
                           res.in_positions[sl],
                           src_line=res.src_line[io[i]:io[i + 1]] if i % 2 else None)
        if i % 7 == 0 or i == S - 1:
            got = out.cpu().numpy().view(np.uint8).reshape(out.shape[0], -1)
            assert np.array_equal(got, sb[ids[io[i]:io[i + 1]]]), i
    addr = cache.addr.cpu().numpy()
    resident = np.nonzero(addr >= 0)[0]
    rows = cache.rows.cpu().numpy().view(np.uint8).reshape(cache.rows.shape[0], -1)
    assert np.array_equal(rows[addr[resident]], sb[resident])


# ---- neighbour cache (Section 3.2) ----------------------------------------------------------

def check_neighbor_cache(nc, ref):
    at, ca, cached = ref
    assert nc.cached_nodes == cached and nc.used_entries == len(ca)
    assert np.array_equal(nc.address_table.cpu().numpy(), at)
    assert np.array_equal(nc.cache_array[:nc.used_entries].cpu().numpy(), ca)


@pytest.mark.parametrize("offsets_64", [False, True])
def test_neighbor_cache_build_matches_oracle_on_small_graphs(ginex, offsets_64):
    rng = np.random.default_rng(41 + offsets_64)
    for trial in range(12):
        n = int(rng.integers(1, 3000))
        e = int(rng.integers(0, 30000))
        off, ind = small_graph(n, e, seed=trial, offsets_64=offsets_64)
        e = int(off[-1])
        for budget in (0, 1, int(rng.integers(0, e + n + 1)), e + n):
            ref = oracle.neighbor_cache_build(off.numpy(), ind.numpy(), budget)
            ind_d = ind.cuda() if e else torch.zeros(1, dtype=torch.int32, device="cuda")[:0]
            nc = ginex.neighbor_cache_build(off.cuda(), ind_d, budget)
            try:
                check_neighbor_cache(nc, ref)
            except AssertionError:
                print("failing case", trial, n, e, budget, flush=True)
                raise


def test_neighbor_cache_build_rejects_indices_out_of_range(ginex):
    off, ind = small_graph(500, 4000, seed=3)
    bad = ind.clone()
    bad[17] = 500
    with pytest.raises(ginex.GinexError, match="outside"):
        ginex.neighbor_cache_build(off.cuda(), bad.cuda(), 1000)
    bad[17] = -3
    with pytest.raises(ginex.GinexError, match="outside"):
        ginex.neighbor_cache_build(off.cuda(), bad.cuda(), 1000)
    ginex.neighbor_cache_build(off.cuda(), ind.cuda(), 1000)


@pytest.mark.parametrize("which", ["case1", "case2"])
def test_neighbor_cache_is_transparent_to_the_sampler(ginex, which, request):
    c = request.getfixturevalue(which)
    E = len(c.ind)
    S, H = c.cfg.S, len(c.cfg.fanout)
    # the graph as the neighbour cache is meant to see it: indices in pinned host memory
    ind_host = torch.from_numpy(c.ind).pin_memory()
    for budget in (E // 50, E // 4, E + c.cfg.num_nodes):
        ref = oracle.neighbor_cache_build(c.off, c.ind, budget)
        nc = ginex.neighbor_cache_build(c.w.offsets, ind_host, budget)
        check_neighbor_cache(nc, ref)
        for indices in (c.w.indices, ind_host):
            res = ginex.sample_superbatch(c.w.offsets, indices, c.w.seeds.cuda(),
                                          c.seed_off, c.cfg.fanout, rng_seed=0, neighbor_cache=nc)
            check_sample(res, c.samp, S, H)
    # without a cache the sampler reads a host-resident CSR just as well
    res = ginex.sample_superbatch(c.w.offsets, ind_host, c.w.seeds.cuda(), c.seed_off,
                                  c.cfg.fanout, rng_seed=0)
    check_sample(res, c.samp, S, H)


# ---- main loop started under the cache initialization ------------------------------------------

@pytest.mark.parametrize("which", ["case1", "case2"])
def test_streamed_initialization_gathers_the_same_bytes(ginex, which, request):
    c = request.getfixturevalue(which)
    n, S = c.cfg.num_nodes, c.cfg.S
    ids, io = c.samp["ids"], c.samp["ids_offsets"]
    distinct = len(np.unique(ids))
    _, first = oracle.next_use(n, ids, io)
    sb = c.w.features.numpy().view(np.uint8).reshape(n, -1)
    res = run_sample(ginex, c)
    longest = int(np.diff(io).max())
    out = torch.empty((longest, c.cfg.feat_dim), dtype=torch.float32, device="cuda")
    for cap in (distinct, distinct - 1, c.cfg.cap, 1000, 0):
        ref = oracle.changeset(n, ids, io, cap)
        cs = ginex.changeset(n, res.ids, res.ids_offsets, cap)
        check_changeset(cs, ref)
        # init_ready[i] = rows of C_0 first accessed in iterations 0..i
        f = first[ref["init_ids"]]
        want_ready = np.array([(f <= i).sum() for i in range(S)], dtype=np.int64)
        assert np.array_equal(cs.init_ready, want_ready)
        assert np.all(np.diff(f) >= 0)                     # C_0 is ordered by first access
        cache = ginex.FeatureCache(c.w.features, cap)
        replay = oracle.Cache(c.w.features.numpy(), cap)
        replay.init(ref["init_ids"])
        co = ref["cs_offsets"]
        for i in range(S):
            replay.gather_update(ids[io[i]:io[i + 1]], ref["in_ids"][co[i]:co[i + 1]],
                                 ref["out_ids"][co[i]:co[i + 1]],
                                 ref["in_positions"][co[i]:co[i + 1]])
        for streamed, piece in ((True, 1), (True, 4096), (False, 1)):
            ex = ginex.Executor(cache, min_piece_rows=piece)
            cache.rows.fill_(float("nan"))                 # stale lines must never be read
            got = {}

            def keep(i, rows):
                got[i] = out[:rows].clone()
            ex.run(res, cs, out, streamed=streamed, after_gather=keep)
            torch.cuda.synchronize()
            for i in range(S):
                g = got[i].cpu().numpy().view(np.uint8).reshape(got[i].shape[0], -1)
                assert np.array_equal(g, sb[ids[io[i]:io[i + 1]]]), (cap, streamed, piece, i)
            assert np.array_equal(cache.addr.cpu().numpy(), replay.addr), (cap, streamed, piece)
            if cap:
                rows = cache.rows.cpu().numpy().view(np.uint8).reshape(cache.rows.shape[0], -1)
                held = np.nonzero(replay.addr >= 0)[0]
                assert np.array_equal(rows[replay.addr[held]], sb[held])


def test_warm_initialization_leaves_the_same_cache_as_a_cold_one(ginex, case2):
    """Consecutive superbatches with two caches taking turns: rows the previous cache holds
    are copied from it, the cache content must not differ from a cold initialization."""
    from workload.configs import seed_batches, train_nodes
    c = case2
    cfg, n = c.cfg, c.cfg.num_nodes
    S = 6
    train = train_nodes(n, cfg.train_frac, cfg.seed)
    feats = c.w.features
    sb = feats.numpy().view(np.uint8).reshape(n, -1)
    for cap in (cfg.cap, 20000):
        warm = ginex.Executor(ginex.FeatureCache(feats, cap), min_piece_rows=2048,
                              second=ginex.FeatureCache(feats, cap))
        cold = ginex.Executor(ginex.FeatureCache(feats, cap))
        out = None
        reused = 0
        for k in range(4):
            seeds, so = seed_batches(train, cfg.batch, S, cfg.seed, first_batch=k * S)
            samp = ginex.sample_superbatch(c.w.offsets, c.w.indices, seeds.cuda(), so.numpy(),
                                           cfg.fanout, rng_seed=0, first_batch_index=k * S)
            cs = ginex.changeset(n, samp.ids, samp.ids_offsets, cap)
            io = samp.ids_offsets
            longest = int(np.diff(io).max())
            if out is None or out.shape[0] < longest:
                out = torch.empty((longest, cfg.feat_dim), dtype=torch.float32, device="cuda")
            if k > 0:
                held = warm.cache.addr[cs.init_ids.long()] >= 0
                reused += int(held.sum())
            ids_h = samp.ids.cpu().numpy()
            for ex, streamed in ((warm, k % 2 == 0), (cold, False)):
                got = {}

                def keep(i, rows):
                    got[i] = out[:rows].clone()
                ex.run(samp, cs, out, streamed=streamed, after_gather=keep)
                torch.cuda.synchronize()
                for i in range(S):
                    g = got[i].cpu().numpy().view(np.uint8).reshape(got[i].shape[0], -1)
                    assert np.array_equal(g, sb[ids_h[io[i]:io[i + 1]]]), (cap, k, i)
            a_w, a_c = warm.cache.addr.cpu().numpy(), cold.cache.addr.cpu().numpy()
            assert np.array_equal(a_w, a_c), (cap, k)
            held = np.nonzero(a_c >= 0)[0]
            lines = torch.from_numpy(a_c[held]).long().cuda()
            assert torch.equal(warm.cache.rows[lines], cold.cache.rows[lines]), (cap, k)
        assert reused > 0      # the superbatches do share rows, so the warm path was taken


# ---- cache carried from superbatch to superbatch ---------------------------------------------

def check_resumed(res, ref, trace=None):
    check_changeset(res, ref, trace)
    assert np.array_equal(res.final_ids.cpu().numpy(), ref["final_ids"])


def test_resumed_changeset_random_small_traces(ginex):
    rng = np.random.default_rng(51)
    for trial in range(60):
        n = int(rng.integers(2, 400))
        S = int(rng.integers(1, 14))
        cap = int(rng.integers(1, n + 1))
        ids, off = random_trace(rng, n, S, int(rng.integers(1, 200)))
        start = rng.permutation(n)[:cap].astype(np.int32)
        ref = oracle.changeset_resume(n, ids, off, cap, start)
        ids_d = dev(ids) if len(ids) else torch.zeros(1, dtype=torch.int32, device="cuda")[:0]
        res = ginex.changeset_resume(n, ids_d, off, dev(start))
        try:
            check_resumed(res, ref, (n, ids, off))
        except AssertionError:
            print("failing trial", trial, n, S, cap, flush=True)
            raise
    # a start state with a repeated or an out-of-range row is refused before the loop runs
    ids, off = random_trace(rng, 50, 4, 20)
    for bad in ([1, 2, 2, 3], [1, 2, 50, 3], [1, -1, 4, 3]):
        with pytest.raises(ginex.GinexError):
            ginex.changeset_resume(50, dev(ids), off, dev(np.array(bad, dtype=np.int32)))


def planned_cases(rng):
    """Traces over a carried cache that holds every distinct row of the trace (the regime in
    which the changesets follow without a loop over the state), shaped to reach every branch
    of that path and every reason to leave it."""
    def revisit(n, S, rows, per_row):          # each of `rows` accessed in per_row iterations
        tr = [[] for _ in range(S)]
        for v in rows:
            for i in rng.choice(S, size=min(per_row, S), replace=False):
                tr[i].append(v)
        tr = [rng.permutation(np.array(t, dtype=np.int32)) for t in tr]
        off = np.cumsum([0] + [len(t) for t in tr]).astype(np.int64)
        return np.concatenate(tr).astype(np.int32), off
    # 1. small id spaces: the replayed id range is the whole space, most insertions may be
    #    evicted again in the same call
    for _ in range(25):
        n = int(rng.integers(20, 600))
        S = int(rng.integers(2, 40))
        ids, off = random_trace(rng, n, S, int(rng.integers(1, 80)))
        distinct = len(np.unique(ids))
        cap = int(rng.integers(max(distinct, 1), n + 1))
        yield "small", n, ids, off, rng.permutation(n)[:cap].astype(np.int32)
    # 2. a larger id space, few start rows are ever accessed, rows come and go
    for _ in range(6):
        n = int(rng.integers(3000, 40000))
        S = int(rng.integers(5, 60))
        rows = rng.choice(n, size=int(rng.integers(50, 1500)), replace=False)
        ids, off = revisit(n, S, rows, int(rng.integers(1, 5)))
        cap = int(rng.integers(len(np.unique(ids)) + 1, n))
        yield "larger", n, ids, off, rng.permutation(n)[:cap].astype(np.int32)
    # 3. thousands of inserted rows that leave again in the same call: their lines are handed
    #    from the pairing thread to the evicting thread iterations later
    n = 8000
    ids, off = revisit(n, 12, np.arange(6000, 8000), 2)
    yield "reinserted", n, ids, off, np.arange(6000, dtype=np.int32)
    # 4. one iteration with more than 4096 insertions: not taken at all; with 3000: taken
    n = 12000
    for kind, count in (("wide", 5000), ("broad", 3000)):
        rows = np.arange(6000, 6000 + count)
        tr = [rows, rows[::-1].copy(), rng.permutation(n)[:100]]
        off = np.cumsum([0] + [len(t) for t in tr]).astype(np.int64)
        yield kind, n, np.concatenate(tr).astype(np.int32), off, np.arange(6000, dtype=np.int32)
    # 4b. thousands of evictions in one iteration whose lines all lie at the upper end of a
    #     large cache (the ranking by line then finds them in a few of its buckets)
    n = 1000000
    rows = np.arange(700000, 703000)
    tr = [rng.permutation(rows), rows[::-1].copy(), rng.permutation(rows)[:1200]]
    off = np.cumsum([0] + [len(t) for t in tr]).astype(np.int64)
    yield "clustered", n, np.concatenate(tr).astype(np.int32), off, np.arange(700000, dtype=np.int32)
    # 4c. tens of thousands of candidates (several bitmap words per thread of the replay): most
    #     rows of the upper half of the start state are accessed once and die on the way, one
    #     in twenty is dead from the start, and two waves of new rows push rows out
    n = 300000
    upper = np.arange(100000, 200000)
    once = upper[upper % 20 != 7]
    tr = [[] for _ in range(6)]
    for i, part in enumerate(np.array_split(rng.permutation(once), 6)):
        tr[i] = list(part)
    first, second = np.arange(200000, 203000), np.arange(203000, 204500)
    tr[0] += list(first); tr[3] += list(first[::-1])
    tr[4] += list(second); tr[5] += list(second)
    tr = [rng.permutation(np.array(t, dtype=np.int32)) for t in tr]
    off = np.cumsum([0] + [len(t) for t in tr]).astype(np.int64)
    yield "many_candidates", n, np.concatenate(tr).astype(np.int32), off, \
        rng.permutation(200000).astype(np.int32)
    # 5. the rows that are dead from the start are spread thinly over a large id space: the
    #    candidates are few although the id range from the lowest possible victim up is wide
    n = 900000
    start = (np.arange(300, dtype=np.int32) * 3000 + 7).astype(np.int32)
    rows = np.setdiff1d(rng.choice(n, size=260, replace=False), start)[:200]
    ids, off = revisit(n, 10, rows, 2)
    yield "sparse", n, ids, off, start
    # 5b. more candidates than the replay's bitmap holds (600 000 resident rows die above the
    #     lowest possible victim): not taken
    n = 710000
    start = np.concatenate([np.arange(1000), np.arange(100000, 700000)]).astype(np.int32)
    tr = [rng.permutation(np.arange(100000 + 120000 * i, 220000 + 120000 * i)) for i in range(5)]
    newcomers = np.arange(700000, 700500)
    tr[0] = np.concatenate([tr[0], newcomers])
    tr[3] = np.concatenate([tr[3], newcomers[::-1]])
    off = np.cumsum([0] + [len(t) for t in tr]).astype(np.int64)
    yield "crowded", n, np.concatenate(tr).astype(np.int32), off, start
    # 6. nothing is ever inserted (single accesses only), and an empty trace
    n = 500
    ids, off = revisit(n, 8, rng.choice(n, size=100, replace=False), 1)
    yield "bypass", n, ids, off, rng.permutation(n)[:300].astype(np.int32)
    yield "empty", n, np.zeros(0, dtype=np.int32), np.zeros(5, dtype=np.int64), \
        rng.permutation(n)[:300].astype(np.int32)


def test_carried_cache_that_holds_the_superbatch_needs_no_loop(ginex, monkeypatch, capfd):
    """A carried cache with a line for every distinct row of the superbatch: hits, misses and
    insertions are known up front and only the choice of the evicted rows is replayed, by one
    workgroup in LDS or, for more candidates or evictions than that holds (or GINEX_PLANNED=2),
    step by step on the bitmap in global memory.  The results equal the oracle's and the
    loop's (GINEX_PLANNED=0), lists, lines and final state."""
    rng = np.random.default_rng(77)
    for kind, n, ids, off, start in planned_cases(rng):
        cap = len(start)
        assert len(np.unique(ids)) <= cap
        ref = oracle.changeset_resume(n, ids, off, cap, start)
        ids_d = dev(ids) if len(ids) else torch.zeros(1, dtype=torch.int32, device="cuda")[:0]
        print("planned case", kind, n, len(ids), cap, flush=True)
        monkeypatch.delenv("GINEX_PLANNED", raising=False)
        monkeypatch.setenv("GINEX_TRACE", "1")
        capfd.readouterr()
        res = ginex.changeset_resume(n, ids_d, off, dev(start))
        said = capfd.readouterr().err
        monkeypatch.delenv("GINEX_TRACE")
        check_resumed(res, ref, (n, ids, off))
        if len(ids):      # the way the call went is the one the case was built for
            big = kind in ("wide", "crowded")   # more than the replay's arrays in LDS hold
            assert ("stepped path" in said) == big and ("planned path" in said) == (not big), said
            assert "gave up" not in said and ": loop" not in said, said
        # the same through the steps on the bitmap in global memory, whatever the sizes ...
        monkeypatch.setenv("GINEX_PLANNED", "2")
        monkeypatch.setenv("GINEX_TRACE", "1")
        capfd.readouterr()
        stepped = ginex.changeset_resume(n, ids_d, off, dev(start))
        said = capfd.readouterr().err
        monkeypatch.delenv("GINEX_TRACE")
        check_resumed(stepped, ref, (n, ids, off))
        if len(ids) and int(ref["cs_offsets"][-1]):
            assert "stepped path" in said and "gave up" not in said, said
        # ... and through the loop
        monkeypatch.setenv("GINEX_PLANNED", "0")
        loop = ginex.changeset_resume(n, ids_d, off, dev(start))
        check_resumed(loop, ref, (n, ids, off))
    monkeypatch.delenv("GINEX_PLANNED", raising=False)


def test_one_workspace_serves_every_kind_of_call_in_any_order(ginex, case1):
    """Sampling, changesets with and without pressure, LRU, resumed changesets through the loop
    and without it, all on ONE workspace filled with junk in between: no call relies on what an
    earlier one left there."""
    c = case1
    n, S = c.cfg.num_nodes, c.cfg.S
    ids, io = c.samp["ids"], c.samp["ids_offsets"]
    ids_d = dev(ids)
    distinct = len(np.unique(ids))
    ws = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(3)
    start_small = rng.permutation(n)[:max(1, distinct // 8)].astype(np.int32)
    rows = np.unique(ids)
    others = np.setdiff1d(np.arange(n), rows)
    keep = rows[rng.random(len(rows)) < 0.9]
    start_big = rng.permutation(np.concatenate([keep, others[:len(rows) - len(keep) + 200]])).astype(np.int32)
    calls = [
        ("belady", lambda: ginex.changeset(n, ids_d, io, distinct // 8, workspace=ws),
         lambda: oracle.changeset(n, ids, io, distinct // 8)),
        ("resume, no loop", lambda: ginex.changeset_resume(n, ids_d, io, dev(start_big), workspace=ws),
         lambda: oracle.changeset_resume(n, ids, io, len(start_big), start_big)),
        ("lru", lambda: ginex.changeset(n, ids_d, io, distinct // 8, workspace=ws, policy="lru"),
         lambda: oracle.changeset_lru(n, ids, io, distinct // 8)),
        ("resume, loop", lambda: ginex.changeset_resume(n, ids_d, io, dev(start_small), workspace=ws),
         lambda: oracle.changeset_resume(n, ids, io, len(start_small), start_small)),
        ("all fit", lambda: ginex.changeset(n, ids_d, io, distinct + 5, workspace=ws),
         lambda: oracle.changeset(n, ids, io, distinct + 5)),
    ]
    refs = [ref() for _, _, ref in calls]
    for order in (range(len(calls)), reversed(range(len(calls))), (1, 1, 3, 1, 0, 1)):
        for k in order:
            ws.random_(0, 256)                     # junk, different every time
            name, run, _ = calls[k]
            res = run()
            check_changeset(res, refs[k], (n, ids, io))
            if "resume" in name:
                assert np.array_equal(res.final_ids.cpu().numpy(), refs[k]["final_ids"]), name
        ws.random_(0, 256)
        samp = ginex.sample_superbatch(c.w.offsets, c.w.indices, c.w.seeds.cuda(), c.seed_off,
                                       c.cfg.fanout, rng_seed=0, workspace=ws)
        check_sample(samp, c.samp, S, len(c.cfg.fanout))


def test_carried_cache_over_consecutive_superbatches(ginex, case2):
    from workload.configs import seed_batches, train_nodes
    c = case2
    cfg, n = c.cfg, c.cfg.num_nodes
    S = 6
    train = train_nodes(n, cfg.train_frac, cfg.seed)
    feats = c.w.features
    sb = feats.numpy().view(np.uint8).reshape(n, -1)
    off, ind = c.off, c.ind
    for cap in (cfg.cap, 20000):
        # start: the rows of the highest out-degree nodes, as a static cache would hold
        start = np.argsort(-np.bincount(ind, minlength=n), kind="stable")[:cap].astype(np.int32)
        cache = ginex.FeatureCache(feats, cap)
        cache.init(dev(start))
        ex = ginex.Executor(cache)
        state_d, state_h = dev(start), start
        out = None
        link_rows = 0
        for k in range(3):
            seeds, so = seed_batches(train, cfg.batch, S, cfg.seed, first_batch=k * S)
            ref_s = oracle.sample_superbatch(off, ind, seeds.numpy(), so.numpy(), cfg.fanout,
                                             rng_seed=0, first_batch_index=k * S)
            samp = ginex.sample_superbatch(c.w.offsets, c.w.indices, seeds.cuda(), so.numpy(),
                                           cfg.fanout, rng_seed=0, first_batch_index=k * S)
            assert np.array_equal(samp.ids.cpu().numpy(), ref_s["ids"])
            ids, io = ref_s["ids"], ref_s["ids_offsets"]
            ref = oracle.changeset_resume(n, ids, io, cap, state_h)
            cs = ginex.changeset_resume(n, samp.ids, samp.ids_offsets, state_d)
            check_resumed(cs, ref, (n, ids, io))
            longest = int(np.diff(io).max())
            if out is None or out.shape[0] < longest:
                out = torch.empty((longest, cfg.feat_dim), dtype=torch.float32, device="cuda")
            got = {}

            def keep(i, rows):
                got[i] = out[:rows].clone()
            ex.run(samp, cs, out, resumed=True, after_gather=keep)
            torch.cuda.synchronize()
            for i in range(S):
                g = got[i].cpu().numpy().view(np.uint8).reshape(got[i].shape[0], -1)
                assert np.array_equal(g, sb[ids[io[i]:io[i + 1]]]), (cap, k, i)
            # the cache now holds exactly the final state, line by line, with the right bytes
            final = ref["final_ids"]
            addr = cache.addr.cpu().numpy()
            assert np.array_equal(np.sort(np.nonzero(addr >= 0)[0]), np.sort(final))
            assert np.array_equal(addr[final], np.arange(cap))
            rows = cache.rows.cpu().numpy().view(np.uint8).reshape(cap, -1)
            assert np.array_equal(rows, sb[final])
            link_rows += int(ref["miss_count"].sum())
            state_d, state_h = cs.final_ids, final
        assert link_rows > 0


@pytest.mark.parametrize("scatter", ["0", "1"])
def test_both_ways_of_finding_dead_evictions_give_the_same_lists(ginex, case1, case2, scatter,
                                                                 monkeypatch):
    """Large caches find the evicted dead rows from the id bitmap, small ones by a pass over
    the cache lines; GINEX_DEAD_SCATTER forces either way at any size."""
    monkeypatch.setenv("GINEX_DEAD_SCATTER", scatter)
    rng = np.random.default_rng(61)
    for trial in range(40):
        n = int(rng.integers(2, 400))
        S = int(rng.integers(1, 14))
        cap = int(rng.integers(1, n + 1))
        ids, off = random_trace(rng, n, S, int(rng.integers(1, 200)))
        ids_d = dev(ids) if len(ids) else torch.zeros(1, dtype=torch.int32, device="cuda")[:0]
        check_changeset(ginex.changeset(n, ids_d, off, cap), oracle.changeset(n, ids, off, cap))
        start = rng.permutation(n)[:cap].astype(np.int32)
        check_resumed(ginex.changeset_resume(n, ids_d, off, dev(start)),
                      oracle.changeset_resume(n, ids, off, cap, start))
    for c in (case1, case2):
        ids, io = c.samp["ids"], c.samp["ids_offsets"]
        distinct = len(np.unique(ids))
        for cap in (1000, distinct // 16, distinct // 2, distinct - 1):
            check_changeset(ginex.changeset(c.cfg.num_nodes, dev(ids), io, cap),
                            oracle.changeset(c.cfg.num_nodes, ids, io, cap),
                            (c.cfg.num_nodes, ids, io))
        start = np.arange(c.cfg.cap, dtype=np.int32)[::-1].copy()
        check_resumed(ginex.changeset_resume(c.cfg.num_nodes, dev(ids), io, dev(start)),
                      oracle.changeset_resume(c.cfg.num_nodes, ids, io, c.cfg.cap, start),
                      (c.cfg.num_nodes, ids, io))


def test_changeset_at_the_largest_superbatch_the_library_accepts(ginex):
    """S = 8191 iterations (the documented limit) of a few ids each, under eviction pressure,
    for both policies and for a resumed cache."""
    rng = np.random.default_rng(71)
    n, S, cap = 500, 8191, 40
    ids, off = random_trace(rng, n, S, 6)
    ids_d = dev(ids)
    check_changeset(ginex.changeset(n, ids_d, off, cap), oracle.changeset(n, ids, off, cap),
                    (n, ids, off))
    check_changeset(ginex.changeset(n, ids_d, off, cap, policy="lru"),
                    oracle.changeset_lru(n, ids, off, cap), (n, ids, off))
    start = rng.permutation(n)[:cap].astype(np.int32)
    check_resumed(ginex.changeset_resume(n, ids_d, off, dev(start)),
                  oracle.changeset_resume(n, ids, off, cap, start), (n, ids, off))
    with pytest.raises(ginex.GinexError):
        ginex.changeset(n, ids_d, np.concatenate([off, off[-1:]]), cap)     # S = 8192


@pytest.mark.parametrize("S", [1, 2, 31, 32, 33, 255, 256, 1024, 1025, 2047, 2048, 2049])
def test_changeset_around_the_sizes_at_which_the_loop_changes_its_way(ginex, S):
    """Iteration counts around the limits of the per-iteration bookkeeping (one, two or three
    histogram bins per thread of the block that rolls the thresholds forward; 2 048 iterations,
    beyond which the thresholds come from the state's histograms), under eviction pressure, for
    Belady from a fresh and from a given cache."""
    rng = np.random.default_rng(S)
    n, cap = 700, 55
    ids, off = random_trace(rng, n, S, 9)
    ids_d = dev(ids) if len(ids) else torch.zeros(1, dtype=torch.int32, device="cuda")[:0]
    check_changeset(ginex.changeset(n, ids_d, off, cap), oracle.changeset(n, ids, off, cap),
                    (n, ids, off))
    start = rng.permutation(n)[:cap].astype(np.int32)
    check_resumed(ginex.changeset_resume(n, ids_d, off, dev(start)),
                  oracle.changeset_resume(n, ids, off, cap, start), (n, ids, off))


def structured_traces():
    """Traces built to sit on the tie rules and the mode switches of the threshold walk."""
    rng = np.random.default_rng(81)
    n = 600
    out = []
    same = rng.permutation(n)[:150]
    out.append(("every iteration the same ids", [same] * 9))
    out.append(("disjoint iterations", [np.arange(i * 60, (i + 1) * 60) for i in range(10)]))
    out.append(("descending ids, shifted by one each iteration",
                [np.arange(200 + i, i, -1) for i in range(12)]))
    out.append(("one huge iteration among tiny ones",
                [rng.permutation(n)[:5], rng.permutation(n)[:590], rng.permutation(n)[:3],
                 rng.permutation(n)[:590], rng.permutation(n)[:1]]))
    out.append(("two alternating sets", [np.arange(0, 300), np.arange(300, 600)] * 5))
    out.append(("a hot core plus a cold stream",
                [np.concatenate([np.arange(40), 40 + (np.arange(50) + 50 * i) % 560])
                 for i in range(14)]))
    out.append(("empty iterations in between",
                [rng.permutation(n)[:80], np.zeros(0, dtype=np.int64), rng.permutation(n)[:80],
                 np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64), rng.permutation(n)[:80]]))
    return n, out


@pytest.mark.parametrize("scatter", ["0", "1"])
def test_changesets_on_structured_traces(ginex, scatter, monkeypatch):
    monkeypatch.setenv("GINEX_DEAD_SCATTER", scatter)
    monkeypatch.setenv("GINEX_STATIC_THRESHOLDS", scatter)   # both ways of finding the thresholds
    n, traces = structured_traces()
    rng = np.random.default_rng(82)
    for name, tr in traces:
        off = np.cumsum([0] + [len(x) for x in tr]).astype(np.int64)
        ids = np.concatenate(tr).astype(np.int32)
        ids_d = dev(ids)
        distinct = len(np.unique(ids))
        for cap in sorted({1, 2, 39, 40, 41, 59, 60, 61, 150, distinct - 1, distinct, n}):
            if cap < 1:
                continue
            try:
                check_changeset(ginex.changeset(n, ids_d, off, cap), oracle.changeset(n, ids, off, cap),
                                (n, ids, off))
                check_changeset(ginex.changeset(n, ids_d, off, cap, policy="lru"),
                                oracle.changeset_lru(n, ids, off, cap), (n, ids, off))
                for start in (np.arange(cap), np.arange(n - 1, n - 1 - cap, -1),
                              rng.permutation(n)[:cap]):
                    start = start.astype(np.int32)
                    check_resumed(ginex.changeset_resume(n, ids_d, off, dev(start)),
                                  oracle.changeset_resume(n, ids, off, cap, start), (n, ids, off))
            except AssertionError:
                print("failing case:", name, "cap", cap, flush=True)
                raise


def csr_from_rows(rows, n, offsets_64):
    off = np.cumsum([0] + [len(rows.get(v, [])) for v in range(n)])
    ind = np.array([u for v in range(n) for u in rows.get(v, [])], dtype=np.int32)
    return off.astype(np.int64 if offsets_64 else np.int32), ind


@pytest.mark.parametrize("offsets_64", [False, True])
def test_sampler_on_structured_graphs(ginex, offsets_64):
    """A hub, a chain, rows of exactly k-1, k and k+1 neighbours, rows of identical neighbours,
    self loops and isolated seeds, with and without a neighbour cache."""
    n = 2000
    rng = np.random.default_rng(91)
    rows = {0: list(range(1, n))}                                  # hub: everyone
    for v in range(1, 300):
        rows[v] = [v + 1]                                          # chain
    for v, d in zip(range(300, 330), [9, 10, 11] * 10):
        rows[v] = rng.integers(0, n, size=d).tolist()              # around the fanout
    for v in range(330, 360):
        rows[v] = [7] * 40                                         # forty times the same
    for v in range(360, 400):
        rows[v] = [v, v, 0, v]                                     # self loops and the hub
    for v in range(400, 1200):
        rows[v] = rng.integers(0, n, size=int(rng.integers(0, 60))).tolist()
    off, ind = csr_from_rows(rows, n, offsets_64)
    batches = [np.array([0]), np.array([1, 2, 3]), np.arange(300, 400), np.arange(1200, 1300),
               rng.permutation(n)[:500], np.array([1999, 0, 330])]
    seeds = np.concatenate(batches).astype(np.int32)
    so = np.cumsum([0] + [len(b) for b in batches])
    off_d, ind_d = torch.from_numpy(off).cuda(), torch.from_numpy(ind).cuda()
    for fanout in ((10, 10, 10), (3, 1), (64, 2), (11,)):
        ref = oracle.sample_superbatch(off, ind, seeds, so, fanout, rng_seed=5, first_batch_index=3)
        res = ginex.sample_superbatch(off_d, ind_d, dev(seeds), so, fanout, rng_seed=5,
                                      first_batch_index=3)
        check_sample(res, ref, len(batches), len(fanout))
        for budget in (50, len(ind) // 3, len(ind) + n):
            nc = ginex.neighbor_cache_build(off_d, ind_d, budget)
            check_neighbor_cache(nc, oracle.neighbor_cache_build(off, ind, budget))
            res = ginex.sample_superbatch(off_d, ind_d, dev(seeds), so, fanout, rng_seed=5,
                                          first_batch_index=3, neighbor_cache=nc)
            check_sample(res, ref, len(batches), len(fanout))


def test_sampler_degenerate_shapes(ginex):
    """Eight hops (the limit), a superbatch of one batch, a superbatch of empty batches only,
    seeds without neighbours, and a list that saturates at the whole graph."""
    off, ind = small_graph(300, 6000, seed=9)
    o, i = off.numpy(), ind.numpy()
    od, idv = off.cuda(), ind.cuda()
    empty = torch.zeros(1, dtype=torch.int32, device="cuda")[:0]
    cases = [
        ("eight hops", np.array([5, 9, 200], dtype=np.int32), [0, 3], (2,) * 8),
        ("one batch", np.arange(40, dtype=np.int32), [0, 40], (10, 10)),
        ("only empty batches", np.zeros(0, dtype=np.int32), [0, 0, 0, 0], (10, 10, 10)),
        ("the list reaches every node", np.arange(300, dtype=np.int32), [0, 150, 300], (64, 64, 64)),
    ]
    for name, seeds, so, fanout in cases:
        ref = oracle.sample_superbatch(o, i, seeds, so, fanout, rng_seed=2)
        res = ginex.sample_superbatch(od, idv, dev(seeds) if len(seeds) else empty, so, fanout,
                                      rng_seed=2)
        try:
            check_sample(res, ref, len(so) - 1, len(fanout))
        except AssertionError:
            print("failing case:", name, flush=True)
            raise
        # the changeset of whatever came out, for a cache of a quarter of it
        cap = max(1, len(np.unique(ref["ids"])) // 4) if len(ref["ids"]) else 3
        check_changeset(ginex.changeset(300, res.ids if len(ref["ids"]) else empty,
                                        res.ids_offsets, cap),
                        oracle.changeset(300, ref["ids"], ref["ids_offsets"], cap))
    # a graph without any edge: every list is its seeds
    n = 50
    z = torch.zeros(n + 1, dtype=torch.int32)
    seeds = np.array([3, 4, 4, 7], dtype=np.int32)
    ref = oracle.sample_superbatch(z.numpy(), np.zeros(0, dtype=np.int32), seeds, [0, 4], (10, 10))
    res = ginex.sample_superbatch(z.cuda(), empty, dev(seeds), [0, 4], (10, 10))
    check_sample(res, ref, 1, 2)
    assert list(res.ids.cpu().numpy()) == [3, 4, 7]


# ---- static highest-out-degree cache (Section 2.3) ------------------------------------

def test_static_select_matches_oracle_on_small_and_structured_graphs(ginex):
    rng = np.random.default_rng(11)
    graphs = []
    for n, e in ((1, 0), (1, 5), (9, 0), (300, 6000), (5000, 40000), (70000, 900000)):
        graphs.append((n, rng.integers(0, n, size=e).astype(np.int32)))
    graphs.append((9, np.full(9, 5, dtype=np.int32)))                              # star
    graphs.append((40, np.concatenate([np.full(v, v, np.int32) for v in range(40)])))  # ladder
    graphs.append((1000, np.arange(1000, dtype=np.int32)[::-1].copy()))            # all tie
    hub = np.concatenate([np.zeros(300000, np.int32) + 77, rng.integers(0, 500, 2000).astype(np.int32)])
    graphs.append((500, hub))                                                       # 19-bit degree
    for n, ind in graphs:
        ind_d = dev(ind) if len(ind) else torch.zeros(0, dtype=torch.int32, device="cuda")
        for cap in sorted({0, 1, n // 3, n, n + 7}):
            got = ginex.static_select(n, ind_d, cap).cpu().numpy()
            want = oracle.static_select(n, ind, cap)
            assert np.array_equal(got, want), (n, len(ind), cap)
    with pytest.raises(ginex.GinexError) as err:
        ginex.static_select(10, dev(np.array([1, 2, 10], dtype=np.int32)), 3)
    assert err.value.code == -4


@pytest.mark.parametrize("which", ["case1", "case2"])
def test_static_cache_through_the_executor(ginex, which, request):
    c = request.getfixturevalue(which)
    n, cap = c.cfg.num_nodes, c.cfg.cap
    sel = ginex.static_select(n, c.w.indices, cap)
    want_sel = oracle.static_select(n, c.ind, cap)
    assert np.array_equal(sel.cpu().numpy(), want_sel)
    # the indices may also sit in pinned host memory
    pinned = torch.empty(c.w.indices.numel(), dtype=torch.int32, pin_memory=True)
    pinned.copy_(c.w.indices)
    assert torch.equal(ginex.static_select(n, pinned, cap), sel)
    slow = c.w.features
    sb = slow.numpy().view(np.uint8).reshape(slow.shape[0], -1)
    cache = ginex.FeatureCache(slow, cap)
    cache.init(sel)
    ref = oracle.Cache(slow.numpy(), cap)
    ref.init(want_sel)
    assert np.array_equal(cache.addr.cpu().numpy(), ref.addr)
    ids_d = dev(c.samp["ids"])
    io = c.samp["ids_offsets"]
    counter = torch.zeros(1, dtype=torch.int64, device="cuda")
    none = np.zeros(0, dtype=np.int32)
    hits = 0
    for i in range(c.cfg.S):
        ids_i = c.samp["ids"][io[i]:io[i + 1]]
        cache.count_misses(ids_d[io[i]:io[i + 1]], counter)
        out = cache.gather(ids_d[io[i]:io[i + 1]])
        got = out.cpu().numpy().view(np.uint8).reshape(out.shape[0], -1)
        want, h = ref.gather_update(ids_i, none, none, none)
        hits += h
        assert np.array_equal(got, want), i
        assert np.array_equal(got, sb[ids_i]), i
    misses = int(counter.item())
    assert misses == len(c.samp["ids"]) - hits
    assert misses == oracle.static_misses(n, c.samp["ids"], want_sel)
    assert np.array_equal(cache.addr.cpu().numpy(), ref.addr)          # a static cache never changes
    assert misses >= int(c.cs["miss_count"].sum())                      # Belady is the lower bound


# ---- gather through the lines resolved by the changeset stage ---------------------------

@pytest.mark.parametrize("which", ["case1", "case2"])
def test_gather_through_resolved_lines_matches_oracle(ginex, which, request):
    """ginex_gather_lines on every iteration: bytes equal to the oracle's gather, address
    table and cache rows equal to the oracle's replay, for a cache under pressure, the
    configured cache, a cache that holds everything and no cache at all."""
    c = request.getfixturevalue(which)
    n, S = c.cfg.num_nodes, c.cfg.S
    ids, io = c.samp["ids"], c.samp["ids_offsets"]
    ids_d = dev(ids)
    slow = c.w.features
    distinct = len(np.unique(ids))
    for cap in (max(1, distinct // 16), c.cfg.cap, distinct + 3, 0):
        ref_cs = oracle.changeset(n, ids, io, cap)
        cs = ginex.changeset(n, ids_d, io, cap)
        check_changeset(cs, ref_cs, (n, ids, io))
        cache = ginex.FeatureCache(slow, cap)
        cache.init(cs.init_ids)
        ref = oracle.Cache(slow.numpy(), cap)
        ref.init(ref_cs["init_ids"])
        co = cs.cs_offsets
        for i in range(S):
            sl = slice(co[i], co[i + 1])
            a, b = io[i], io[i + 1]
            out = cache.gather(ids_d[a:b], None, cs.in_ids[sl], cs.out_ids[sl], cs.in_positions[sl],
                               src_line=cs.src_line[a:b])
            want, _ = ref.gather_update(ids[a:b], ref_cs["in_ids"][sl], ref_cs["out_ids"][sl],
                                        ref_cs["in_positions"][sl])
            got = out.cpu().numpy().view(np.uint8).reshape(out.shape[0], -1)
            assert np.array_equal(got, want), (cap, i)
            assert np.array_equal(got, oracle.gather(slow.numpy(), ids[a:b])), (cap, i)
        assert np.array_equal(cache.addr.cpu().numpy(), ref.addr), cap
        if cap:
            rows = cache.rows.cpu().numpy().view(np.uint8).reshape(cache.rows.shape[0], -1)
            used = len(ref_cs["init_ids"])
            assert np.array_equal(rows[:used], ref.rows[:used]), cap


@pytest.mark.parametrize("row_bytes", [16, 48, 512, 3072])
def test_gather_lines_row_sizes(ginex, row_bytes):
    rng = np.random.default_rng(row_bytes)
    n, cap = 5000, 700
    slow = torch.from_numpy(rng.integers(0, 2 ** 31, size=(n, row_bytes // 4)).astype(np.int32)).pin_memory()
    cache = ginex.FeatureCache(slow, cap)
    init = rng.permutation(n)[:cap].astype(np.int32)
    cache.init(dev(init))
    line_of = np.full(n, -1, dtype=np.int32)
    line_of[init] = np.arange(cap, dtype=np.int32)
    for count in (0, 1, 63, 64, 65, 1000, 4097):
        ids = rng.integers(0, n, size=count).astype(np.int32)
        ids_d = dev(ids) if count else torch.zeros(0, dtype=torch.int32, device="cuda")
        lines = dev(line_of[ids]) if count else torch.zeros(0, dtype=torch.int32, device="cuda")
        out = cache.gather(ids_d, src_line=lines)
        assert np.array_equal(out.cpu().numpy().view(np.uint8).reshape(count, row_bytes),
                              oracle.gather(slow.numpy(), ids))


# ---- determinism across launch shapes ------------------------------------------------------

@pytest.mark.parametrize("tiles", ["1", "3", "100000"])
def test_sampler_is_independent_of_the_launch_shape(ginex, case1, case2, tiles, monkeypatch):
    """Another assignment of tiles to blocks (fewer, longer-running blocks, or one block per
    tile) changes the order in which candidates reach the hash tables, not the result."""
    for c in (case1, case2):
        base = run_sample(ginex, c)
        monkeypatch.setenv("GINEX_SAMPLER_TILES", tiles)
        other = run_sample(ginex, c)
        monkeypatch.delenv("GINEX_SAMPLER_TILES")
        for name in ("ids", "adj_rowptr", "adj_col"):
            assert torch.equal(getattr(base, name), getattr(other, name)), (tiles, name)
        assert np.array_equal(base.ids_offsets, other.ids_offsets)
        assert np.array_equal(base.hop_sizes, other.hop_sizes)
        check_sample(other, c.samp, c.cfg.S, len(c.cfg.fanout))


def test_seeds_and_first_hop_in_lds_equal_the_tables_in_hbm(ginex, case1, case2, monkeypatch):
    """Seeds and hop 0 of a batch are deduplicated in the LDS of one workgroup when their hash
    set fits there; GINEX_SAMPLER_LDS=0 sends them through the tables in HBM like the later
    hops.  Both ways against the oracle and against each other, with and without adj, on
    the fixtures and on shapes at the edges of what the LDS path takes (1024 seeds, a
    repeated seed, an empty batch, a fanout that selects 32- and 64-lane groups)."""
    from workload import make_workload
    for c in (case1, case2):
        ref = run_sample(ginex, c)
        check_sample(ref, c.samp, c.cfg.S, len(c.cfg.fanout))
        monkeypatch.setenv("GINEX_SAMPLER_LDS", "0")
        other = run_sample(ginex, c)
        no_adj = run_sample(ginex, c, with_adj=False)
        monkeypatch.delenv("GINEX_SAMPLER_LDS")
        check_sample(other, c.samp, c.cfg.S, len(c.cfg.fanout))
        for name in ("ids", "adj_rowptr", "adj_col"):
            assert torch.equal(getattr(ref, name), getattr(other, name)), name
        assert np.array_equal(ref.hop_sizes, other.hop_sizes)
        assert torch.equal(no_adj.ids, ref.ids)
    w = make_workload(1)
    off, ind = w.offsets.numpy(), w.indices.numpy()
    n = w.cfg.num_nodes
    rng = np.random.default_rng(9)
    shapes = [([1024, 0, 1, 700], (10, 3)), ([300, 299], (20, 2)), ([150, 1], (40, 2)),
              ([1025, 10], (5, 2))]          # the last one does not fit: 1025 seeds
    for sizes, fanout in shapes:
        seeds = [rng.integers(0, n, size=m).astype(np.int32) for m in sizes]
        if len(seeds[0]) > 4:
            seeds[0][3] = seeds[0][1]            # a repeated seed
        so = np.cumsum([0] + sizes).astype(np.int64)
        flat = np.concatenate(seeds).astype(np.int32)
        want = oracle.sample_superbatch(off, ind, flat, so, list(fanout), rng_seed=5,
                                        first_batch_index=7)
        results = []
        for lds in ("1", "0"):
            monkeypatch.setenv("GINEX_SAMPLER_LDS", lds)
            got = ginex.sample_superbatch(w.offsets.cuda(), w.indices.cuda(), dev(flat), so,
                                          list(fanout), rng_seed=5, first_batch_index=7)
            check_sample(got, want, len(sizes), len(fanout))
            results.append(got)
        monkeypatch.delenv("GINEX_SAMPLER_LDS")
        assert torch.equal(results[0].adj_col, results[1].adj_col)


def test_changeset_is_independent_of_the_eviction_path_and_repeatable(ginex, case2, monkeypatch):
    """The two ways of finding evictions among dead rows use different grids and atomics; both,
    and a second run of each, give byte-identical lists, lines and final states."""
    c = case2
    n = c.cfg.num_nodes
    ids_d = dev(c.samp["ids"])
    io = c.samp["ids_offsets"]
    # a carried cache with room for every row of the superbatch: the short launch sequence
    big = len(np.unique(c.samp["ids"])) + 1000
    start = dev(np.arange(big, dtype=np.int32)[::-1].copy())
    results = []
    for scatter, live, planned in (("0", "0", "1"), ("1", "0", "1"), ("0", "1", "1"), ("1", "1", "1"),
                                   ("0", "0", "0"), ("1", "0", "0"), ("0", "0", "2"), ("1", "0", "2")):
        monkeypatch.setenv("GINEX_DEAD_SCATTER", scatter)
        monkeypatch.setenv("GINEX_LIVE_SELECT", live)   # keeps the live-select launches in the loop
        monkeypatch.setenv("GINEX_PLANNED", planned)    # 0: the loop also where no loop is needed
        # the thresholds of the general loop from histograms of the state (0) or in front of it
        monkeypatch.setenv("GINEX_STATIC_THRESHOLDS", scatter)
        a = ginex.changeset(n, ids_d, io, 20000)
        b = ginex.changeset_resume(n, ids_d, io, start)
        results.append((a, b))
    first = results[0]
    for a, b in results[1:]:
        for x, y in ((a, first[0]), (b, first[1])):
            for name in ("in_ids", "out_ids", "in_positions", "src_line"):
                assert torch.equal(getattr(x, name), getattr(y, name)), name
            assert np.array_equal(x.cs_offsets, y.cs_offsets)
            assert np.array_equal(x.miss_count, y.miss_count)
        assert torch.equal(b.final_ids, first[1].final_ids)
