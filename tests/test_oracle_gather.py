"""Pins for the oracle's gather / cache update / cache initialization (CPU only).

Section 3.1 ("Feature Cache Initialization", "Main Loop") and Section 3.3 ("Feature Cache
Update" with its worked example).
"""
import os

import numpy as np

import oracle
from workload import make_workload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def load_example():
    kv = {}
    for line in open(os.path.join(GOLDEN, "gather_update_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        kv[k] = [int(x) for x in v]
    return kv


def test_worked_example_of_the_paper():
    ex = load_example()
    n = ex["num_nodes"][0]
    slow = np.arange(n * 4, dtype=np.float32).reshape(n, 4) + 0.5
    c = oracle.Cache(slow, len(ex["cached"]))
    c.init(ex["cached"])
    assert [int(v) for v in np.nonzero(c.addr >= 0)[0]] == ex["cached"]
    line_of_0, line_of_6 = int(c.addr[0]), int(c.addr[6])
    out, hits = c.gather_update(ex["ids"], ex["in_ids"], ex["out_ids"], ex["in_positions"])
    # the batch input is in ids order, whatever tier served the row
    assert np.array_equal(out.view(np.float32), slow[ex["ids"]])
    assert hits == len(ex["hits"])
    # node 0 was a hit and is evicted in the same iteration; 2 and 5 inherit the lines
    assert c.addr[0] == -1 and c.addr[6] == -1
    assert c.addr[2] == line_of_0 and c.addr[5] == line_of_6
    assert [int(v) for v in np.nonzero(c.addr >= 0)[0]] == ex["cached_after"]
    for v in ex["cached_after"]:
        assert np.array_equal(c.rows[c.addr[v]].view(np.float32), slow[v])


def test_gather_is_row_selection_and_cache_stays_coherent():
    w = make_workload(1)
    r = oracle.sample_superbatch(w.offsets.numpy(), w.indices.numpy(), w.seeds.numpy(),
                                 w.seed_offsets.numpy(), w.cfg.fanout)
    cs = oracle.changeset(w.cfg.num_nodes, r["ids"], r["ids_offsets"], w.cfg.cap)
    slow = w.features.numpy()
    sb = slow.view(np.uint8).reshape(slow.shape[0], -1)
    c = oracle.Cache(slow, w.cfg.cap)
    c.init(cs["init_ids"])
    for i in range(w.cfg.S):
        ids = r["ids"][r["ids_offsets"][i]:r["ids_offsets"][i + 1]]
        lo, hi = cs["cs_offsets"][i], cs["cs_offsets"][i + 1]
        expect_hits = len(ids) - cs["miss_count"][i]
        out, hits = c.gather_update(ids, cs["in_ids"][lo:hi], cs["out_ids"][lo:hi],
                                    cs["in_positions"][lo:hi])
        assert hits == expect_hits
        assert np.array_equal(out, sb[ids])                    # closed form
        assert np.array_equal(out, oracle.gather(slow, ids))
        res = np.nonzero(c.addr >= 0)[0]
        assert len(res) <= w.cfg.cap
        assert np.array_equal(c.rows[c.addr[res]], sb[res])    # every cached row is right


def test_resolved_lines_on_the_worked_example_and_against_the_cache_replay():
    ex = load_example()
    n = ex["num_nodes"][0]
    # one iteration, then the same ids once more: after the update 2 and 5 sit in the lines
    # of 0 and 6, and 0 is gone
    ids = ex["ids"] + ex["ids"]
    lines = oracle.resolve_lines(n, ids, [0, 4, 8], ex["cached"], ex["in_ids"], ex["out_ids"],
                                 [0, 2, 2])
    assert lines[:4].tolist() == ex["src_line"]
    assert lines[4:].tolist() == [-1, 0, 4, 3]
    # on a sampled workload: equal to the address table of the full cache replay, iteration
    # by iteration, and consistent with the miss counts
    w = make_workload(1)
    r = oracle.sample_superbatch(w.offsets.numpy(), w.indices.numpy(), w.seeds.numpy(),
                                 w.seed_offsets.numpy(), w.cfg.fanout)
    for cap in (w.cfg.cap, 300, 10 ** 6, 0):
        cs = oracle.changeset(w.cfg.num_nodes, r["ids"], r["ids_offsets"], cap)
        lines = oracle.resolve_lines(w.cfg.num_nodes, r["ids"], r["ids_offsets"], cs["init_ids"],
                                     cs["in_ids"], cs["out_ids"], cs["cs_offsets"])
        c = oracle.Cache(w.features.numpy(), cap)
        c.init(cs["init_ids"])
        for i in range(w.cfg.S):
            a, b = r["ids_offsets"][i], r["ids_offsets"][i + 1]
            lo, hi = cs["cs_offsets"][i], cs["cs_offsets"][i + 1]
            assert np.array_equal(lines[a:b], c.addr[r["ids"][a:b]])
            assert int((lines[a:b] < 0).sum()) == cs["miss_count"][i]
            c.gather_update(r["ids"][a:b], cs["in_ids"][lo:hi], cs["out_ids"][lo:hi],
                            cs["in_positions"][lo:hi])
