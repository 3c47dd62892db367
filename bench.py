#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

A step is one pass of the inspector-executor path over one superbatch:
  ginex_sample_superbatch -> ginex_changeset -> ginex_cache_init ->
  S x (ginex_gather_lines + ginex_cache_update)
on a synthetic R-MAT workload (default: configuration 4, the 111M-node graph with the
feature table in host-pinned memory).  Consecutive steps take consecutive, different
superbatches.  Prints ONE JSON line.

Besides the timed steps the same run times, by default, the legs in which the parts of the
path that configuration 4's own cache size never exercises do run (--legs):
  pressure   the last superbatch again with a cache of distinct/16 rows: the Belady loop
             evicts every iteration, the executor updates the cache and reads misses from
             the slow tier (gather "G3": real hit/miss mix against the two-term bound)
  carried    the cache carried from superbatch to superbatch (ginex_changeset_resume), steady
             state: no initialization; where the cache holds every row of a superbatch
             (configurations 3 and 4) the changesets follow without the loop over the state,
             elsewhere the loop runs from the carried state
  allmiss    the gather kernel with nothing resident (gather "G2": pure host link)
The gathers of the timed steps are "G1" whenever the configuration never misses (3 and 4).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--legs a,b|none]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "sampled edges/s; Belady changeset accesses/s; gather GB/s vs HBM peak"
HBM_PEAK_GBPS = 8000.0
HOST_LINK_GBPS = 64.0     # PCIe Gen5 x16, raw
LINE_BYTES = 128          # what one random access moves between HBM and L2
# random lines a sampled edge cannot avoid: its neighbour id and its hash-table slot
# (the two row offsets of a frontier node are shared by its picks, everything else is
# sequential)
SAMPLER_LINES_PER_EDGE = 2.0
# algorithmic bytes per sampled edge: 4 index read + 4 adj_col write + 8 hash probe +
# 1.6 offsets (two 8-byte offsets per frontier node, fanout 10) + 4 x (share of new ids)
SAMPLER_BYTES_PER_EDGE = 20.0
# changeset, per access: four radix passes of the (node, position) pairs (8-byte histogram
# read, 8 read, 8 written each; the first pass reads the 4-byte ids instead, twice) and the
# look-right pass (12); then the loop's id, key, address-table probe and key refresh (16)
CHANGESET_BUILD_BYTES_PER_ACCESS = 100
CHANGESET_LOOP_BYTES_PER_ACCESS = 16
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch (or per call) of `kernel` from the rocprofv3 --pmc runs recorded
    under profiles/ (FETCH_SIZE and WRITE_SIZE, scaled by the plain-copy calibration), or
    None when no counter run exists for this workload."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)[workload][kernel]
        return rec["fetch_bytes_per_launch"] + rec["write_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def event():
    return torch.cuda.Event(enable_timing=True)


def med(v):
    return float(np.median(v)) if len(v) else 0.0


class Runner:
    """Holds every buffer of the path so that steps allocate (almost) nothing."""

    def __init__(self, ginex, w, superbatches):
        from paper_2208_09151_amd import _lib, api
        self.g, self.w, self.cfg = ginex, w, w.cfg
        cfg = w.cfg
        self.sbs = superbatches          # (seeds device, seed_offsets host, first batch index)
        self.S = len(superbatches[0][1]) - 1
        lib = _lib.load()
        fo = np.asarray(cfg.fanout, dtype=np.int32)
        so_all = [sb[1] for sb in superbatches]
        max_batch = max(int(np.max(np.diff(so))) for so in so_all)
        ws_s = lib.ginex_sample_workspace_bytes(cfg.num_nodes, self.S, max_batch,
                                                fo.ctypes.data, len(fo))
        caps = [api.sample_capacity(cfg.num_nodes, so, cfg.fanout) for so in so_all]
        ci, cr, cc = (max(c[j] for c in caps) for j in range(3))
        ws_c = lib.ginex_changeset_workspace_bytes(cfg.num_nodes, ci, self.S, cfg.cap)
        log(f"workspace: sample {ws_s / 2**30:.2f} GiB, changeset {ws_c / 2**30:.2f} GiB")
        # the two stages run one after the other: one workspace serves both
        self.ws = torch.empty(max(ws_s, ws_c), dtype=torch.uint8, device="cuda")
        self.out_bufs = (torch.empty(ci, dtype=torch.int32, device="cuda"),
                         torch.empty(cr, dtype=torch.int64, device="cuda"),
                         torch.empty(cc, dtype=torch.int32, device="cuda"))
        self.cache = ginex.FeatureCache(w.features, cfg.cap)
        self.executor = ginex.Executor(self.cache)
        self.batch_input = torch.empty((min(cfg.num_nodes, max_batch * 11 ** len(cfg.fanout)),
                                        cfg.feat_dim), dtype=torch.float32, device="cuda")
        self.last = None
        # event pairs around every gather launch, created once: the executor loop must
        # enqueue faster than the GPU drains, or the event pair would also time the host
        self.pairs = [(event(), event()) for _ in range(self.S)]
        self.stage_events = [event() for _ in range(5)]

    def sample(self, k):
        seeds, so, first = self.sbs[k % len(self.sbs)]
        return self.g.sample_superbatch(self.w.offsets, self.w.indices, seeds, so, self.cfg.fanout,
                                        rng_seed=0, first_batch_index=first, workspace=self.ws,
                                        out=self.out_bufs)

    def step(self, k, timers=None, events=None, streamed=False):
        """Superbatch k through the whole path.  All timing is by HIP events on the stream
        the kernels are launched on (torch's current stream)."""
        g, cfg = self.g, self.cfg
        e = self.stage_events
        e[0].record()
        samp = self.sample(k)
        e[1].record()
        cs = g.changeset(cfg.num_nodes, samp.ids, samp.ids_offsets, cfg.cap, workspace=self.ws)
        e[2].record()
        # the executor: cache initialization, then per iteration one gather (one kernel) and,
        # when the changeset is not empty, one cache update
        pairs = self.pairs if events is not None else None
        before = (lambda i: pairs[i][0].record()) if pairs is not None else None
        after = (lambda i, n: pairs[i][1].record()) if pairs is not None else None
        fill_end = self.executor.run(samp, cs, self.batch_input, streamed=streamed,
                                     before_gather=before, after_gather=after)
        e[3].record()
        torch.cuda.synchronize()
        if timers is not None:
            timers["sample_s"].append(e[0].elapsed_time(e[1]) / 1e3)
            timers["changeset_s"].append(e[1].elapsed_time(e[2]) / 1e3)
            timers["cache_init_s"].append(e[2].elapsed_time(fill_end) / 1e3)
            timers["gather_update_s"].append(fill_end.elapsed_time(e[3]) / 1e3)
            timers["executor_s"].append(e[2].elapsed_time(e[3]) / 1e3)
            timers["edges"].append(int(samp.totals[2]))
            timers["accesses"].append(int(samp.totals[0]))
            timers["misses"].append(int(cs.miss_count.sum()))
            timers["changes"].append(int(cs.cs_offsets[-1]))
            timers["init_rows"].append(int(cs.init_ids.numel()))
        if events is not None:
            events.extend(a.elapsed_time(b) for a, b in self.pairs)
        self.last = (samp, cs)
        return samp, cs


def cpu_baseline(w, n_batches):
    """The oracle, as it stands, on the first `n_batches` batches of the same workload,
    one thread: sample, changeset (cache scaled to the sample), gather + cache update."""
    import oracle
    cfg = w.cfg
    S = len(w.seed_offsets) - 1
    nb = min(n_batches, S)
    off = w.offsets.cpu().numpy()
    ind = w.indices.cpu().numpy()
    so = w.seed_offsets.numpy()[:nb + 1]
    seeds = w.seeds.numpy()[:so[-1]]
    try:
        os.sched_setaffinity(0, {sorted(os.sched_getaffinity(0))[0]})
    except OSError:
        pass
    t0 = time.perf_counter()
    s = oracle.sample_superbatch(off, ind, seeds, so, cfg.fanout, rng_seed=0)
    t1 = time.perf_counter()
    cap = max(1, cfg.cap * nb // S)
    c = oracle.changeset(cfg.num_nodes, s["ids"], s["ids_offsets"], cap)
    t2 = time.perf_counter()
    slow = w.features.numpy()
    cache = oracle.Cache(slow, cap)
    cache.init(c["init_ids"])
    rows = 0
    for i in range(nb):
        sl = slice(c["cs_offsets"][i], c["cs_offsets"][i + 1])
        ids_i = s["ids"][s["ids_offsets"][i]:s["ids_offsets"][i + 1]]
        cache.gather_update(ids_i, c["in_ids"][sl], c["out_ids"][sl], c["in_positions"][sl])
        rows += len(ids_i)
    t3 = time.perf_counter()
    edges = int(len(s["adj_col"]))
    row_bytes = cfg.feat_dim * 4
    return {
        "value": edges / (t3 - t0),
        "unit": "sampled edges/s (whole hot path)",
        "cores": 1,
        "kind": "oracle",
        "sample": f"first {nb} of {S} batches of the same workload; cache scaled to "
                  f"{cap} rows; sample {t1 - t0:.2f}s, changeset {t2 - t1:.2f}s, "
                  f"init+gather+update {t3 - t2:.2f}s",
        "sample_edges_per_s": edges / (t1 - t0),
        "changeset_accesses_per_s": len(s["ids"]) / (t2 - t1),
        "gather_GBps": 2 * rows * row_bytes / (t3 - t2) / 1e9,
        "host_cpus": os.cpu_count(),
    }


def two_term_bound_s(hits, misses, row_bytes):
    """Lower bound on the time of a gather: resident rows are read from and written to HBM,
    missing rows cross the host link once (their HBM write hides under the link)."""
    return (hits * 2 * row_bytes + (hits + misses) * 8) / (HBM_PEAK_GBPS * 1e9) + \
        misses * row_bytes / (HOST_LINK_GBPS * 1e9)


def changeset_roofline(name, accesses, iterations, cap, changes, seconds, line_passes, traffic):
    """Algorithmic bytes of a changeset call whose loop ran: build + per-access loop work +
    one 4-byte key per cache line and iteration for every pass over the lines + 12 bytes per
    changeset record."""
    algo = accesses * (CHANGESET_BUILD_BYTES_PER_ACCESS + CHANGESET_LOOP_BYTES_PER_ACCESS) + \
        iterations * cap * 4 * line_passes + 12 * changes
    r = {"kernel": name, "bound": "hbm", "achieved": algo / seconds / 1e9, "peak": HBM_PEAK_GBPS,
         "unit": "GB/s", "traffic": traffic, "algorithmic_bytes": algo,
         "call_ms": seconds * 1e3, "accesses_per_s": accesses / seconds}
    r["frac"] = r["achieved"] / r["peak"]
    return r


def pressure_leg(ginex, w, run, samp, divisor, reps=3):
    """The same superbatch with a cache of distinct/divisor rows: every iteration evicts, the
    executor updates the cache and reads its misses over the host link."""
    cfg = w.cfg
    distinct = int(torch.unique(samp.ids).numel())
    cap = max(1, distinct // divisor)
    times = []
    cs = None
    for _ in range(reps):
        a, b = event(), event()
        a.record()
        cs = ginex.changeset(cfg.num_nodes, samp.ids, samp.ids_offsets, cap, workspace=run.ws)
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b) / 1e3)
    cache = ginex.FeatureCache(w.features, cap)
    ex = ginex.Executor(cache)
    pairs = run.pairs
    e0, e1 = event(), event()
    e0.record()
    fill_end = ex.run(samp, cs, run.batch_input, streamed=False,
                      before_gather=lambda i: pairs[i][0].record(),
                      after_gather=lambda i, n: pairs[i][1].record())
    e1.record()
    torch.cuda.synchronize()
    accesses, misses = int(samp.totals[0]), int(cs.miss_count.sum())
    S = run.S
    row_bytes = cfg.feat_dim * 4
    gather_ms = [a.elapsed_time(b) for a, b in pairs]
    n_i = np.diff(samp.ids_offsets)
    bound_ms = [two_term_bound_s(int(n_i[i] - cs.miss_count[i]), int(cs.miss_count[i]), row_bytes) * 1e3
                for i in range(S)]
    g_s = float(np.sum(gather_ms)) / 1e3
    t = med(times)
    changes = int(cs.cs_offsets[-1])
    leg = {"cache_rows": cap, "distinct_rows": distinct, "accesses": accesses, "misses": misses,
           "miss_ratio": misses / accesses, "changes": changes,
           "changeset_ms": t * 1e3, "changeset_accesses_per_s": accesses / t,
           "cache_init_ms": e0.elapsed_time(fill_end),
           "gather_update_ms": fill_end.elapsed_time(e1),
           "gather_launch_ms_median": med(gather_ms)}
    g3 = {"kernel": "k_gather_lines (G3: real hit/miss mix, misses read from host-pinned memory)",
          "bound": "hbm + host link",
          "achieved": accesses * (8 + 2 * row_bytes) / g_s / 1e9, "unit": "GB/s",
          "host_link_GBps": misses * row_bytes / g_s / 1e9,
          "two_term_bound_ms_per_launch": float(np.mean(bound_ms)),
          "avg_launch_ms": float(np.mean(gather_ms)), "launches": S,
          "frac": float(np.sum(bound_ms)) / float(np.sum(gather_ms)),
          "miss_fraction": misses / accesses}
    roof = changeset_roofline("ginex_changeset (build + Belady loop, every iteration evicts)",
                              accesses, S, cap, changes, t, 1,
                              measured_traffic(cfg.name, "changeset_pressure"))
    del cache, ex
    return leg, g3, roof


def carried_leg(ginex, w, run, first_sb, warm=3, timed=3):
    """The cache carried from superbatch to superbatch (ginex_changeset_resume): no
    initialization, only rows that are not resident any more cross the host link.  `warm`
    superbatches bring the cache towards its steady state, `timed` more are measured, each
    stage after the other."""
    cfg = w.cfg
    start = ginex.static_select(cfg.num_nodes, w.indices, cfg.cap)
    cache = ginex.FeatureCache(w.features, cfg.cap)
    cache.init(start)
    ex = ginex.Executor(cache)
    state = start
    rows = {k: [] for k in ("sample_ms", "changeset_ms", "executor_ms", "total_ms", "edges",
                            "accesses", "misses", "changes")}
    for j in range(warm + timed):
        e = [event() for _ in range(4)]
        e[0].record()
        samp = run.sample(first_sb + j)
        e[1].record()
        cs = ginex.changeset_resume(cfg.num_nodes, samp.ids, samp.ids_offsets, state,
                                    workspace=run.ws)
        e[2].record()
        ex.run(samp, cs, run.batch_input, resumed=True)
        e[3].record()
        torch.cuda.synchronize()
        state = cs.final_ids
        if j >= warm:
            rows["sample_ms"].append(e[0].elapsed_time(e[1]))
            rows["changeset_ms"].append(e[1].elapsed_time(e[2]))
            rows["executor_ms"].append(e[2].elapsed_time(e[3]))
            rows["total_ms"].append(e[0].elapsed_time(e[3]))
            rows["edges"].append(int(samp.totals[2]))
            rows["accesses"].append(int(samp.totals[0]))
            rows["misses"].append(int(cs.miss_count.sum()))
            rows["changes"].append(int(cs.cs_offsets[-1]))
    acc, t = med(rows["accesses"]), med(rows["changeset_ms"]) / 1e3
    leg = {"cache_rows": cfg.cap, "superbatches_timed": timed, "superbatches_before": warm,
           "accesses": acc, "misses": med(rows["misses"]), "changes": med(rows["changes"]),
           "miss_ratio": float(np.sum(rows["misses"])) / float(np.sum(rows["accesses"])),
           "sample_ms": med(rows["sample_ms"]), "changeset_ms": t * 1e3,
           "changeset_accesses_per_s": acc / t, "executor_ms": med(rows["executor_ms"]),
           "ms_per_superbatch": med(rows["total_ms"]),
           "edges_per_s": med(rows["edges"]) / (med(rows["total_ms"]) / 1e3)}
    roof = changeset_roofline("ginex_changeset_resume (next-use sort + changesets of a carried cache "
                              "that holds the superbatch: no loop over the state)",
                              acc, run.S, 0, med(rows["changes"]), t, 0,
                              measured_traffic(cfg.name, "changeset_carried"))
    del cache, ex
    return leg, roof


def allmiss_leg(ginex, w, run, samp, launches=16):
    """G2: the gather kernel with nothing resident, every row read over the host link."""
    cfg = w.cfg
    cache = ginex.FeatureCache(w.features, 0)
    cache.init(torch.zeros(0, dtype=torch.int32, device="cuda"))
    io = samp.ids_offsets
    lines = torch.full((int(np.diff(io).max()),), -1, dtype=torch.int32, device="cuda")
    ms, rows = [], 0
    for i in range(min(launches, run.S - 1) + 1):
        a, b = event(), event()
        n = int(io[i + 1] - io[i])
        a.record()
        cache.gather(samp.ids[io[i]:io[i + 1]], run.batch_input[:n], src_line=lines[:n], n_slow=n)
        b.record()
        if i:                       # the first launch warms up
            ms.append((a, b))
            rows += n
    torch.cuda.synchronize()
    if not ms:
        return None
    t = float(np.sum([a.elapsed_time(b) for a, b in ms])) / 1e3
    row_bytes = cfg.feat_dim * 4
    g = rows * row_bytes / t / 1e9
    del cache
    return {"kernel": "k_gather_lines (G2: nothing resident, every row from host-pinned memory)",
            "bound": "host link", "achieved": g, "peak": HOST_LINK_GBPS, "unit": "GB/s",
            "frac": g / HOST_LINK_GBPS, "avg_launch_ms": t * 1e3 / len(ms), "launches": len(ms),
            "rows_per_launch": rows / len(ms)}


def pipeline_leg(ginex, w, K):
    """Inspector of K consecutive superbatches, three ways: sampling only, sampling and
    changesets one after the other, changeset(k) overlapped with sample(k+1)."""
    from workload.configs import seed_batches, train_nodes
    cfg = w.cfg
    train = train_nodes(cfg.num_nodes, cfg.train_frac, cfg.seed, device="cuda")
    sbs = []
    for k in range(K):
        seeds, so = seed_batches(train, cfg.batch, cfg.S, cfg.seed, first_batch=k * cfg.S)
        sbs.append((seeds.cuda(), so.numpy(), k * cfg.S))
    pipe = ginex.InspectorPipeline(w.offsets, w.indices, cfg.num_nodes, cfg.fanout, cfg.cap,
                                   cfg.batch, cfg.S)
    out = {"superbatches": K}
    for mode in ("sample_only", "sequential", "overlap"):
        pipe.run(sbs[:2], mode=mode)                       # warm-up
        out[mode + "_ms"] = min(pipe.run(sbs, mode=mode) for _ in range(3)) * 1e3
    out["changeset_hidden_ms"] = out["sequential_ms"] - out["overlap_ms"]
    out["changeset_exposed_ms"] = out["overlap_ms"] - out["sample_only_ms"]

    # the whole path: executor of superbatch k under the inspector of superbatch k+1
    cache = ginex.FeatureCache(w.features, cfg.cap)
    batch_input = torch.empty((min(cfg.num_nodes, cfg.batch * 11 ** len(cfg.fanout)), cfg.feat_dim),
                              dtype=torch.float32, device="cuda")
    edges = [0]

    executor = ginex.Executor(cache)
    streamed = [True]
    reuse = [0, 0]

    def execute(k, samp, cs):
        if len(executor.caches) > 1 and executor.warm:
            reuse[0] += int((executor.cache.addr[cs.init_ids.long()] >= 0).sum())
            reuse[1] += cs.init_ids.numel()
        executor.run(samp, cs, batch_input, streamed=streamed[0])
        torch.cuda.current_stream().synchronize()
        edges[0] += int(samp.totals[2])

    for key, overlap, st, warm in (("whole_path_stage_by_stage", False, False, False),
                                   ("whole_path_sequential", False, True, False),
                                   ("whole_path_overlapped", True, True, False),
                                   ("whole_path_overlapped_warm_init", True, True, True)):
        streamed[0] = st
        if warm:
            # a second cache array: rows that the previous superbatch's cache still holds
            # are copied from it instead of crossing the host link again
            executor = ginex.Executor(cache, second=ginex.FeatureCache(w.features, cfg.cap))
        pipe.run_with_executor(sbs[:2], execute, overlap=overlap)      # warm-up
        edges[0] = 0
        t = pipe.run_with_executor(sbs, execute, overlap=overlap)
        out[key + "_ms_per_superbatch"] = t * 1e3 / K
        out[key + "_edges_per_s"] = edges[0] / t
    out["warm_init_rows_found_in_previous_cache"] = reuse[0] / max(reuse[1], 1)

    # The cache carried from superbatch to superbatch: no initialization at all, every
    # superbatch starts from what the one before left (ginex_changeset_resume); only rows
    # that are not resident any more cross the host link, as misses of the gathers.
    # K more superbatches first bring the cache to its steady state.
    more = []
    for k in range(K, 2 * K):
        seeds, so = seed_batches(train, cfg.batch, cfg.S, cfg.seed, first_batch=k * cfg.S)
        more.append((seeds.cuda(), so.numpy(), k * cfg.S))
    del executor
    start = ginex.static_select(cfg.num_nodes, w.indices, cfg.cap)
    cache.init(start)
    carried = ginex.Executor(cache)
    pipe.carry_cache_from(start)
    stats = [0, 0, 0]

    def execute_carried(k, samp, cs):
        carried.run(samp, cs, batch_input, resumed=True)
        torch.cuda.current_stream().synchronize()
        stats[0] += int(samp.totals[2])
        stats[1] += int(cs.miss_count.sum())
        stats[2] += int(samp.totals[0])

    pipe.run_with_executor(sbs, execute_carried, overlap=True)          # towards steady state
    for key, overlap in (("whole_path_carried_cache_sequential", False),
                         ("whole_path_carried_cache_overlapped", True)):
        stats[:] = [0, 0, 0]
        t = pipe.run_with_executor(more, execute_carried, overlap=overlap)
        out[key + "_ms_per_superbatch"] = t * 1e3 / K
        out[key + "_edges_per_s"] = stats[0] / t
        out[key + "_miss_ratio"] = stats[1] / max(stats[2], 1)
    stats[:] = [0, 0, 0]
    t = pipe.run_three_stage(more, execute_carried)
    out["whole_path_carried_cache_three_stage_ms_per_superbatch"] = t * 1e3 / K
    out["whole_path_carried_cache_three_stage_edges_per_s"] = stats[0] / t
    pipe.carry_cache_from(None)
    return out


def neighbor_cache_leg(ginex, w, run):
    """Sampling with the adjacency lists outside HBM (Section 3.2): `indices` in pinned host
    memory, first without, then with a neighbour cache of a fraction of the edges in HBM.
    The sampled result is the same in every row (checked against the all-in-HBM ids)."""
    cfg = w.cfg
    E = w.indices.numel()
    # this leg runs last and needs no features: hand their pinned memory back first
    run.cache = run.executor = run.batch_input = run.ws = None
    w.features = None
    import gc
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    if hasattr(torch._C, "_host_emptyCache"):
        torch._C._host_emptyCache()
    ind_host = torch.empty(E, dtype=torch.int32, pin_memory=True)
    ind_host.copy_(w.indices)
    seeds, so, first = run.sbs[0]
    samp = ginex.sample_superbatch(w.offsets, w.indices, seeds, so, cfg.fanout, rng_seed=0,
                                   first_batch_index=first)

    def timed_sample(indices, nc):
        best, res = None, None
        for _ in range(3):
            torch.cuda.synchronize()
            t = time.perf_counter()
            res = ginex.sample_superbatch(w.offsets, indices, seeds, so, cfg.fanout, rng_seed=0,
                                          first_batch_index=first, neighbor_cache=nc)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t
            best = dt if best is None else min(best, dt)
        assert torch.equal(res.ids, samp.ids)
        return best

    io, hs = samp.ids_offsets, samp.hop_sizes
    ends = (io[:-1, None] + hs[:, :-1]).reshape(-1)         # one row fetch per frontier node
    starts = np.repeat(io[:-1], hs.shape[1] - 1)
    lookups = int((ends - starts).sum())
    edges = int(samp.totals[2])
    out = {"edges_in_graph": E, "row_lookups": lookups,
           "all_in_hbm_ms": timed_sample(w.indices, None) * 1e3,
           "host_csr_no_cache_ms": timed_sample(ind_host, None) * 1e3, "caches": []}
    for frac in (0.05, 0.2, 0.5):
        budget = int(E * frac)
        torch.cuda.synchronize()
        t = time.perf_counter()
        nc = ginex.neighbor_cache_build(w.offsets, ind_host, budget)
        torch.cuda.synchronize()
        build_s = time.perf_counter() - t
        cached = torch.cumsum((nc.address_table[samp.ids.long()] >= 0).to(torch.int64), 0)
        cached = torch.cat([cached.new_zeros(1), cached]).cpu().numpy()
        hits = int((cached[ends] - cached[starts]).sum())
        ms = timed_sample(ind_host, nc) * 1e3
        out["caches"].append({"budget_entries": budget, "fraction_of_edges": frac,
                              "cached_nodes": nc.cached_nodes, "used_entries": nc.used_entries,
                              "build_ms": build_s * 1e3, "hit_ratio": hits / max(lookups, 1),
                              "sample_ms": ms, "sample_edges_per_s": edges / (ms * 1e-3)})
        del nc, cached
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--cpu-batches", type=int, default=40,
                    help="batches of the workload the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--legs", default="pressure,carried,allmiss",
                    help="comma-separated extra legs timed in the same run (pressure, carried, "
                         "allmiss), or 'none'")
    ap.add_argument("--pressure-divisor", type=int, default=16,
                    help="cache of the pressure leg = distinct rows of the superbatch / this")
    ap.add_argument("--pipeline", type=int, default=0, metavar="K",
                    help="also run K superbatches through the superbatch-level pipeline "
                         "(changeset of k under the sampling of k+1) and report the overlap")
    ap.add_argument("--streamed-init", action="store_true",
                    help="also time the step with the main loop started under the cache "
                         "initialization (Executor(streamed=True))")
    ap.add_argument("--neighbor-cache", action="store_true",
                    help="also sample with the adjacency lists in pinned host memory, without and "
                         "with a neighbour cache in HBM")
    ap.add_argument("--allhit", action="store_true",
                    help="also time the gather kernel with the whole feature table in HBM")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    legs = set() if args.legs == "none" else set(args.legs.split(","))
    unknown = legs - {"pressure", "carried", "allmiss"}
    if unknown or args.steps < 1 or args.warmup < 0:
        print(f"bench.py: bad arguments (unknown legs {sorted(unknown)}, steps {args.steps}, "
              f"warmup {args.warmup})", file=sys.stderr)
        sys.exit(2)

    import paper_2208_09151_amd as ginex
    from workload import make_workload
    from workload.configs import seed_batches, train_nodes

    t = time.perf_counter()
    log(f"building workload {args.config} on the GPU ...")
    w = make_workload(args.config, device="cuda", verbose=True)
    cfg = w.cfg
    torch.cuda.synchronize()
    log(f"workload ready in {time.perf_counter() - t:.1f}s: N={cfg.num_nodes} "
        f"E={w.indices.numel()} F={cfg.feat_dim} S={cfg.S} cap={cfg.cap}")
    # consecutive superbatches: warm-up and timed steps take different ones, and the carried
    # leg continues the sequence
    step_sbs = args.warmup + args.steps
    n_sb = step_sbs + (6 if "carried" in legs else 0)
    train = train_nodes(cfg.num_nodes, cfg.train_frac, cfg.seed, device="cuda")
    sbs = []
    for k in range(n_sb):
        seeds, so = seed_batches(train, cfg.batch, cfg.S, cfg.seed, first_batch=k * cfg.S)
        sbs.append((seeds.cuda(), so.numpy(), k * cfg.S))
    del train
    run = Runner(ginex, w, sbs)

    for i in range(args.warmup):
        t = time.perf_counter()
        run.step(i)
        log(f"warmup step {i}: {time.perf_counter() - t:.3f}s")
    timers = {k: [] for k in ("sample_s", "changeset_s", "cache_init_s", "gather_update_s",
                              "executor_s", "edges", "accesses", "misses", "changes",
                              "init_rows")}
    gather_ms = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run.step(args.warmup + i, timers, gather_ms)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    samp, cs = run.last
    S = run.S
    row_bytes = cfg.feat_dim * 4
    edges_total = int(np.sum(timers["edges"]))
    accesses_total = int(np.sum(timers["accesses"]))
    misses_total = int(np.sum(timers["misses"]))
    edges, accesses = med(timers["edges"]), med(timers["accesses"])
    mid = {k: med(timers[k]) for k in ("sample_s", "changeset_s", "cache_init_s",
                                       "gather_update_s", "executor_s")}
    step_s = elapsed / args.steps
    launches = len(gather_ms)
    g_ms = float(np.mean(gather_ms))            # average launch duration over the timed region
    rows_per_launch = accesses_total / launches
    miss_per_launch = misses_total / launches
    # algorithmic bytes of one gather launch: id + resolved line + row in + row out
    algo_bytes = rows_per_launch * (4 + 4 + 2 * row_bytes)
    all_hit = misses_total == 0
    roof = {
        "kernel": "k_gather_lines (" + ("G1: every row resident in the HBM cache"
                                        if all_hit else "real hit/miss mix") + ")",
        "bound": "hbm", "achieved": algo_bytes / (g_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS,
        "unit": "GB/s", "traffic": measured_traffic(cfg.name, "k_gather_lines"),
        "avg_launch_ms": g_ms, "median_launch_ms": med(gather_ms), "launches": launches,
        "rows_per_launch": rows_per_launch, "algorithmic_bytes_per_launch": algo_bytes,
        "miss_fraction": misses_total / max(accesses_total, 1),
        "host_link_GBps": miss_per_launch * row_bytes / (g_ms * 1e-3) / 1e9,
    }
    roof["frac"] = roof["achieved"] / roof["peak"]
    if all_hit and int(np.sum(timers["changes"])) == 0:
        # The same S launches of the last step once more, back to back inside ONE pair of
        # events: the per-launch pairs above put two event markers between consecutive kernels,
        # and each interval includes its share of them.
        io = samp.ids_offsets
        ids_p, lines_p = samp.ids.data_ptr(), cs.src_line.data_ptr()
        out_p = run.batch_input.data_ptr()
        stream_p = torch.cuda.current_stream().cuda_stream
        a, b = event(), event()
        torch.cuda.synchronize()
        a.record()
        for i in range(S):
            run.cache.gather_lines_raw(ids_p + 4 * int(io[i]), lines_p + 4 * int(io[i]),
                                       int(io[i + 1] - io[i]), 0, out_p, stream_p)
        b.record()
        torch.cuda.synchronize()
        bb_ms = a.elapsed_time(b) / S
        bb_rows = float(io[S]) / S
        # This is the launch duration the roofline is priced with (it is the one that agrees
        # with the kernel time rocprofv3 reports); the event-pair figures stay beside it.
        roof.update({
            "event_pairs_avg_launch_ms": g_ms, "event_pairs_GBps": roof["achieved"],
            "event_pairs_frac": roof["frac"], "event_pairs_launches": launches,
            "avg_launch_ms": bb_ms, "launches": S, "rows_per_launch": bb_rows,
            "algorithmic_bytes_per_launch": bb_rows * (4 + 4 + 2 * row_bytes),
            "timing": "one pair of HIP events around the S launches of the last timed "
                      "superbatch, issued back to back; event_pairs_*: a pair around every "
                      "launch of the timed steps (two event markers between kernels)",
        })
        roof["achieved"] = roof["algorithmic_bytes_per_launch"] / (bb_ms * 1e-3) / 1e9
        roof["frac"] = roof["achieved"] / roof["peak"]
    # By wall time the largest kernel of a step is the cache fill, which neither HBM nor the
    # ALUs bound: every row of C_0 crosses the host link once (PCIe Gen5 x16, 64 GB/s raw).
    init_rows = med(timers["init_rows"])
    fill_GBps = init_rows * row_bytes / max(mid["cache_init_s"], 1e-9) / 1e9
    link_roof = {"kernel": "k_cache_fill", "bound": "host link", "achieved": fill_GBps,
                 "peak": HOST_LINK_GBPS, "unit": "GB/s", "frac": fill_GBps / HOST_LINK_GBPS,
                 "avg_launch_ms": mid["cache_init_s"] * 1e3, "rows_per_launch": init_rows}
    # Sampling: random 4-byte neighbour reads and 8-byte table slots, each behind a 128-byte
    # line; the honest ceiling is the rate at which HBM delivers that many lines.
    eps = edges / mid["sample_s"]
    sector_bound = HBM_PEAK_GBPS * 1e9 / (LINE_BYTES * SAMPLER_LINES_PER_EDGE)
    samp_traffic = measured_traffic(cfg.name, "ginex_sample_superbatch")
    samp_roof = {"kernel": "ginex_sample_superbatch (all kernels of the call)",
                 "bound": "hbm, random 128-byte lines",
                 "edges_per_s": eps, "achieved": eps * SAMPLER_BYTES_PER_EDGE / 1e9,
                 "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                 "frac_of_peak_by_algorithmic_bytes": eps * SAMPLER_BYTES_PER_EDGE / 1e9 / HBM_PEAK_GBPS,
                 "algorithmic_bytes_per_edge": SAMPLER_BYTES_PER_EDGE,
                 "line_bytes": LINE_BYTES, "lines_per_edge": SAMPLER_LINES_PER_EDGE,
                 "sector_roofline_edges_per_s": sector_bound, "frac": eps / sector_bound,
                 "traffic": samp_traffic,
                 "counter_bytes_per_edge": samp_traffic / edges if samp_traffic else None,
                 "counter_GBps": samp_traffic / mid["sample_s"] / 1e9 if samp_traffic else None,
                 "call_ms": mid["sample_s"] * 1e3}

    stages = {
        "statistic": "median over the timed steps (consecutive, different superbatches), HIP events",
        "sample_edges_per_s": eps,
        "sample_ms": mid["sample_s"] * 1e3,
        "changeset_accesses_per_s": accesses / mid["changeset_s"],
        "changeset_ms": mid["changeset_s"] * 1e3,
        "changeset_note": ("every row of the superbatch fits the cache: next-use sort and C_0 only, "
                           "the Belady loop does not run (it does in legs.pressure)"
                           if int(np.sum(timers["changes"])) == 0 and all_hit else
                           "the Belady loop runs in the timed steps"),
        "cache_init_ms": mid["cache_init_s"] * 1e3,
        "cache_init_GBps": fill_GBps,
        "gather_update_ms": mid["gather_update_s"] * 1e3,   # what is left after the fill ends
        "executor_ms": mid["executor_s"] * 1e3,
        "gather_GBps": roof["achieved"],
        "sampled_edges": edges, "accesses": accesses, "misses": med(timers["misses"]),
        "changes": med(timers["changes"]),
    }

    # The timed steps run the executor stage by stage, as the paper does (the whole cache
    # initialization in front of the main loop), which also times the gather kernel by
    # itself.  The same step with the main loop started under the initialization:
    if args.streamed_init:
        run.step(step_sbs - 1, streamed=True)
        st = {k: [] for k in timers}
        gather_streamed = []
        t = time.perf_counter()
        for i in range(args.steps):
            run.step(args.warmup + i, st, gather_streamed, streamed=True)
        torch.cuda.synchronize()
        streamed_step_s = (time.perf_counter() - t) / args.steps
        stages["streamed_init"] = {
            "ms_per_step": streamed_step_s * 1e3,
            "edges_per_s": edges_total / args.steps / streamed_step_s,
            "cache_init_ms": med(st["cache_init_s"]) * 1e3,
            "executor_ms": med(st["executor_s"]) * 1e3,
            "after_init_ms": med(st["gather_update_s"]) * 1e3,
            "gather_avg_launch_ms_beside_the_fill": float(np.mean(gather_streamed)),
        }
        samp, cs = run.last

    if args.allhit:
        # the same kernel on the same ids with every row in HBM (pure HBM number)
        free, _ = torch.cuda.mem_get_info()
        need = w.features.numel() * 4
        if need + (8 << 30) < free:
            hbm_tier = w.features.cuda()
            c2 = ginex.FeatureCache(hbm_tier, cfg.cap)
            c2.init(cs.init_ids)
            io = samp.ids_offsets
            ms = []
            for rep in range(2):
                for i in range(S):
                    a, b = event(), event()
                    a.record()
                    c2.gather(samp.ids[io[i]:io[i + 1]], run.batch_input[:io[i + 1] - io[i]],
                              src_line=cs.src_line[io[i]:io[i + 1]])
                    b.record()
                    if rep:
                        ms.append((a, b))
            torch.cuda.synchronize()
            t_ms = float(np.mean([a.elapsed_time(b) for a, b in ms]))
            one = int(samp.totals[0]) / S * (8 + 2 * row_bytes)
            stages["gather_all_in_hbm_GBps"] = one / (t_ms * 1e-3) / 1e9
            stages["gather_all_in_hbm_frac_of_peak"] = stages["gather_all_in_hbm_GBps"] / HBM_PEAK_GBPS
            stages["gather_all_in_hbm_ms"] = t_ms
            del c2, hbm_tier
        else:
            log("not enough free HBM for the all-in-HBM gather measurement; skipped")

    result = {
        "metric": METRIC,
        "value": edges_total / elapsed,
        "unit": "sampled edges/s (whole hot path: sample + changeset + cache init + S x (gather + update))",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": step_s * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: R-MAT N={cfg.num_nodes} E={w.indices.numel()} "
                               f"feat={cfg.feat_dim}xfp32 (slow tier host-pinned) batch={cfg.batch} "
                               f"fanout={list(cfg.fanout)} S={S} cache_rows={cfg.cap}, "
                               f"{args.steps} consecutive superbatches"},
        "stages": stages,
        "roofline": roof,
        "roofline_cache_fill": link_roof,
        "roofline_sampler": samp_roof,
    }
    leg_out = {}
    if "pressure" in legs:
        log("pressure leg ...")
        leg_out["pressure"], result["roofline_gather_mix"], result["roofline_changeset"] = \
            pressure_leg(ginex, w, run, samp, args.pressure_divisor)
    if "allmiss" in legs:
        log("all-miss gather leg ...")
        result["roofline_gather_all_miss"] = allmiss_leg(ginex, w, run, samp)
    if "carried" in legs:
        log("carried-cache leg ...")
        leg_out["carried"], result["roofline_changeset_carried"] = \
            carried_leg(ginex, w, run, step_sbs)
    result["legs"] = leg_out
    if args.pipeline > 0:
        stages["pipeline"] = pipeline_leg(ginex, w, args.pipeline)
    if args.cpu_batches > 0:
        log("timing the CPU oracle on a bounded sample ...")
        result["cpu_baseline"] = cpu_baseline(w, args.cpu_batches)
    else:
        result["cpu_baseline"] = None
    if args.neighbor_cache:     # last: it gives the feature table's pinned memory back
        stages["neighbor_cache"] = neighbor_cache_leg(ginex, w, run)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
