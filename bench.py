#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

A step is one pass of the inspector-executor path over one superbatch:
  ginex_sample_superbatch -> ginex_changeset -> ginex_cache_init ->
  S x (ginex_gather + ginex_cache_update)
on a synthetic R-MAT workload (default: configuration 4, the 111M-node graph with the
feature table in host-pinned memory).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5]
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
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` from the rocprofv3 --pmc runs recorded under
    profiles/ (FETCH_SIZE and WRITE_SIZE, scaled by the plain-copy calibration), or None
    when no counter run exists for this workload."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)[workload][kernel]
        return rec["fetch_bytes_per_launch"] + rec["write_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


class Runner:
    """Holds every buffer of the path so that steps allocate (almost) nothing."""

    def __init__(self, ginex, w):
        from paper_2208_09151_amd import _lib, api
        self.g, self.w, self.cfg = ginex, w, w.cfg
        cfg = w.cfg
        self.seeds = w.seeds.cuda()
        self.seed_off = w.seed_offsets.numpy()
        self.S = len(self.seed_off) - 1
        lib = _lib.load()
        fo = np.asarray(cfg.fanout, dtype=np.int32)
        max_batch = int(np.max(np.diff(self.seed_off)))
        ws_s = lib.ginex_sample_workspace_bytes(cfg.num_nodes, self.S, max_batch,
                                                fo.ctypes.data, len(fo))
        ci, cr, cc = api.sample_capacity(cfg.num_nodes, self.seed_off, cfg.fanout)
        ws_c = lib.ginex_changeset_workspace_bytes(cfg.num_nodes, ci, self.S, cfg.cap)
        log(f"workspace: sample {ws_s / 2**30:.2f} GiB, changeset {ws_c / 2**30:.2f} GiB")
        # the two stages run one after the other: one workspace serves both
        self.ws = torch.empty(max(ws_s, ws_c), dtype=torch.uint8, device="cuda")
        self.out_bufs = (torch.empty(ci, dtype=torch.int32, device="cuda"),
                         torch.empty(cr, dtype=torch.int64, device="cuda"),
                         torch.empty(cc, dtype=torch.int32, device="cuda"))
        self.cache = ginex.FeatureCache(w.features, cfg.cap)
        self.executor = ginex.Executor(self.cache)
        self.batch_input = None
        self.last = None
        # event pairs around every gather launch, created once: the executor loop must
        # enqueue faster than the GPU drains, or the event pair would also time the host
        ev = torch.cuda.Event
        self.pairs = [(ev(enable_timing=True), ev(enable_timing=True)) for _ in range(self.S)]

    def step(self, timers=None, events=None, streamed=False):
        g, cfg = self.g, self.cfg
        t0 = time.perf_counter()
        samp = g.sample_superbatch(self.w.offsets, self.w.indices, self.seeds, self.seed_off,
                                   cfg.fanout, rng_seed=0, workspace=self.ws, out=self.out_bufs)
        t1 = time.perf_counter()
        cs = g.changeset(cfg.num_nodes, samp.ids, samp.ids_offsets, cfg.cap, workspace=self.ws)
        t2 = time.perf_counter()
        io, co = samp.ids_offsets, cs.cs_offsets
        max_n = int(np.max(np.diff(io)))
        if self.batch_input is None or self.batch_input.shape[0] < max_n:
            self.batch_input = torch.empty((max_n, cfg.feat_dim), dtype=torch.float32, device="cuda")
        ev = torch.cuda.Event
        e_init0, e_end = ev(enable_timing=True), ev(enable_timing=True)
        # the executor: cache initialization in pieces on a second stream and, per iteration,
        # one ginex_gather (one kernel) as soon as the rows it can touch are loaded, then
        # one ginex_cache_update when the changeset is not empty
        pairs = self.pairs if events is not None else None
        before = (lambda i: pairs[i][0].record()) if pairs is not None else None
        after = (lambda i, n: pairs[i][1].record()) if pairs is not None else None
        e_init0.record()
        fill_end = self.executor.run(samp, cs, self.batch_input, streamed=streamed,
                                     before_gather=before, after_gather=after)
        e_end.record()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        if timers is not None:
            timers["sample_s"].append(t1 - t0)
            timers["changeset_s"].append(t2 - t1)
            timers["cache_init_s"].append(e_init0.elapsed_time(fill_end) / 1e3)
            timers["gather_update_s"].append(fill_end.elapsed_time(e_end) / 1e3)
            timers["executor_s"].append(e_init0.elapsed_time(e_end) / 1e3)
            timers["executor_wall_s"].append(t3 - t2)
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


def pressure_leg(ginex, w, run, samp, divisor):
    """The same superbatch with a cache of distinct/divisor rows: every iteration evicts."""
    cfg = w.cfg
    distinct = int(torch.unique(samp.ids).numel())
    cap = max(1, distinct // divisor)
    times = []
    for _ in range(3):
        torch.cuda.synchronize()
        t = time.perf_counter()
        cs = ginex.changeset(cfg.num_nodes, samp.ids, samp.ids_offsets, cap, workspace=run.ws)
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t)
    cache = ginex.FeatureCache(w.features, cap)
    io, co = samp.ids_offsets, cs.cs_offsets
    ev = torch.cuda.Event
    e0, e1, e2 = ev(enable_timing=True), ev(enable_timing=True), ev(enable_timing=True)
    e0.record()
    cache.init(cs.init_ids)
    e1.record()
    for i in range(run.S):
        sl = slice(co[i], co[i + 1])
        cache.gather(samp.ids[io[i]:io[i + 1]], run.batch_input, cs.in_ids[sl], cs.out_ids[sl],
                     cs.in_positions[sl])
    e2.record()
    torch.cuda.synchronize()
    accesses, misses = int(samp.totals[0]), int(cs.miss_count.sum())
    row_bytes = cfg.feat_dim * 4
    loop_s = e1.elapsed_time(e2) / 1e3
    return {"cache_rows": cap, "distinct_rows": distinct, "misses": misses,
            "miss_ratio": misses / accesses, "changes": int(co[-1]),
            "changeset_ms": min(times) * 1e3,
            "changeset_accesses_per_s": accesses / min(times),
            "cache_init_ms": e0.elapsed_time(e1),
            "gather_update_ms": loop_s * 1e3,
            "host_link_GBps": misses * row_bytes / loop_s / 1e9,
            "gather_algorithmic_GBps": accesses * (8 + 2 * row_bytes) / loop_s / 1e9}


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


def neighbor_cache_leg(ginex, w, samp, run):
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
    seeds, so = w.seeds.cuda(), w.seed_offsets.numpy()

    def timed_sample(indices, nc):
        best, res = None, None
        for _ in range(3):
            torch.cuda.synchronize()
            t = time.perf_counter()
            res = ginex.sample_superbatch(w.offsets, indices, seeds, so, cfg.fanout, rng_seed=0,
                                          neighbor_cache=nc)
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
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--cpu-batches", type=int, default=40,
                    help="batches of the workload the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--pipeline", type=int, default=0, metavar="K",
                    help="also run K superbatches through the superbatch-level pipeline "
                         "(changeset of k under the sampling of k+1) and report the overlap")
    ap.add_argument("--pressure", type=int, default=0, metavar="D",
                    help="also run changesets and the executor with a cache of distinct/D rows "
                         "(configurations 3 and 4 never miss with their own cache size)")
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

    import paper_2208_09151_amd as ginex
    from workload import make_workload

    t = time.perf_counter()
    log(f"building workload {args.config} on the GPU ...")
    w = make_workload(args.config, device="cuda", verbose=True)
    cfg = w.cfg
    torch.cuda.synchronize()
    log(f"workload ready in {time.perf_counter() - t:.1f}s: N={cfg.num_nodes} "
        f"E={w.indices.numel()} F={cfg.feat_dim} S={cfg.S} cap={cfg.cap}")
    run = Runner(ginex, w)

    for i in range(args.warmup):
        t = time.perf_counter()
        run.step()
        log(f"warmup step {i}: {time.perf_counter() - t:.3f}s")
    timers = {k: [] for k in ("sample_s", "changeset_s", "cache_init_s", "gather_update_s",
                              "executor_s", "executor_wall_s")}
    gather_ms = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run.step(timers, gather_ms)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    samp, cs = run.last
    S = run.S
    row_bytes = cfg.feat_dim * 4
    edges = int(samp.totals[2])
    accesses = int(samp.totals[0])
    misses = int(cs.miss_count.sum())
    changes = int(cs.cs_offsets[-1])
    mean = {k: float(np.mean(v)) for k, v in timers.items()}
    step_s = elapsed / args.steps
    g_ms = float(np.mean(gather_ms))
    rows_per_launch = accesses / S
    miss_per_launch = misses / S
    # algorithmic bytes of one gather launch: id + address-table entry + row in + row out
    algo_bytes = rows_per_launch * (4 + 4 + 2 * row_bytes)
    roof = {
        "kernel": "k_gather (real hit/miss mix; misses are read from host-pinned memory)",
        "bound": "hbm", "achieved": algo_bytes / (g_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS,
        "unit": "GB/s", "traffic": measured_traffic(cfg.name, "k_gather"),
        "avg_launch_ms": g_ms, "launches": len(gather_ms),
        "rows_per_launch": rows_per_launch, "miss_fraction": misses / max(accesses, 1),
        "host_link_GBps": miss_per_launch * row_bytes / (g_ms * 1e-3) / 1e9,
    }
    roof["frac"] = roof["achieved"] / roof["peak"]
    # By wall time the largest kernel of a step is the cache fill, which neither HBM nor the
    # ALUs bound: every row of C_0 crosses the host link once (PCIe Gen5 x16, 64 GB/s raw).
    fill_GBps = len(cs.init_ids) * row_bytes / mean["cache_init_s"] / 1e9
    link_roof = {"kernel": "k_cache_fill", "bound": "host link", "achieved": fill_GBps,
                 "peak": HOST_LINK_GBPS, "unit": "GB/s", "frac": fill_GBps / HOST_LINK_GBPS,
                 "avg_launch_ms": mean["cache_init_s"] * 1e3, "rows_per_launch": len(cs.init_ids)}

    stages = {
        "sample_edges_per_s": edges / mean["sample_s"],
        "sample_ms": mean["sample_s"] * 1e3,
        "changeset_accesses_per_s": accesses / mean["changeset_s"],
        "changeset_ms": mean["changeset_s"] * 1e3,
        "cache_init_ms": mean["cache_init_s"] * 1e3,
        "cache_init_GBps": len(cs.init_ids) * row_bytes / mean["cache_init_s"] / 1e9,
        "gather_update_ms": mean["gather_update_s"] * 1e3,   # what is left after the fill ends
        "executor_ms": mean["executor_s"] * 1e3,
        "gather_mix_GBps": roof["achieved"],
        "sampled_edges": edges, "accesses": accesses, "misses": misses, "changes": changes,
    }

    # The timed steps run the executor stage by stage, as the paper does (the whole cache
    # initialization in front of the main loop), which also times the gather kernel by
    # itself.  The same step with the main loop started under the initialization:
    if args.streamed_init:
        run.step(streamed=True)
        st = {k: [] for k in timers}
        gather_streamed = []
        t = time.perf_counter()
        for _ in range(args.steps):
            run.step(st, gather_streamed, streamed=True)
        torch.cuda.synchronize()
        streamed_step_s = (time.perf_counter() - t) / args.steps
        stages["streamed_init"] = {
            "ms_per_step": streamed_step_s * 1e3, "edges_per_s": edges / streamed_step_s,
            "cache_init_ms": float(np.mean(st["cache_init_s"])) * 1e3,
            "executor_ms": float(np.mean(st["executor_s"])) * 1e3,
            "after_init_ms": float(np.mean(st["gather_update_s"])) * 1e3,
            "gather_avg_launch_ms_beside_the_fill": float(np.mean(gather_streamed)),
        }

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
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                    c2.gather(samp.ids[io[i]:io[i + 1]], run.batch_input)
                    b.record()
                    if rep:
                        ms.append((a, b))
            torch.cuda.synchronize()
            t_ms = float(np.mean([a.elapsed_time(b) for a, b in ms]))
            stages["gather_all_in_hbm_GBps"] = algo_bytes / (t_ms * 1e-3) / 1e9
            stages["gather_all_in_hbm_frac_of_peak"] = stages["gather_all_in_hbm_GBps"] / HBM_PEAK_GBPS
            stages["gather_all_in_hbm_ms"] = t_ms
            del c2, hbm_tier
        else:
            log("not enough free HBM for the all-in-HBM gather measurement; skipped")

    if args.pipeline > 0:
        stages["pipeline"] = pipeline_leg(ginex, w, args.pipeline)
    if args.pressure > 0:
        stages["pressure"] = pressure_leg(ginex, w, run, samp, args.pressure)

    result = {
        "metric": METRIC,
        "value": edges / step_s,
        "unit": "sampled edges/s (whole hot path: sample + changeset + cache init + S x (gather + update))",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": step_s * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: R-MAT N={cfg.num_nodes} E={w.indices.numel()} "
                               f"feat={cfg.feat_dim}xfp32 (slow tier host-pinned) batch={cfg.batch} "
                               f"fanout={list(cfg.fanout)} S={S} cache_rows={cfg.cap}"},
        "stages": stages,
        "roofline": roof,
        "roofline_cache_fill": link_roof,
    }
    if args.cpu_batches > 0:
        log("timing the CPU oracle on a bounded sample ...")
        result["cpu_baseline"] = cpu_baseline(w, args.cpu_batches)
    else:
        result["cpu_baseline"] = None
    if args.neighbor_cache:     # last: it gives the feature table's pinned memory back
        stages["neighbor_cache"] = neighbor_cache_leg(ginex, w, samp, run)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
