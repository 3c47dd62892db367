"""Sensitivity sweeps on the synthetic workloads (the paper's Section 5.4 questions, asked of
this build): how sampling, changeset precomputation and gather respond to batch size,
superbatch size, cache size and feature dimension.  Prints markdown tables.

  python -m paper_2208_09151_amd.sweeps [--config 3]

Only the binding is called.  The policy tables put Belady's changesets next to LRU
changesets (ginex_changeset_lru) and a static cache of the highest out-degree rows (the two
policies the paper compares with, Section 2.3 and Figures 2 and 5).  The static selection is
ginex_static_select and its misses are counted from the address table by
ginex_cache_count_misses (in the first table over a dummy slow tier of 16-byte rows, since
only the address table matters there); in the last table all three policies run through the
same executor (cache initialization, then S gathers with their changesets; a static cache
has none), the static misses being counted before the timed loop.
"""
from __future__ import annotations

import argparse
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def timed(fn, reps=3):
    best, out = None, None
    for _ in range(reps):
        torch.cuda.synchronize()
        t = time.perf_counter()
        out = fn()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        best = dt if best is None else min(best, dt)
    return best, out


def main():
    import paper_2208_09151_amd as ginex
    from workload import make_workload
    from workload.configs import seed_batches, train_nodes

    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--no-executor", action="store_true",
                    help="skip the last table (it needs the feature table in host memory)")
    args = ap.parse_args()
    w = make_workload(args.config, device="cuda", features=False)
    cfg = w.cfg
    train = train_nodes(cfg.num_nodes, cfg.train_frac, cfg.seed, device="cuda")
    total_seeds = cfg.batch * cfg.S
    print(f"# Sweeps on {cfg.name}: N={cfg.num_nodes} E={w.indices.numel()} "
          f"fanout={list(cfg.fanout)}, {total_seeds} seeds per superbatch\n")

    def inspect(batch, S, cap):
        seeds, so = seed_batches(train, batch, S, cfg.seed)
        seeds = seeds.cuda()
        ts, samp = timed(lambda: ginex.sample_superbatch(w.offsets, w.indices, seeds, so.numpy(),
                                                         cfg.fanout, rng_seed=0))
        tc, cs = timed(lambda: ginex.changeset(cfg.num_nodes, samp.ids, samp.ids_offsets, cap))
        return ts, tc, samp, cs

    # 1. cache size: Belady against a static highest-out-degree cache
    _, _, samp, _ = inspect(cfg.batch, cfg.S, 1)
    distinct = int(torch.unique(samp.ids).numel())
    accesses = int(samp.totals[0])
    order = ginex.static_select(cfg.num_nodes, w.indices, distinct)   # a smaller cache is a prefix
    dummy_tier = torch.zeros((cfg.num_nodes, 4), dtype=torch.float32, device="cuda")
    print(f"## Cache size (batch {cfg.batch}, S={cfg.S}; {accesses} accesses, {distinct} distinct rows)\n")
    print("| cache rows | % of distinct | Belady miss ratio | LRU miss ratio | static out-degree miss ratio "
          "| Belady changeset ms | G accesses/s | LRU changeset ms |")
    print("|---:|---:|---:|---:|---:|---:|---:|---:|")
    for pct in (1, 2, 5, 10, 20, 50, 100):
        cap = max(1, distinct * pct // 100)
        tc, cs = timed(lambda: ginex.changeset(cfg.num_nodes, samp.ids, samp.ids_offsets, cap))
        tl, lru = timed(lambda: ginex.changeset(cfg.num_nodes, samp.ids, samp.ids_offsets, cap,
                                                policy="lru"))
        static_cache = ginex.FeatureCache(dummy_tier, cap)
        static_cache.init(order[:cap])
        counter = torch.zeros(1, dtype=torch.int64, device="cuda")
        static_cache.count_misses(samp.ids, counter)
        static_miss = int(counter.item())
        del static_cache
        print(f"| {cap} | {pct} | {cs.miss_count.sum() / accesses:.4f} | {lru.miss_count.sum() / accesses:.4f} "
              f"| {static_miss / accesses:.4f} | {tc * 1e3:.2f} | {accesses / tc / 1e9:.2f} | {tl * 1e3:.2f} |")
        del cs, lru

    del dummy_tier
    # 2. batch size at a fixed number of seeds per superbatch
    cap = max(1, distinct // 10)
    print(f"\n## Batch size (seeds per superbatch fixed, cache = {cap} rows = 10% of distinct)\n")
    print("| batch | S | sampled edges | accesses | sample ms | changeset ms | changeset / sample |")
    print("|---:|---:|---:|---:|---:|---:|---:|")
    for batch in (250, 500, 1000, 2000, 4000):
        S = max(1, total_seeds // batch)
        ts, tc, samp_b, _ = inspect(batch, S, cap)
        print(f"| {batch} | {S} | {int(samp_b.totals[2])} | {int(samp_b.totals[0])} | {ts * 1e3:.2f} "
              f"| {tc * 1e3:.2f} | {tc / ts:.2f} |")

    # 3. superbatch size at the configured batch size
    print(f"\n## Superbatch size (batch {cfg.batch}, cache = {cap} rows)\n")
    print("| S | accesses | Belady miss ratio | sample ms | changeset ms | ms per iteration |")
    print("|---:|---:|---:|---:|---:|---:|")
    for S in (cfg.S // 4, cfg.S // 2, cfg.S, cfg.S * 2, cfg.S * 4):
        if S < 1:
            continue
        ts, tc, samp_s, cs_s = inspect(cfg.batch, S, cap)
        acc = int(samp_s.totals[0])
        print(f"| {S} | {acc} | {cs_s.miss_count.sum() / acc:.4f} | {ts * 1e3:.2f} | {tc * 1e3:.2f} "
              f"| {tc * 1e3 / S:.3f} |")

    # 4. feature dimension: the gather kernel with every row in HBM
    print("\n## Feature dimension (gather of one iteration's ids, all rows resident in HBM)\n")
    print("| dim | row bytes | rows | us per launch | algorithmic GB/s | fraction of 8 TB/s |")
    print("|---:|---:|---:|---:|---:|---:|")
    io = samp.ids_offsets
    rows_n = int(io[1] - io[0])
    for dim in (128, 256, 512, 768):
        nodes = min(cfg.num_nodes, (40 << 30) // (dim * 4))     # a 40 GB table at most
        table = torch.empty((nodes, dim), dtype=torch.float32, device="cuda")
        cache = ginex.FeatureCache(table, 1024)
        cache.init(torch.arange(1024, dtype=torch.int32, device="cuda"))
        out = torch.empty((rows_n, dim), dtype=torch.float32, device="cuda")
        ev = []
        for rep in range(40):
            # fresh ids every launch, so that no row is served from the Infinity Cache
            ids = torch.randint(0, nodes, (rows_n,), device="cuda", dtype=torch.int32)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            cache.gather(ids, out)
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        us = float(np.median([a.elapsed_time(b) for a, b in ev[5:]])) * 1e3
        gbps = rows_n * (8 + 2 * dim * 4) / us / 1e3
        print(f"| {dim} | {dim * 4} | {rows_n} | {us:.1f} | {gbps:.0f} | {gbps / 8000:.3f} |")
        del table, cache, out

    # 5. the three policies through the same executor, features in pinned host memory
    if args.no_executor:
        return
    from workload.configs import make_features
    feats = make_features(cfg.num_nodes, cfg.feat_dim, cfg.seed, "cuda")
    row_bytes = cfg.feat_dim * 4
    print(f"\n## Policies through the executor (rows of {row_bytes} B in pinned host memory; "
          f"cache initialization + {cfg.S} gathers with their changesets)\n")
    print("| cache rows | % of distinct | policy | misses | miss ratio | init ms | gathers ms | total ms "
          "| slow-tier GB |")
    print("|---:|---:|---|---:|---:|---:|---:|---:|---:|")
    io = samp.ids_offsets
    longest = int(np.diff(io).max())
    out = torch.empty((longest, cfg.feat_dim), dtype=torch.float32, device="cuda")
    for pct in (5, 20, 50):
        cap = max(1, distinct * pct // 100)
        plans = {
            "Belady": ginex.changeset(cfg.num_nodes, samp.ids, io, cap),
            "LRU": ginex.changeset(cfg.num_nodes, samp.ids, io, cap, policy="lru"),
        }
        cache = ginex.FeatureCache(feats, cap)
        for name in ("Belady", "LRU", "static"):
            cs = plans.get(name)
            init = cs.init_ids if cs is not None else order[:cap].contiguous()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            cache.init(init)
            torch.cuda.synchronize()
            init_s = time.perf_counter() - t0
            misses = torch.zeros(1, dtype=torch.int64, device="cuda")
            if cs is None:      # a static cache never changes: count once, outside the timing
                cache.count_misses(samp.ids, misses)
                torch.cuda.synchronize()
            t1 = time.perf_counter()
            for i in range(cfg.S):
                ids_i = samp.ids[io[i]:io[i + 1]]
                if cs is None:
                    cache.gather(ids_i, out[:ids_i.numel()])
                else:
                    sl = slice(cs.cs_offsets[i], cs.cs_offsets[i + 1])
                    cache.gather(ids_i, out[:ids_i.numel()], cs.in_ids[sl], cs.out_ids[sl],
                                 cs.in_positions[sl])
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            m = int(cs.miss_count.sum()) if cs is not None else int(misses.item())
            print(f"| {cap} | {pct} | {name} | {m} | {m / accesses:.4f} | {init_s * 1e3:.1f} "
                  f"| {(t2 - t1) * 1e3:.1f} | {(init_s + t2 - t1) * 1e3:.1f} "
                  f"| {(m + init.numel()) * row_bytes / 1e9:.2f} |")
        del cache, plans


if __name__ == "__main__":
    main()
