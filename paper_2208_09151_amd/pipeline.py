"""Superbatch-level pipeline (paper Section 3.1 "Superbatch-level Pipeline"): the changeset
precomputation of superbatch k runs while superbatch k+1 is being sampled.

In the paper the two stages sit on different processors (CPU sampling, GPU changesets); here
both are GPU work, so the overlap only fills the gaps each stage leaves (host round trips,
small dependent launches).  Each stage runs on its own HIP stream (default priority) from
its own host thread, with its own workspace and output buffers (double buffering); the
library keeps no global state, and ctypes drops the GIL during the calls.

``run_with_executor`` goes one step further than the paper: the whole inspector of
superbatch k+1 (sampling and changesets, bound by HBM and atomics) runs under the executor
of superbatch k (cache initialization and gathers, bound by the host link).

``Executor`` runs one superbatch through the cache (initialization, then gather and update
per iteration) and can start the main loop under the initialization: C_0 is ordered by
first access, so iteration i needs only a prefix of it.

This module only sequences calls of the binding: no step of the path runs here.
"""
from __future__ import annotations

import threading
import time

import numpy as np
import torch

from . import _lib, api


class Executor:
    """Cache initialization and main loop of one superbatch (paper Section 3.1).

    With ``streamed=True`` the initialization is issued in pieces on a second stream
    (default priority) and the gather of iteration i waits only for the piece that completes
    the rows first accessed up to i (``ChangesetResult.init_ready``).  From the first
    non-empty changeset on, iterations wait for the whole initialization, since an update may
    evict a row that is not loaded yet.  The initialization is bound by the host link, the
    gathers of resident rows by HBM, so the two overlap almost completely."""

    def __init__(self, cache: api.FeatureCache, min_piece_rows: int = 1 << 16,
                 second: api.FeatureCache = None):
        """``second``: another cache of the same shape over the same slow tier.  The two then
        take turns from superbatch to superbatch, and the initialization copies every row the
        previous superbatch's cache still holds from there instead of the slow tier."""
        self.caches = [cache] if second is None else [cache, second]
        self.turn = 0               # caches[turn] takes the next superbatch
        self.warm = False           # the other cache holds a finished superbatch
        self.min_piece_rows = min_piece_rows
        self.fill_stream = torch.cuda.Stream(device=cache.rows.device)
        self.events = []

    @property
    def cache(self):
        """The cache of the superbatch that ran last (or will run first)."""
        return self.caches[self.turn - 1] if self.warm else self.caches[self.turn]

    def _event(self, k):
        while len(self.events) <= k:
            self.events.append(torch.cuda.Event(enable_timing=True))
        return self.events[k]

    def run(self, samp, cs, out, streamed=True, before_gather=None, after_gather=None,
            resumed=False, use_lines=True):
        """``out``: device buffer [>= longest iteration, feat_dim] that receives every batch
        input in turn; ``before_gather(i)`` / ``after_gather(i, n)`` are called right before
        and after the gather kernel of iteration i is enqueued (timing events; the consumer
        enqueues its own work on the current stream in ``after_gather``).  With ``resumed``
        the cache already holds ``cs.init_ids`` line by line (the changesets come from
        ``changeset_resume`` on the state the last superbatch left) and nothing is loaded.
        With ``use_lines`` (and ``cs.src_line`` present) the gathers take their cache lines from
        the changeset stage instead of probing the address table.
        Returns the event that marks the end of the initialization."""
        cache = self.caches[self.turn]
        prev = self.caches[self.turn - 1] if self.warm and len(self.caches) > 1 else None

        def load(begin, end, stream_ptr):
            if prev is not None:
                cache.init_warm_raw(prev, init_ptr, begin, end, stream_ptr)
            else:
                cache.init_part_raw(init_ptr, begin, end, stream_ptr)

        main = torch.cuda.current_stream()
        mp = main.cuda_stream
        io, co = samp.ids_offsets.tolist(), cs.cs_offsets.tolist()
        S = len(io) - 1
        n_init = cs.init_ids.numel()
        ids_base, out_ptr = samp.ids.data_ptr(), out.data_ptr()
        bases = (cs.in_ids.data_ptr(), cs.out_ids.data_ptr(), cs.in_positions.data_ptr())
        init_ptr = cs.init_ids.data_ptr()
        lines_base = cs.src_line.data_ptr() if use_lines and cs.src_line is not None else 0
        slow = cs.miss_count.tolist() if lines_base else None
        wait_for = None
        if resumed:
            self._event(0).record(main)
            cuts = [n_init]
        elif streamed and cs.init_ready is not None and S > 0:
            ready = cs.init_ready.tolist()
            fs = self.fill_stream
            fp = fs.cuda_stream
            fs.wait_stream(main)        # earlier readers of the cache lines are done
            first_change = next((i for i in range(S) if co[i + 1] > co[i]), S)
            need = [ready[i] if i < first_change else n_init for i in range(S)]
            need[S - 1] = n_init
            # pieces end at iteration boundaries and hold at least min_piece_rows rows; the
            # first one is always issued, since it resets the address table
            cuts, done = [], 0
            for i in range(S):
                if i == 0 or need[i] - done >= self.min_piece_rows or \
                        (need[i] == n_init and need[i] > done):
                    load(done, need[i], fp)
                    self._event(len(cuts)).record(fs)
                    done = need[i]
                    cuts.append(done)
            wait_for, k = [0] * S, 0
            for i in range(S):
                while cuts[k] < need[i]:
                    k += 1
                wait_for[i] = k
        else:
            load(0, n_init, mp)
            self._event(0).record(main)
            cuts = [n_init]
        waited = -1
        for i in range(S):
            if wait_for is not None and wait_for[i] > waited:
                waited = wait_for[i]
                main.wait_event(self.events[waited])
            n = io[i + 1] - io[i]
            if before_gather is not None:
                before_gather(i)
            if lines_base:
                cache.gather_lines_raw(ids_base + 4 * io[i], lines_base + 4 * io[i], n, slow[i],
                                       out_ptr, mp)
            else:
                cache.gather_raw(ids_base + 4 * io[i], n, out_ptr, mp)
            if after_gather is not None:
                after_gather(i, n)
            nc = co[i + 1] - co[i]
            if nc:
                cache.update_raw(out_ptr, bases[0] + 4 * co[i], bases[1] + 4 * co[i],
                                 bases[2] + 4 * co[i], nc, mp)
        if len(self.caches) > 1 and not resumed:
            self.turn = 1 - self.turn
            self.warm = True
        return self.events[len(cuts) - 1]


class InspectorPipeline:
    def __init__(self, offsets, indices, num_nodes, fanout, cap, max_batch, S):
        lib = _lib.load()
        self.offsets, self.indices = offsets, indices
        self.num_nodes, self.fanout, self.cap, self.S = num_nodes, tuple(fanout), cap, S
        fo = np.asarray(fanout, dtype=np.int32)
        so = np.arange(S + 1, dtype=np.int64) * max_batch
        ci, cr, cc = api.sample_capacity(num_nodes, so, fanout)
        dev = offsets.device
        ws_s = lib.ginex_sample_workspace_bytes(num_nodes, S, max_batch, fo.ctypes.data, len(fo))
        ws_c = lib.ginex_changeset_workspace_bytes(num_nodes, ci, S, cap)
        self.ws_sample = torch.empty(ws_s, dtype=torch.uint8, device=dev)
        self.ws_changeset = torch.empty(ws_c, dtype=torch.uint8, device=dev)
        # two sets of sampler outputs: one being filled while the other is consumed (a third
        # one is added by run_three_stage)
        self.bufs = [(torch.empty(ci, dtype=torch.int32, device=dev),
                      torch.empty(cr, dtype=torch.int64, device=dev),
                      torch.empty(cc, dtype=torch.int32, device=dev)) for _ in range(2)]
        self.streams = (torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev))
        self.state = None

    def _sample(self, k, seeds, seed_offsets, first_batch, rng_seed, nbuf=2):
        with torch.cuda.stream(self.streams[0]):
            return api.sample_superbatch(self.offsets, self.indices, seeds, seed_offsets, self.fanout,
                                         rng_seed=rng_seed, first_batch_index=first_batch,
                                         workspace=self.ws_sample, out=self.bufs[k % nbuf])

    def carry_cache_from(self, start_ids):
        """From now on every superbatch starts from the cache state the one before it left
        (``changeset_resume``); ``start_ids`` (device int32 [cap]) is what the cache holds
        now, line by line.  ``None`` goes back to a fresh prefetch per superbatch."""
        self.state = start_ids

    def _changeset(self, samp):
        with torch.cuda.stream(self.streams[1]):
            if self.state is not None:
                cs = api.changeset_resume(self.num_nodes, samp.ids, samp.ids_offsets, self.state,
                                          workspace=self.ws_changeset)
                self.state = cs.final_ids
                return cs
            return api.changeset(self.num_nodes, samp.ids, samp.ids_offsets, self.cap,
                                 workspace=self.ws_changeset)

    def run(self, superbatches, rng_seed=0, mode="overlap", consume=None):
        """``superbatches``: list of (seeds device tensor, seed_offsets host array, first global
        batch index).  ``mode``: "overlap" (changeset of k under the sampling of k+1),
        "sequential" (one after the other) or "sample_only".  ``consume(k, samp, cs)`` is
        called once superbatch k is inspected and before its buffers go back to the sampler
        (the executor would run there); results are only valid inside that call.
        Returns the wall time in seconds."""
        if mode not in ("overlap", "sequential", "sample_only"):
            raise ValueError(mode)
        box = {}

        def sample(k):
            try:
                box["samp"] = self._sample(k, *superbatches[k], rng_seed)
            except BaseException as e:      # re-raised on the calling thread
                box["error"] = e

        n = len(superbatches)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        sample(0)
        for k in range(n):
            if "error" in box:
                raise box["error"]
            samp, cs = box["samp"], None
            if mode == "overlap" and k + 1 < n:
                th = threading.Thread(target=sample, args=(k + 1,))
                th.start()
                try:
                    cs = self._changeset(samp)
                finally:
                    th.join()
                if consume:
                    consume(k, samp, cs)
            else:
                if mode != "sample_only":
                    cs = self._changeset(samp)
                if consume:
                    consume(k, samp, cs)
                if k + 1 < n:
                    sample(k + 1)
        if "error" in box:
            raise box["error"]
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def inspect(self, k, seeds, seed_offsets, first_batch, rng_seed=0):
        """Sampling then changesets of one superbatch on the inspector streams."""
        samp = self._sample(k, seeds, seed_offsets, first_batch, rng_seed)
        return samp, self._changeset(samp)

    def run_three_stage(self, superbatches, execute, rng_seed=0):
        """Three stages in flight: sampling of superbatch k+2, changesets of k+1 and
        ``execute(k, samp, cs)`` (on the calling thread), each stage on its own host thread
        and streams, with three sets of sampler outputs.  Worth it when no stage dominates
        (a cache carried over: sampling, the changeset loop and the executor are of the same
        order).  ``execute`` must have finished its GPU work when it returns (synchronize the
        stream it used): right after it returns the sampler may overwrite the ids and adj
        buffers of that superbatch, and the changeset tensors, which were allocated on the
        inspector's stream, may be freed and reused.  Returns the wall time in seconds."""
        import queue
        while len(self.bufs) < 3:
            self.bufs.append(tuple(torch.empty_like(t) for t in self.bufs[0]))
        n = len(superbatches)
        free_bufs = threading.Semaphore(3)
        sampled, inspected = queue.Queue(), queue.Queue()
        errors = []

        def sample_all():
            try:
                for k in range(n):
                    free_bufs.acquire()
                    if errors:
                        break
                    sampled.put((k, self._sample(k, *superbatches[k], rng_seed, nbuf=3)))
            except BaseException as e:      # re-raised on the calling thread
                errors.append(e)
            finally:
                sampled.put(None)

        def inspect_all():
            try:
                while True:
                    item = sampled.get()
                    if item is None:
                        break
                    k, samp = item
                    inspected.put((k, samp, self._changeset(samp)))
            except BaseException as e:
                errors.append(e)
            finally:
                inspected.put(None)

        torch.cuda.synchronize()
        t0 = time.perf_counter()
        threads = [threading.Thread(target=sample_all), threading.Thread(target=inspect_all)]
        for th in threads:
            th.start()
        try:
            while True:
                item = inspected.get()
                if item is None:
                    break
                execute(*item)
                free_bufs.release()
        except BaseException as e:
            errors.append(e)
        finally:
            for _ in range(n + 3):          # let a sampler that waits for a buffer run out
                free_bufs.release()
            # drain so that neither producer blocks (the queues are unbounded; this only
            # matters after an error on this thread)
            for th in threads:
                th.join()
        if errors:
            raise errors[0]
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def run_with_executor(self, superbatches, execute, rng_seed=0, overlap=True):
        """Two-stage pipeline over superbatches: ``execute(k, samp, cs)`` (cache init,
        gathers, updates; it must finish its GPU work before returning) runs on the calling
        thread while, with ``overlap``, the inspector of superbatch k+1 runs on a second
        thread and its own streams.  Returns the wall time in seconds."""
        box = {}

        def inspect(k):
            try:
                box["next"] = self.inspect(k, *superbatches[k], rng_seed)
            except BaseException as e:
                box["error"] = e

        n = len(superbatches)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        inspect(0)
        for k in range(n):
            if "error" in box:
                raise box["error"]
            samp, cs = box["next"]
            th = None
            if k + 1 < n:
                if overlap:
                    th = threading.Thread(target=inspect, args=(k + 1,))
                    th.start()
            try:
                execute(k, samp, cs)
            finally:
                if th is not None:
                    th.join()
            if k + 1 < n and not overlap:
                inspect(k + 1)
        if "error" in box:
            raise box["error"]
        torch.cuda.synchronize()
        return time.perf_counter() - t0
