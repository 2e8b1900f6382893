"""Minibatch preparation loop over the C ABI (binding calls only).

The paper overlaps the stages of minibatch preparation in an asynchronous
pipeline (Sec. 3.3).  On one GPU the stage that sets the pace is the miss fetch
over the host link, so the loop is built to keep the link busy:

  chain stream   lookup(i) -> lists(i) -> hit gather(i) -> miss fetch(i) -> lookup(i+1) ...
                 one queue, so the next lookup starts the moment a fetch ends
                 (a hand-over between streams costs ~20 us here)
  work stream    sample(i+2), map update(i): they run while fetch(i) holds the link;
                 both wait for hit gather(i), so nothing competes with the gather.
                 In write-through mode also lookup(i+1) and lists(i+1), right behind
                 map update(i) (then only the hit gather sits between two fetches); with
                 a staging ring (a host tier of capacity 0) the host then packs batch
                 i+1's miss rows while fetch(i) is still on the link
  sampling stream  only with such a ring or tier: sample(i+2) runs there, so that
                 lookup(i+1) need not queue behind it and the host gets the missed ids
                 at once; every row is then packed before the link is free
  (copy stream)  the tier's own, when its copy-engine transport is on: the packed rows of
                 batch i+1 are copied into device memory right behind those of batch i,
                 and the "miss fetch" on the chain stream is the short kernel that
                 scatters the landed rows

The cache is put in write-through mode (every lookup here is followed by the
insert of all its misses), which makes the FIFO update a map update that needs no
fetched row.  The cache state still advances strictly batch by batch (lookup i,
insert i, lookup i+1, ...), so results do not depend on the overlap.  Sampling
runs up to two batches ahead of the fetch, hence three sampling workspaces.
The host waits only for each sampling call's sizes.
"""
from __future__ import annotations

from typing import Callable, Optional

import numpy as np
import torch

from . import binding as B


class MinibatchPipeline:
    def __init__(self, graph: B.Graph, cache: B.Cache, batch: int, fanouts, row_bytes: int,
                 write_through: bool = True, tier: Optional[B.HostTier] = None, spare_rows: bool = True):
        self.graph = graph
        self.fanouts = tuple(int(f) for f in fanouts)
        self.K = len(self.fanouts)
        self.samplers = [B.Sampler(graph, batch, self.fanouts) for _ in range(3)]
        self.cap = int(min(graph.num_nodes, batch * np.prod([1 + f for f in self.fanouts])))
        self.out_rows = torch.empty((self.cap, row_bytes), dtype=torch.uint8, device="cuda")
        self.out_slot = torch.empty(self.cap, dtype=torch.int32, device="cuda")
        self.miss_pos = torch.empty(self.cap, dtype=torch.int32, device="cuda")
        self.chain = torch.cuda.Stream()          # lookups, hit gathers, miss fetches
        self.work = torch.cuda.current_stream()   # map updates, early lookups, (sampling)
        self.write_through = write_through
        # One spare row position in the cache buffer per id of the largest batch: a batch's new rows then
        # never land on a row the same batch still has to read, and the one-pass output of the staged miss
        # path (copy-engine transport, mode 2) is one launch.  Costs cap * row_bytes of device memory.
        self.spare_rows = spare_rows
        # an early lookup adds two hand-overs between streams: it pays for batches of many thousand ids
        self.early_ok = self.cap >= 65536
        # With early lookups and host threads that pack the miss rows, sampling gets a stream of its
        # own: the next batch's lookup then follows the map update at once instead of queueing behind
        # the sampling of the batch after it, and the host has the missed ids half a millisecond sooner
        # (all rows are then packed before the link is free, and one launch fetches them).
        self.samp_stream = None                   # created when first needed (hardware queues are few)
        self.tier = tier                          # second cache level in host memory (Sec. 3.2.3), or None
        self.last_ids, self.last_n = None, 0      # input nodes of the most recent batch
        self.set_cache(cache)

    def set_cache(self, cache: B.Cache) -> None:
        """`cache` must be new (no insertion yet) when the pipeline gives it spare row positions."""
        self.cache = cache
        if self.spare_rows:
            cache.set_spare_rows(self.cap)
        cache.set_write_through(self.write_through)

    def run(self, seeds_dev: torch.Tensor, rng_seeds, steps: int,
            on_batch: Optional[Callable] = None, first_step: int = 0):
        """Prepare `steps` minibatches; batch i uses seeds_dev[i % len] and rng_seeds[i % len]
        (xor the pass number, so that a second pass over the seeds samples differently).
        on_batch(i, sampled_batch, n, pipeline) is called after lookup_gather(i) and
        insert_fifo(i) have been enqueued; work it enqueues on the chain stream after
        cache.wait_rows(chain) sees batch i's complete outputs (out_slot and miss_pos are
        rewritten by the next batch's lookup, which with a staging ring runs on the work
        stream: whoever needs them beyond on_batch enqueues its reads there).
        first_step offsets the batch numbering (a later pass over the seeds).
        Returns (n_input per batch, n_hit per batch)."""
        nb = seeds_dev.shape[0]
        K, cache, chain, work = self.K, self.cache, self.chain, self.work
        samp = work
        if self.tier is not None and self.write_through and self.early_ok:
            if self.samp_stream is None:
                self.samp_stream = torch.cuda.Stream()
            samp = self.samp_stream
        n_hits = torch.zeros(max(steps, 1), dtype=torch.int64).pin_memory()
        n_list = []
        self.tier_hits = []
        sampled_ev = [torch.cuda.Event() for _ in range(3)]

        def sample(i):
            smp = self.samplers[i % 3]
            b = (first_step + i) % nb
            sb = smp.sample(seeds_dev[b], int(rng_seeds[b]) ^ ((first_step + i) // nb), stream=samp)
            sampled_ev[i % 3].record(samp)
            return sb

        def sizes(i):
            sampled_ev[i % 3].synchronize()
            smp = self.samplers[i % 3]
            status = int(smp.counts_host[B.BGL_COUNTS_LEN - 1])
            if status != 0:
                raise B.BglError(status, "sampling reported an error on the device")
            return int(smp.counts_host[K])

        if samp is not work:
            samp.wait_stream(work)      # the seeds, and whatever the caller enqueued before
        sbs = {0: sample(0)}
        if steps > 1:
            sbs[1] = sample(1)
        for i in range(steps):
            n = sizes(i)
            sb = sbs.pop(i)
            ids = sb.input_nodes(self.cap)
            chain.wait_event(sampled_ev[i % 3])
            if samp is not work:
                work.wait_event(sampled_ev[i % 3])
            if self.tier is None:
                # in write-through mode the map lookup and the lists run early, on the work stream
                cache.lookup_gather(ids, n, self.out_rows, self.out_slot, self.miss_pos,
                                    main_stream=chain, side_stream=chain,
                                    n_hit_ptr=n_hits.data_ptr() + 8 * i,
                                    lookup_stream=work if (self.write_through and self.early_ok) else None)
            else:
                # Blocks until the host tier has served the GPU cache's misses.  The map lookups run
                # early, on the work stream (behind the previous batch's map update), so the host brings
                # this batch's rows in while the previous fetch is on the link.
                early = self.write_through and self.early_ok
                # In write-through mode the call comes in two halves: once the host has the lists its threads
                # pack the rows, and this thread enqueues the map update and the sampling of batch i+2
                # meanwhile (a short batch would otherwise wait for those launches).
                n_hits[i], h2 = cache.lookup_gather_tiered(self.tier, ids, n, self.out_rows, self.out_slot,
                                                           self.miss_pos, main_stream=chain, side_stream=chain,
                                                           lookup_stream=work if early else None,
                                                           begin_only=self.write_through)
                self.tier_hits.append(h2)
            if self.tier is not None:
                # the map update first: the next lookup is waiting for it
                cache.insert_fifo(ids, self.miss_pos, -1, self.out_rows, stream=work)
            if i + 2 < steps:
                # workspace (i+2) % 3 was batch i-1's; its fetch ended before hit gather(i)
                cache.wait_lists(samp)
                sbs[i + 2] = sample(i + 2)
            if self.tier is not None and self.write_through:
                cache.lookup_tiered_finish()
            if self.tier is None:
                cache.insert_fifo(ids, self.miss_pos, -1, self.out_rows, stream=work)
            n_list.append(n)
            self.last_ids, self.last_n = ids, n
            if on_batch is not None:
                on_batch(i, sb, n, self)
        torch.cuda.synchronize()
        return n_list, [int(x) for x in n_hits[:steps]]


class NativePipeline:
    """The same loop as one call into the library (bgl_pipeline_run): write-through mode only.  Same
    attributes and run() as MinibatchPipeline; the buffers are torch tensors handed to the library."""

    def __init__(self, graph: B.Graph, cache: B.Cache, batch: int, fanouts, row_bytes: int,
                 tier: Optional[B.HostTier] = None, spare_rows: bool = True):
        import ctypes as C
        self.graph, self.cache = graph, cache
        self.batch = int(batch)
        self.fanouts = np.ascontiguousarray([int(f) for f in fanouts], dtype=np.int32)
        self.K = len(self.fanouts)
        self.samplers = [B.Sampler(graph, batch, self.fanouts) for _ in range(3)]   # workspaces and counts blocks
        self.cap = int(min(graph.num_nodes, batch * np.prod([1 + int(f) for f in self.fanouts])))
        self.out_rows = torch.empty((self.cap, row_bytes), dtype=torch.uint8, device="cuda")
        self.out_slot = torch.empty(self.cap, dtype=torch.int32, device="cuda")
        self.miss_pos = torch.empty(self.cap, dtype=torch.int32, device="cuda")
        self.write_through = True
        self.spare_rows = spare_rows
        self.early_ok = self.cap >= 65536
        self.work = torch.cuda.current_stream()
        buf = B.PipelineBuffers()
        for k, smp in enumerate(self.samplers):
            buf.workspace[k] = smp.workspace.data_ptr()
            buf.counts_host[k] = smp.counts_host.data_ptr()
        buf.workspace_bytes = self.samplers[0].workspace_bytes
        buf.out_rows, buf.out_slot, buf.miss_pos = (self.out_rows.data_ptr(), self.out_slot.data_ptr(),
                                                    self.miss_pos.data_ptr())
        buf.cap_rows = self.cap
        h = C.c_void_p()
        B._check(B.lib().bgl_pipeline_create(graph._h, cache._h, None if tier is None else tier._h, self.batch,
                                             self.fanouts.ctypes.data, self.K, C.byref(buf), 1 if spare_rows else 0,
                                             B._stream_handle(self.work), C.byref(h)))
        self._h = h
        self._tier = tier
        chain = C.c_void_p()
        B._check(B.lib().bgl_pipeline_streams(self._h, C.byref(chain), None))
        self.chain = torch.cuda.ExternalStream(chain.value or 0)
        self.tier_hits = []
        self.last_ids, self.last_n = None, 0

    def set_cache(self, cache: B.Cache) -> None:
        """`cache` must be new (no insertion yet) when the pipeline gives it spare row positions."""
        B._check(B.lib().bgl_pipeline_set_cache(self._h, cache._h, 1 if self.spare_rows else 0))
        self.cache = cache

    @property
    def tier(self):
        return self._tier

    @tier.setter
    def tier(self, tier):
        B._check(B.lib().bgl_pipeline_set_tier(self._h, None if tier is None else tier._h))
        self._tier = tier

    def run(self, seeds_dev: torch.Tensor, rng_seeds, steps: int,
            on_batch: Optional[Callable] = None, first_step: int = 0):
        import ctypes as C
        nb = seeds_dev.shape[0]
        seeds_dev = seeds_dev.contiguous()
        rng = np.ascontiguousarray(rng_seeds, dtype=np.uint64)
        n_input = np.zeros(max(steps, 1), dtype=np.int64)
        n_hit = torch.zeros(max(steps, 1), dtype=torch.int64).pin_memory()
        n_tier = np.zeros(max(steps, 1), dtype=np.int64)
        raised = []

        def hook(_user, i, k, sg, n):
            if raised:
                return
            try:
                st = B.SubgraphStruct()
                C.memmove(C.byref(st), sg, C.sizeof(st))
                sb = B.SampledBatch(self.samplers[k], st)
                self.last_ids, self.last_n = sb.input_nodes(self.cap), int(n)
                on_batch(int(i), sb, int(n), self)
            except BaseException as e:       # (an exception cannot cross the C frames: it is raised afterwards)
                raised.append(e)

        cb = B.BATCH_FN(hook) if on_batch is not None else C.cast(None, B.BATCH_FN)
        B._check(B.lib().bgl_pipeline_run(self._h, B._dev_ptr(seeds_dev, torch.int32), nb, rng.ctypes.data, steps,
                                          first_step, n_input.ctypes.data, n_hit.data_ptr(), n_tier.ctypes.data, cb, None))
        if raised:
            raise raised[0]
        self.tier_hits = [int(x) for x in n_tier[:steps]] if self._tier is not None else []
        ids, n = C.c_void_p(), C.c_int64()
        B._check(B.lib().bgl_pipeline_last_batch(self._h, C.byref(ids), C.byref(n)))
        if ids.value:
            for smp in self.samplers:       # the ids are a view into the workspace that holds them
                off = ids.value - smp.workspace.data_ptr()
                if 0 <= off < smp.workspace_bytes:
                    self.last_ids = smp.workspace[off: off + 4 * self.cap].view(torch.int32)
            self.last_n = int(n.value)
        return [int(x) for x in n_input[:steps]], [int(x) for x in n_hit[:steps]]

    def close(self):
        if getattr(self, "_h", None):
            B._check(B.lib().bgl_pipeline_destroy(self._h))
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
