"""Two-deep minibatch preparation loop over the C ABI (binding calls only).

The paper overlaps the stages of minibatch preparation in an asynchronous
pipeline (Sec. 3.3); on one GPU that reduces to this: while the misses of batch
i cross the host link on the cache's side stream, batch i+1 is sampled on the
main stream.  The cache state still advances strictly batch by batch
(lookup i, insert i, lookup i+1, ...), so results do not depend on the overlap.

Per batch i, in enqueue order:
  lookup_gather(i)   main: map lookup, miss/hit lists, hit gather; side: miss fetch
  sample(i+1)        main, overlapping the fetch (second sampling workspace)
  insert_fifo(i)     main; in write-through mode (default here) only the map update, which
                     runs under the fetch; otherwise map update, wait for the fetch, row copy
  host waits for sample(i+1)'s sizes only (one event), never for the whole stream
"""
from __future__ import annotations

from typing import Callable, Optional

import numpy as np
import torch

from . import binding as B


class MinibatchPipeline:
    def __init__(self, graph: B.Graph, cache: B.Cache, batch: int, fanouts, row_bytes: int,
                 write_through: bool = True):
        self.graph, self.cache = graph, cache
        # every lookup here is followed by the insert of all its misses, so the miss fetch may
        # fill the cache buffer itself (bgl_cache_set_write_through)
        self.write_through = write_through
        cache.set_write_through(write_through)
        self.fanouts = tuple(int(f) for f in fanouts)
        self.K = len(self.fanouts)
        self.samplers = [B.Sampler(graph, batch, self.fanouts) for _ in range(2)]
        self.cap = int(min(graph.num_nodes, batch * np.prod([1 + f for f in self.fanouts])))
        self.out_rows = torch.empty((self.cap, row_bytes), dtype=torch.uint8, device="cuda")
        self.out_slot = torch.empty(self.cap, dtype=torch.int32, device="cuda")
        self.miss_pos = torch.empty(self.cap, dtype=torch.int32, device="cuda")
        self.side = torch.cuda.Stream()
        self.main = torch.cuda.current_stream()
        self.last_ids, self.last_n = None, 0    # input nodes of the most recent batch

    def set_cache(self, cache: B.Cache) -> None:
        self.cache = cache
        cache.set_write_through(self.write_through)

    def run(self, seeds_dev: torch.Tensor, rng_seeds, steps: int,
            on_batch: Optional[Callable] = None):
        """Prepare `steps` minibatches; batch i uses seeds_dev[i % len] and rng_seeds[i % len]
        (xor the pass number, so that a second pass over the seeds samples differently).
        on_batch(i, sampled_batch, n, pipeline) is called after insert_fifo(i) has been
        enqueued; work it enqueues on the main stream sees batch i's complete outputs.
        Returns (n_input per batch, n_hit per batch)."""
        nb = seeds_dev.shape[0]
        K, cache, main = self.K, self.cache, self.main
        n_list, hit_list = [], []
        smp = self.samplers[0]
        sb = smp.sample(seeds_dev[0], int(rng_seeds[0]))
        main.synchronize()
        n = int(smp.counts_host[K])
        status = int(smp.counts_host[B.BGL_COUNTS_LEN - 1])
        ev = torch.cuda.Event()
        for i in range(steps):
            if status != 0:
                raise B.BglError(status, "sampling reported an error on the device")
            ids = sb.input_nodes(self.cap)
            cache.lookup_gather(ids, n, self.out_rows, self.out_slot, self.miss_pos,
                                main_stream=main, side_stream=self.side)
            nxt = i + 1
            if nxt < steps:
                b = nxt % nb
                smp = self.samplers[nxt % 2]
                sb_next = smp.sample(seeds_dev[b], int(rng_seeds[b]) ^ (nxt // nb), stream=main)
                ev.record(main)
            cache.insert_fifo(ids, self.miss_pos, -1, self.out_rows, stream=main)
            n_list.append(n)
            self.last_ids, self.last_n = ids, n
            if on_batch is not None:
                on_batch(i, sb, n, self)
            if nxt < steps:
                ev.synchronize()      # sizes of batch i+1 and the hit count of batch i are on the host
                hit_list.append(int(cache.n_hit_host[0]))
                n = int(smp.counts_host[K])
                status = int(smp.counts_host[B.BGL_COUNTS_LEN - 1])
                sb = sb_next
        torch.cuda.synchronize()
        hit_list.append(int(cache.n_hit_host[0]))
        return n_list, hit_list
