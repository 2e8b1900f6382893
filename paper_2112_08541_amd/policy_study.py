"""Hit ratio against cache size for the policies the paper compares (Sec. 2.3,
Sec. 3.2.1, Sec. 3.2.2): static degree-based, LRU, LFU (host simulators in
csrc/policy_sim.c) and FIFO with random and with proximity-aware seed order (the
library's GPU cache).  Streams of input nodes come from the library's GPU
sampler on a synthetic workload.

    python -m paper_2112_08541_amd.policy_study [--config mid] [--batches 200]

Prints a markdown table.  An analysis tool, not part of the minibatch path.
"""
from __future__ import annotations

import argparse
import ctypes as C
import os
import subprocess
import time

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csrc", "policy_sim.c")
_LIB = os.path.join(_HERE, "libbgl_policy.so")
KINDS = {"static": 0, "lru": 1, "lfu": 2}


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def _sim():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.psim_create.restype = C.c_void_p
        L.psim_create.argtypes = [C.c_int, C.c_int64, C.c_int64]
        L.psim_destroy.argtypes = [C.c_void_p]
        L.psim_static_fill.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        L.psim_batch.restype = C.c_int64
        L.psim_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        _lib = L
    return _lib


class PolicySim:
    """One simulated cache: kind in {"static", "lru", "lfu"}."""

    def __init__(self, kind: str, num_nodes: int, capacity: int, hottest=None):
        self._h = _sim().psim_create(KINDS[kind], num_nodes, capacity)
        if kind == "static":
            hot = np.ascontiguousarray(hottest[:capacity], dtype=np.int32)
            _sim().psim_static_fill(self._h, hot.ctypes.data, len(hot))

    def batch(self, ids: np.ndarray) -> int:
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        return int(_sim().psim_batch(self._h, ids.ctypes.data, len(ids)))

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.psim_destroy(self._h)
            self._h = None


def sample_streams(graph, cfg, seed_batches, rng_seeds):
    """Input-node lists of every batch, sampled on the GPU."""
    import torch
    from . import binding as B
    smp = B.Sampler(graph, cfg.batch, cfg.fanouts)
    seeds_dev = torch.from_numpy(np.ascontiguousarray(seed_batches)).cuda()
    K = len(cfg.fanouts)
    out = []
    for b in range(seed_batches.shape[0]):
        sb = smp.sample(seeds_dev[b], int(rng_seeds[b]))
        torch.cuda.current_stream().synchronize()
        n = int(smp.counts_host[K])
        out.append(sb.input_nodes(n).cpu().numpy())
    return out


def gpu_fifo_hits(streams, num_nodes, capacity, timing=None):
    """Hits of the library's FIFO cache over the batches (16-byte dummy rows: only hits are counted).
    `timing`, a list, receives the mean milliseconds per batch of the calls (lookup + FIFO update with
    rows of 16 bytes: the policy's bookkeeping, Sec. 3.2.1's "overhead", next to no row traffic)."""
    import torch
    from . import binding as B
    feats = torch.zeros((num_nodes, 16), dtype=torch.uint8, device="cuda")
    cache = B.Cache(capacity, feats, num_nodes=num_nodes, row_bytes=16)
    cap = max(len(s) for s in streams)
    out_rows = torch.empty((cap, 16), dtype=torch.uint8, device="cuda")
    out_slot = torch.empty(cap, dtype=torch.int32, device="cuda")
    miss_pos = torch.empty(cap, dtype=torch.int32, device="cuda")
    on_dev = [torch.from_numpy(s).cuda() for s in streams]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for ids in on_dev:
        cache.lookup_gather(ids, len(ids), out_rows, out_slot, miss_pos)
        cache.insert_fifo(ids, miss_pos, -1, out_rows)
    cache.wait_rows()
    e1.record()
    torch.cuda.synchronize()
    if timing is not None:
        timing.append(e0.elapsed_time(e1) / max(len(streams), 1))
    st = cache.stats()
    cache.close()
    assert st["lookups"] == sum(len(s) for s in streams)
    return int(st["hits"])


COLUMNS = ("static", "lru", "lfu", "fifo_random", "fifo_po", "lru_po")


def run_study(cfg, row_ptr, col, num_batches, fractions):
    """The study on one graph: seed orders (random, and proximity-aware from the library's
    bgl_order_proximity), the input nodes of every batch from the library's sampler, and per cache
    size the hits of every policy.  Returns a dictionary with the inputs it drew (train, roots,
    shifts, rng_seeds, both seed orders), the streams, the capacities and `hits[capacity][column]`."""
    from . import binding as B
    N = cfg.num_nodes
    graph = B.Graph(row_ptr, col)
    nb = num_batches
    rng = np.random.default_rng(cfg.seed + 7)
    train = rng.choice(N, max(cfg.train_size, nb * cfg.batch), replace=False).astype(np.int32)
    rng_seeds = rng.integers(0, 2**64, size=nb, dtype=np.uint64)
    roots = rng.integers(0, N, cfg.po_sequences)
    shifts = rng.integers(0, len(train), cfg.po_sequences)
    po = B.order_proximity(graph, train, roots, shifts, nb * cfg.batch).reshape(nb, cfg.batch)
    rnd = rng.permutation(train)[: nb * cfg.batch].reshape(nb, cfg.batch).astype(np.int32)
    streams = {"random": sample_streams(graph, cfg, rnd, rng_seeds),
               "po": sample_streams(graph, cfg, po, rng_seeds)}
    # static cache: the nodes that appear most often as a neighbor, ties by id
    hottest = np.argsort(-np.bincount(col, minlength=N), kind="stable").astype(np.int32)
    hits, overhead_ms, caps = {}, {}, []

    def simulate(kind, cap, which, ms):
        sim = PolicySim(kind, N, cap, hottest)
        t0 = time.perf_counter()
        h = sum(sim.batch(s) for s in streams[which])
        ms.append(1e3 * (time.perf_counter() - t0) / nb)
        return h

    for frac in fractions:
        cap = max(1, int(round(frac * N)))
        caps.append(cap)
        row, ms = {}, {c: [] for c in COLUMNS}
        for kind in ("static", "lru", "lfu"):
            row[kind] = simulate(kind, cap, "random", ms[kind])
        row["fifo_random"] = gpu_fifo_hits(streams["random"], N, cap, ms["fifo_random"])
        row["fifo_po"] = gpu_fifo_hits(streams["po"], N, cap, ms["fifo_po"])
        row["lru_po"] = simulate("lru", cap, "po", ms["lru_po"])
        hits[cap] = row
        overhead_ms[cap] = {c: v[0] for c, v in ms.items()}
    graph.close()
    return dict(train=train, roots=roots, shifts=shifts, rng_seeds=rng_seeds, order_random=rnd, order_po=po,
                streams=streams, hottest=hottest, capacities=caps, hits=hits, overhead_ms=overhead_ms,
                lookups={k: sum(len(s) for s in v) for k, v in streams.items()})


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="mid")
    ap.add_argument("--batches", type=int, default=200)
    ap.add_argument("--fractions", default="0.025,0.05,0.1,0.2,0.4")
    ap.add_argument("--nodes", type=int, default=0, help="run the configuration's shape at this node count")
    ap.add_argument("--p-local", type=float, default=None,
                    help="override the generator's share of edges that stay inside a community")
    ap.add_argument("--batch", type=int, default=0, help="override the number of seeds per batch")
    args = ap.parse_args()
    import torch
    from . import inputs
    cfg = inputs.CONFIGS[args.config]
    if args.nodes:
        cfg = inputs.scaled(cfg, args.nodes)
    import dataclasses
    if args.p_local is not None:
        cfg = dataclasses.replace(cfg, p_local=args.p_local, name=f"{cfg.name},p_local={args.p_local}")
    if args.batch:
        cfg = dataclasses.replace(cfg, batch=args.batch, name=f"{cfg.name},batch={args.batch}")
    t0 = time.time()
    row_ptr, col, _keep = inputs.make_graph(cfg)          # no feature table: only ids matter here
    N = cfg.num_nodes
    nb = min(args.batches, cfg.num_batches)
    fractions = [float(x) for x in args.fractions.split(",")]
    r = run_study(cfg, row_ptr, col, nb, fractions)
    total = r["lookups"]
    print(f"# Cache policy study on the `{cfg.name}` workload ({nb} batches, "
          f"{total['random'] / nb:.0f} input nodes per batch; generated and run in {time.time() - t0:.0f} s)\n")
    print("| cache size (fraction of nodes) | static (in-degree) | LRU | LFU | FIFO, random order | "
          "FIFO, proximity-aware order | LRU, proximity-aware order |")
    print("|---|---|---|---|---|---|---|")
    for frac, cap in zip(fractions, r["capacities"]):
        row = r["hits"][cap]
        ratios = [row[c] / total["po" if c.endswith("_po") else "random"] for c in COLUMNS]
        print(f"| {frac:.3f} ({cap} rows) | " + " | ".join(f"{x:.3f}" for x in ratios) + " |")
    print("\nBookkeeping per batch in milliseconds (lookup + policy update, Sec. 3.2.1's overhead; FIFO columns: the library's "
          "calls on the GPU with 16-byte rows, one after the other on one stream; the others: the host simulators on one core, "
          "O(1) list updates per id):\n")
    print("| cache size | static | LRU | LFU | FIFO, random order | FIFO, proximity-aware order | LRU, proximity-aware order |")
    print("|---|---|---|---|---|---|---|")
    for frac, cap in zip(fractions, r["capacities"]):
        print(f"| {frac:.3f} | " + " | ".join(f"{r['overhead_ms'][cap][c]:.2f}" for c in COLUMNS) + " |")
    torch.cuda.synchronize()


if __name__ == "__main__":
    main()
