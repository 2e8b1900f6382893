#!/usr/bin/env python3
"""Benchmark of the minibatch-preparation hot path on one MI355X.

One "step" = one minibatch through the whole path: k-hop neighbor sampling,
cache lookup, gather of the hits from HBM, fetch of the misses from page-locked
host memory, FIFO insertion.  By default all five configurations run, one after
the other, each from an empty cache; the headline is the largest one that fits
one GPU, "large" (111 M nodes, ~1.6 B edges with 64-bit offsets and the CSR in
page-locked host memory, fp32 x 128 features, 1,024 seeds, fanout 15/10/5, cache
of 25 M rows; 200 random-order batches), a synthetic stand-in with the shape of
Ogbn-papers; the others ("wide", "mid" = the shape of Ogbn-products, "bfs",
"tiny") are reported beside it in `configs`.  `--config NAME` runs one of them.

Prints ONE JSON line: the headline value, the roofline of the dominant HBM-bound
kernel (kernel time recorded by the kernel's own dispatch), the host-link rate of
the miss fetch, and the CPU oracle timed on the same box on the same batches.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
LINK_SAMPLE_EVERY = 10          # the miss fetch is timed in every 10th batch of the timed epoch
GATHER_SAMPLE_EVERY = 4         # the hit gather in every 4th
HOST_LINK_NOMINAL_GBS = 64.0   # PCIe Gen5 x16, one direction, nominal


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="all",
                    help="workload preset: tiny, mid, bfs, large, wide, or all (default): all five, one after the "
                         "other, the headline on `large`, the others beside it in `configs`")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stage-timers", action="store_true",
                    help="leave the per-kernel HIP events out of the timed region")
    ap.add_argument("--all-stage-timers", action="store_true",
                    help="bracket every cache kernel with events (default: hit gather and miss fetch only)")
    ap.add_argument("--miss-path", choices=("auto", "trial", "zero_copy", "staged", "staged_scatter", "staged_kernel"), default="auto",
                    help="how miss rows cross the host link: kernels read the page-locked table in place "
                         "(zero_copy), or host threads pack the rows into a page-locked ring (no partial 128-byte "
                         "lines on the link) from where plain copies move them into device memory and kernels "
                         "scatter them (staged), or from where the kernels read them over the link themselves "
                         "(staged_kernel); auto = staged when batches are large (65,536 input nodes or more) "
                         "and the box has 8 or more host threads for the packing, else zero_copy; trial = the "
                         "faster of zero_copy and staged in the warm-up")
    ap.add_argument("--no-write-through", action="store_true",
                    help="FIFO update copies the rows after the fetch instead of the fetch filling the cache buffer")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run three plain 1 GiB device-to-device copies (the known-size "
                         "kernel that scales the rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--hit-gather-sweep", action="store_true",
                    help="only time the hit gather of bgl_cache_lookup_gather over row widths, launch sizes and "
                         "hit densities (lookups into a full cache; one JSON line, not the headline metric)")
    ap.add_argument("--graph-placement", choices=("config", "device", "host_pinned", "host_pinned_col"), default="config",
                    help="where the CSR lives: as the configuration says (default), in HBM, in page-locked host "
                         "memory, or column ids in page-locked host memory with the row offsets in HBM")
    ap.add_argument("--feature-placement", choices=("host_pinned", "device"), default="host_pinned",
                    help="where the feature table lives: page-locked host memory (the path this benchmark is "
                         "about, default) or a copy in HBM (then a miss is an HBM gather; context only)")
    ap.add_argument("--pipeline", choices=("native", "python"), default="native",
                    help="the overlapped batch loop: one call into the library (bgl_pipeline_run), or the same loop "
                         "written in Python over the binding (pipeline.py)")
    ap.add_argument("--two-level", type=float, default=-1.0, metavar="FRACTION",
                    help="also time the same batches with a FIFO tier in host memory (this fraction of the "
                         "nodes) between the GPU cache and a feature store in ordinary host memory; "
                         "reported beside the headline, not part of it")
    ap.add_argument("--tier-threads", type=int, default=0, help="copy threads of the staging ring and of that tier (0 = three quarters of min(cores, 16))")
    ap.add_argument("--cpu-batches", type=int, default=200,
                    help="upper limit of the batches the oracle is timed on (it runs the first of the batches the "
                         "GPU leg timed; with --config all at most 100 for the headline configuration and 20 for "
                         "each of the others)")
    return ap.parse_args()


def measure_h2d_peak(torch, nbytes=256 << 20, windows=4):
    """Pinned-memory host-to-device copy rate on this machine (GB/s), the practical
    ceiling of the host link that the miss fetch is compared with.  Every timed copy
    reads another window of the source, so that none is served from the host's caches
    (the miss rows of a batch are not either)."""
    src = torch.empty(windows * nbytes, dtype=torch.uint8).pin_memory()
    src.fill_(1)
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dst.copy_(src[:nbytes], non_blocking=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(windows):
        dst.copy_(src[k * nbytes:(k + 1) * nbytes], non_blocking=True)
    torch.cuda.synchronize()
    return windows * nbytes / (time.perf_counter() - t0) / 1e9


def hit_gather_sweep(torch, np, B):
    """The hit gather through the C ABI on lookups into a full cache, per row width, launch size
    and hit density (all hits, or hits spread among misses as in an epoch).  The backing table is
    in HBM so that the set-up is quick; only the gather kernel is timed (by its own dispatch).
    Before every launch a 512 MiB copy displaces what the caches hold; every launch looks up a
    fresh random id set; the first launch of a case is checked against the table."""
    cases = [  # row_bytes, cache rows, ids per lookup, fraction of them that hit
        (400, 490_000, 426_000, 0.315),      # `mid`: 134 K hits among 426 K ids
        (400, 490_000, 490_000, 1.0),
        (400, 4_000_000, 1_000_000, 1.0),
        (400, 4_000_000, 4_000_000, 1.0),
        (512, 4_000_000, 1_000_000, 1.0),
        (512, 4_000_000, 4_000_000, 1.0),
        (1024, 4_000_000, 285_000, 0.37),    # `wide`: 106 K hits among 285 K ids
        (1024, 4_000_000, 250_000, 1.0),
        (1024, 4_000_000, 1_000_000, 1.0),
        (1024, 4_000_000, 4_000_000, 1.0),
    ]
    flush_a = torch.zeros(512 << 20, dtype=torch.uint8, device="cuda")
    flush_b = torch.empty_like(flush_a)
    out, built = [], {}
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20211208)
    for rb, cap, n, frac in cases:
        if (rb, cap) not in built:
            built.clear()                        # frees the previous table and cache
            torch.cuda.empty_cache()
            nodes = 2 * cap                      # ids >= cap are never inserted: they miss
            table = torch.empty((nodes, rb), dtype=torch.uint8, device="cuda")
            table.view(torch.int32).random_(generator=gen)
            cache = B.Cache(cap, table.data_ptr(), num_nodes=nodes, row_bytes=rb)
            rows = torch.empty((cap, rb), dtype=torch.uint8, device="cuda")
            slot = torch.empty(cap, dtype=torch.int32, device="cuda")
            mpos = torch.empty(cap, dtype=torch.int32, device="cuda")
            ids = torch.arange(cap, dtype=torch.int32, device="cuda")
            cache.lookup_gather(ids, cap, rows, slot, mpos)       # all miss
            cache.insert_fifo(ids, mpos, -1, rows)                 # the cache now holds ids 0 .. cap-1
            built[(rb, cap)] = (table, cache, rows, slot, mpos)
        table, cache, rows, slot, mpos = built[(rb, cap)]
        n_hit = int(round(n * frac))
        reps, hits = 5, 0
        cache.set_profiling(("gather_hit",))     # (re-)enabling resets the timers
        for r in range(reps):
            ids = torch.randperm(cap, device="cuda", generator=gen)[:n_hit].to(torch.int32)
            if n_hit < n:                        # spread the hits among ids that miss
                ids = torch.cat([ids, cap + torch.randperm(cap, device="cuda", generator=gen)[:n - n_hit].to(torch.int32)])
                ids = ids[torch.randperm(n, device="cuda", generator=gen)].contiguous()
            flush_b.copy_(flush_a)
            torch.cuda.synchronize()
            cache.lookup_gather(ids, n, rows, slot, mpos)
            torch.cuda.synchronize()
            hits += int(cache.n_hit_host[0])
            if r == 0:
                assert int(cache.n_hit_host[0]) == n_hit
                sample = torch.randperm(n, device="cuda", generator=gen)[:65536]
                assert torch.equal(rows[sample], table[ids[sample].long()]), "gathered rows differ from the table"
        ms, launches = cache.profile()["gather_hit"]
        gbps = 2.0 * rb * hits / (ms * 1e-3) / 1e9
        out.append({"row_bytes": rb, "cache_rows": cap, "cache_buffer_MB": cap * rb / 1e6, "ids_per_lookup": n,
                    "hits_per_lookup": n_hit, "bytes_per_launch": 2.0 * rb * n_hit, "launches": launches,
                    "avg_launch_us": 1e3 * ms / launches, "achieved_GBps": gbps, "frac_of_hbm_peak": gbps / HBM_PEAK_GBS})
    return {"hit_gather_sweep": out, "kernel": "k_gather_hits", "peak_GBps": HBM_PEAK_GBS,
            "bytes": "2 x row_bytes x hits (algorithmic: every hit row read once and written once)",
            "timing": "begin/end of each kernel recorded on the device by its own dispatch"}


def frac_in_lines(rb, hits, misses, assembled, write_through):
    """Bytes the dominant kernel moves when every access is counted in whole 128-byte lines (what the
    memory system moves): a row read at a random slot of the cache buffer touches every line it overlaps,
    streams (the landed rows, the assembled output, the run of slots the misses go to) touch exactly
    their bytes."""
    def lines(off_step):
        # mean 128-byte lines touched by a row of rb bytes that starts at a multiple of off_step
        import math
        g = math.gcd(off_step, 128)
        offs = range(0, 128, g)
        return sum(((o % 128) + rb + 127) // 128 for o in offs) / len(offs) * 128
    row_lines = lines(rb)
    if assembled:
        return hits * (row_lines + rb) + misses * (3.0 if write_through else 2.0) * rb
    return hits * 2.0 * row_lines            # hit rows land between miss rows that another kernel writes later


def run_config(cfg, args, torch, np, B, inputs, MinibatchPipeline, want_cpu):
    """One configuration: generate its inputs, warm up on a scratch cache, time `steps` minibatches of the
    whole path from an empty cache, then the side measurements.  Returns the result dictionary."""
    def library_order(row_ptr, col, train, roots, shifts, num_out):
        # the proximity-aware seed order (Sec. 3.2.2) of such a configuration comes from the library itself
        g = B.Graph(row_ptr, col)
        order = B.order_proximity(g, train, roots, shifts, num_out)
        g.close()
        return order

    w = inputs.make_workload(cfg, pinned=True, order_fn=library_order if cfg.order == "po" else None)
    feat_t = w.features.ctypes.data      # address of the page-locked feature table
    feat_dev = None
    if args.feature_placement == "device":
        feat_dev = torch.empty((cfg.num_nodes, cfg.row_bytes), dtype=torch.uint8, device="cuda")
        step = max(1, (1 << 30) // cfg.row_bytes)
        fb = w.features.view(np.uint8).reshape(cfg.num_nodes, cfg.row_bytes)
        for lo in range(0, cfg.num_nodes, step):
            feat_dev[lo:lo + step].copy_(torch.from_numpy(fb[lo:lo + step]))
        feat_t = feat_dev.data_ptr()
    where = cfg.graph_placement if args.graph_placement == "config" else args.graph_placement
    placement = {"host_pinned": B.BGL_HOST_PINNED, "host_pinned_col": B.BGL_HOST_PINNED_COL}.get(where, B.BGL_DEVICE)
    graph = B.Graph(w.row_ptr, w.col, placement)
    seeds_dev = torch.from_numpy(w.seed_batches).cuda()      # inputs resident in HBM
    nb = cfg.num_batches
    steps = min(args.steps, nb) if args.steps_capped else args.steps

    def new_cache():
        return B.Cache(cfg.cache_rows, feat_t, num_nodes=cfg.num_nodes, row_bytes=cfg.row_bytes)

    # warm-up on a scratch cache of the same size, so the timed epoch starts from an empty cache
    scratch = new_cache()
    if args.pipeline == "native" and not args.no_write_through:
        # the overlapped loop as one call into the library (bgl_pipeline_run); same calls, same streams
        from paper_2112_08541_amd.pipeline import NativePipeline
        pipe = NativePipeline(graph, scratch, cfg.batch, cfg.fanouts, cfg.row_bytes)
    else:
        pipe = MinibatchPipeline(graph, scratch, cfg.batch, cfg.fanouts, cfg.row_bytes,
                                 write_through=not args.no_write_through)
    # Miss path.  Staging pays when batches are large (a quarter more for rows that are not multiples
    # of 128 bytes, a few per cent otherwise: the link never waits for the hit gather), provided the
    # box has the host cores for the copy threads (with 3 of them zero-copy was the faster path):
    # "auto" decides by that rule, "trial" times both in the warm-up (each from an empty scratch
    # cache, untimed for the benchmark) and keeps the faster one.
    miss_path = args.miss_path
    host_threads = args.tier_threads or max(1, min(os.cpu_count() or 2, 16) * 3 // 4)
    eligible = pipe.cap >= 65536 and feat_dev is None
    if miss_path == "auto":
        miss_path = "staged" if (eligible and host_threads >= 8) else "zero_copy"
    stage_ring = None
    trial = {}
    if miss_path in ("staged", "staged_scatter", "staged_kernel") or (miss_path == "trial" and eligible):
        # capacity 0: nothing is kept in host memory, every miss row passes through the ring
        stage_ring = B.HostTier(w.features.view(np.uint8).reshape(cfg.num_nodes, cfg.row_bytes), 0, pipe.cap,
                                args.tier_threads)
        # staged: one pass writes the whole output once the rows have landed; staged_scatter: hit gather at
        # lookup time, landed rows scattered later; staged_kernel: kernels read the packed rows over the link
        stage_ring.set_copy_engine({"staged_kernel": 0, "staged_scatter": 1}.get(miss_path, 2))
    if miss_path == "trial":
        miss_path = "zero_copy"
        if stage_ring is not None:
            for name, tier in (("zero_copy", None), ("staged", stage_ring)):
                pipe.tier = tier
                pipe.run(seeds_dev, w.rng_seeds, 3)
                scratch.close()
                scratch = new_cache()
                pipe.set_cache(scratch)
                torch.cuda.synchronize()
                q0 = time.perf_counter()
                pipe.run(seeds_dev, w.rng_seeds, max(args.warmup, 10))
                trial[name] = 1e3 * (time.perf_counter() - q0) / max(args.warmup, 10)
                scratch.close()
                scratch = new_cache()
                pipe.set_cache(scratch)
            miss_path = min(trial, key=trial.get)
    staged = miss_path in ("staged", "staged_scatter", "staged_kernel")
    copies_over_link = miss_path in ("staged", "staged_scatter")
    pipe.tier = stage_ring if staged else None
    if args.warmup > 0:
        pipe.run(seeds_dev, w.rng_seeds, args.warmup)
    scratch.close()

    cache = new_cache()
    pipe.set_cache(cache)
    # (a run of a few batches times every one of them)
    g_every = 1 if (args.all_stage_timers or steps < 2 * GATHER_SAMPLE_EVERY) else GATHER_SAMPLE_EVERY
    l_every = 1 if (args.all_stage_timers or steps < 2 * LINK_SAMPLE_EVERY) else LINK_SAMPLE_EVERY
    if not args.no_stage_timers:
        # A timed launch holds its stream up for ~10 us, so the kernels that move the rows in HBM are timed
        # in every 4th batch only and what crosses the link (several launches per batch) in every 10th.
        cache.set_profiling(True if args.all_stage_timers else ("gather_hit", "fetch_miss", "link_copy",
                                                                 "assemble_pre", "assemble"))
        if not args.all_stage_timers:
            for stage in ("gather_hit", "assemble_pre", "assemble"):
                cache.set_profiling_every(stage, g_every)
            cache.set_profiling_every("fetch_miss", l_every)
            cache.set_profiling_every("link_copy", l_every)
    ring_before = stage_ring.stats() if staged else None
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n_list, hit_list = pipe.run(seeds_dev, w.rng_seeds, steps)   # ends with a device synchronise
    t1 = time.perf_counter()
    elapsed = t1 - t0

    n_arr, h_arr = np.array(n_list, dtype=np.int64), np.array(hit_list, dtype=np.int64)
    tot_n, tot_hit = int(n_arr.sum()), int(h_arr.sum())
    st = cache.stats()
    assert st["status"] == 0 and st["lookups"] == tot_n and st["hits"] == tot_hit
    # steady state: batches issued after the cache has filled once
    filled = np.cumsum(n_arr - h_arr) >= cfg.cache_rows
    steady = slice(int(np.argmax(filled)) + 1, None) if filled.any() else slice(0, 0)
    steady_ratio = (float(h_arr[steady].sum()) / float(n_arr[steady].sum())) if n_arr[steady].sum() else None
    ms_map = cache.map_stats()

    rb = cfg.row_bytes
    result = {
        "metric": "minibatches/sec + gathered feature GB/s (% HBM peak) + cache hit ratio",
        "value": steps / elapsed,
        "unit": "minibatches/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": args.warmup,
        "ms_per_step": 1e3 * elapsed / steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {
            "workload": f"{cfg.name}: N={cfg.num_nodes} E={w.num_edges} power-law graph, "
                        f"{cfg.feat_dtype} x {cfg.feat_dim} features, batch {cfg.batch}, "
                        f"fanout {list(cfg.fanouts)}, FIFO cache {cfg.cache_rows} rows, "
                        f"{cfg.order} seed order, epoch from an empty cache, miss path {miss_path}"
                        + ("" if args.graph_placement == "config" else f", CSR placement {where}")
                        + ("" if feat_dev is None else ", feature table in HBM"),
            "name": cfg.name,
            "row_bytes": rb,
            "mean_input_nodes": tot_n / steps,
            "hit_ratio_cumulative": tot_hit / max(tot_n, 1),
            "hit_ratio_steady_state": steady_ratio,
            "miss_path": miss_path, "pipeline": type(pipe).__name__,
            "miss_path_trial_ms_per_batch": trial or None,
            "host_copy_threads": (stage_ring.stats()["threads"] if staged else 0),
            "host_copy_ms_per_batch": ((stage_ring.stats()["copy_ms"] - ring_before["copy_ms"]) / steps
                                       if staged else None),
            "gathered_feature_GBps": rb * tot_n / elapsed / 1e9,
            "map_bucket_lines_per_lookup": ms_map["lines_per_id"],
        },
    }
    if not args.no_stage_timers:
        prof = cache.profile()
        g_sampled = [i for i in range(steps) if (i + 1) % g_every == 0]  # the cache counts its lookups from 1
        g_hit = int(sum(h_arr[i] for i in g_sampled))
        g_miss = int(sum(n_arr[i] - h_arr[i] for i in g_sampled))
        # HBM bytes per batch of the dominant kernel from the committed rocprofv3 --pmc summary of this same
        # workload (a builder-run profile, not measured in this run: counters need the profiler)
        traffic, tsrc = None, None
        tpath = os.path.join(ROOT, "profiles", f"pmc_hbm_traffic_{cfg.name}.md")
        assembled = prof["assemble"][1] > 0
        if os.path.exists(tpath):
            import re
            key = "k_assemble_rows" if assembled else "k_gather_hits"
            m = re.search(r"^%s hbm_bytes_per_launch = (\d+)" % key, open(tpath).read(), re.M)
            if m:
                traffic = float(m.group(1))
                tsrc = f"profiles/pmc_hbm_traffic_{cfg.name}.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, committed; not measured in this run)"
        # The library has the kernel dispatch itself record the kernel's begin and end on the
        # device, so the stage times are sums of the kernels' own durations (what a kernel trace shows).
        timing = ("begin/end of each kernel recorded on the device by its own dispatch (hipExtLaunchKernelGGL "
                  "events), every %d-th batch of the timed epoch" % g_every)
        if assembled:
            # One pass writes the whole output: per hit a row read from the cache buffer and written to out_rows,
            # per miss a landed row read, written to out_rows and (write-through) to the cache buffer.  Where the
            # buffer has no spare row positions a short pass runs before it (hits whose rows this batch's misses
            # overwrite); it is then counted with it, bytes and time.
            a_ms, a_n = prof["assemble"]
            p_ms, p_n = prof["assemble_pre"]
            per_miss = 3.0 if pipe.write_through else 2.0
            moved = 2.0 * rb * g_hit + per_miss * rb * g_miss
            k_ms = max(a_ms + p_ms, 1e-9)
            achieved = moved / (k_ms * 1e-3) / 1e9
            result["roofline"] = {
                "kernel": "k_assemble_rows" + (" (with k_assemble_pre)" if p_n else ""), "bound": "hbm", "achieved": achieved,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                "traffic_source": tsrc,
                "frac_lines": frac_in_lines(rb, g_hit, g_miss, True, pipe.write_through) / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "bytes_per_launch": moved / max(a_n, 1), "avg_launch_us": 1e3 * k_ms / max(a_n, 1), "launches": a_n,
                "avg_us": {"k_assemble_rows": 1e3 * a_ms / max(a_n, 1), "k_assemble_pre": 1e3 * p_ms / max(p_n, 1)},
                "bytes": "per launch (= per batch): 2 x row_bytes x hits + %d x row_bytes x misses" % per_miss
                         + ("; the first pass of a batch is counted with its launch" if p_n else ""),
                "timing": timing,
            }
        else:
            g_ms, g_n = prof["gather_hit"]
            g_kernel_ms = max(g_ms, 1e-9)
            achieved = 2.0 * rb * g_hit / (g_kernel_ms * 1e-3) / 1e9 if g_n > 0 else 0.0
            result["roofline"] = {
                "kernel": "k_gather_hits", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": tsrc,
                "frac_lines": frac_in_lines(rb, g_hit, g_miss, False, pipe.write_through) / (g_kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "bytes_per_launch": 2.0 * rb * g_hit / max(g_n, 1),
                "avg_launch_us": 1e3 * g_kernel_ms / max(g_n, 1), "launches": g_n,
                "bytes": "per launch: 2 x row_bytes x hits",
                "timing": timing,
            }
        skip = ("fetch_miss", "link_copy", "gather_hit", "assemble", "assemble_pre")
        result["stage_ms_per_step"] = {k: (v[0] / steps if k != "event_overhead" else v[0])
                                       for k, v in prof.items() if v[1] > 0 and k not in skip}
        for k in ("gather_hit", "assemble", "assemble_pre"):
            if prof[k][1] > 0:
                result["stage_ms_per_step"][k] = prof[k][0] / max(len(g_sampled), 1)
        # Host link: what carries the miss rows of the sampled batches of the timed epoch
        every = l_every
        sampled = [i for i in range(steps) if (i + 1) % every == 0]      # the cache counts its lookups from 1
        # staged: the link is the copies' (timed by event records on the copy stream), the fetch stage is
        # the kernels that scatter the landed rows in device memory
        over_link = "link_copy" if copies_over_link else "fetch_miss"
        f_ms, f_n = prof[over_link]
        miss3 = int(sum(n_arr[i] - h_arr[i] for i in sampled))
        link = miss3 * rb / (f_ms * 1e-3) / 1e9 if f_ms > 0 else 0.0
        h2d = measure_h2d_peak(torch)
        result["host_link"] = {
            "kernel": {"staged": "hipMemcpyAsync of the packed rows", "staged_scatter": "hipMemcpyAsync of the packed rows",
                       "staged_kernel": "k_fetch_rows"}.get(miss_path, "k_fetch_miss"),
            "achieved": link, "unit": "GB/s",
            "nominal_peak": HOST_LINK_NOMINAL_GBS, "measured_h2d_copy_peak": h2d,
            "frac_of_nominal": link / HOST_LINK_NOMINAL_GBS, "frac_of_measured": link / h2d,
            "avg_launch_us": 1e3 * f_ms / max(f_n, 1), "launches_per_step": f_n / max(len(sampled), 1),
            "link_ms_per_step": f_ms / max(len(sampled), 1),
            "link_bound_ms_per_step": 1e3 * (tot_n - tot_hit) / steps * rb / (h2d * 1e9),
            "note": "%s of every %d-th batch of the timed epoch (%d batches), timed by %s"
                    % ("copies" if copies_over_link else "fetch kernels", every, len(sampled),
                       "event records around each copy" if copies_over_link else "their dispatches"),
        }
        if miss_path == "staged_scatter":
            s_ms, s_n = prof["fetch_miss"]
            result["host_link"]["scatter_kernels_us_per_step"] = 1e3 * s_ms / max(len(sampled), 1)
            # the kernel that scatters the landed rows: every miss row read once from HBM and written
            # once to out_rows, and once more to the cache buffer in write-through mode
            moved = (3.0 if pipe.write_through else 2.0) * rb * miss3
            a3 = moved / (s_ms * 1e-3) / 1e9 if s_ms > 0 else 0.0
            result["roofline_scatter"] = {
                "kernel": "k_fetch_rows", "bound": "hbm", "achieved": a3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": a3 / HBM_PEAK_GBS, "bytes_per_step": moved / max(len(sampled), 1),
                "avg_us_per_step": 1e3 * s_ms / max(len(sampled), 1), "launches": s_n,
                "note": "landed miss rows to out_rows and the cache buffer, every %d-th batch" % every,
            }

        # The stand-alone hit gather (k_gather_hits, the kernel of bgl_cache_lookup_gather) on a launch that
        # is mostly hits (outside the timed region, not part of `value`): the epoch's last batch is looked up
        # again right after its insertion; only the rows its own insertions evicted miss.
        if pipe.last_n:
            cache.set_write_through(False)       # lookups without inserts follow
            cache.set_profiling(("gather_hit",))
            cache.set_profiling_every("gather_hit", 1)
            reps, hits2 = 5, 0
            for _ in range(reps):
                cache.lookup_gather(pipe.last_ids, pipe.last_n, pipe.out_rows, pipe.out_slot, pipe.miss_pos)
                torch.cuda.synchronize()
                hits2 += int(cache.n_hit_host[0])
            p2 = cache.profile()
            k_ms = max(p2["gather_hit"][0], 1e-9)
            a2 = 2.0 * rb * hits2 / (k_ms * 1e-3) / 1e9
            result["roofline_repeat_lookup"] = {
                "kernel": "k_gather_hits", "bound": "hbm", "achieved": a2, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": a2 / HBM_PEAK_GBS, "bytes_per_launch": 2.0 * rb * hits2 / reps,
                "avg_launch_us": 1e3 * k_ms / reps, "launches": reps,
                "hit_ratio": hits2 / (reps * pipe.last_n),
                "note": "last batch of the epoch looked up again after its insertion; not part of value",
            }

    # k-hop sampling on its own (outside the timed region; in the pipeline it hides under the
    # miss fetch): back-to-back sampling calls, no host round trip in between.
    reps = min(50, nb)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    smp = pipe.samplers[0]
    smp.sample(seeds_dev[0], int(w.rng_seeds[0]))
    torch.cuda.synchronize()
    e0.record()
    for b in range(reps):
        smp.sample(seeds_dev[b], int(w.rng_seeds[b]))
    e1.record()
    torch.cuda.synchronize()
    s_ms = e0.elapsed_time(e1) / reps
    counts = smp.counts_host.numpy()
    result["sampling_only"] = {
        "ms_per_batch": s_ms, "minibatches_per_s": 1e3 / s_ms,
        "sampled_edges_per_s": float(counts[B.BGL_MAX_HOPS + 1: B.BGL_MAX_HOPS + 1 + len(cfg.fanouts)].sum()) / (s_ms * 1e-3),
        "note": "bgl_sample_khop alone, %d batches back to back" % reps,
    }

    if args.two_level >= 0:
        # Two-level cache (Sec. 3.2.3) on the same batches, outside the timed region of `value`:
        # the feature table in ordinary host memory plays the graph store, the tier is a FIFO
        # cache in page-locked memory in front of it.  The lookup blocks the host while the
        # tier serves the GPU cache's misses.
        store = np.array(w.features.view(np.uint8).reshape(cfg.num_nodes, rb), copy=True)
        tier_rows = int(args.two_level * cfg.num_nodes)
        steps2 = min(steps, 100)
        tier = B.HostTier(store, tier_rows, pipe.cap, args.tier_threads)
        tier.set_copy_engine(args.miss_path != "staged_kernel")
        c2 = B.Cache(cfg.cache_rows, None, num_nodes=cfg.num_nodes, row_bytes=rb)
        pipe2 = pipe                 # the same streams and workspaces (hardware queues are few)
        pipe2.write_through = True
        pipe2.tier = tier
        pipe2.set_cache(c2)
        torch.cuda.synchronize()
        q0 = time.perf_counter()
        n2, h2 = pipe2.run(seeds_dev, w.rng_seeds, steps2)
        q1 = time.perf_counter()
        t2_first = list(pipe2.tier_hits)
        # a second pass over the same seeds (other sampling seeds): both levels warm
        na, ha = pipe2.run(seeds_dev, w.rng_seeds, steps2, first_step=steps2 if nb == steps2 else nb)
        q2 = time.perf_counter()
        n2, h2, t2 = np.array(n2), np.array(h2), np.array(t2_first)
        ts = tier.stats()
        result["two_level"] = {
            "minibatches_per_s": steps2 / (q1 - q0), "ms_per_batch": 1e3 * (q1 - q0) / steps2, "steps": steps2,
            "tier_rows": tier_rows, "tier_fraction_of_nodes": args.two_level, "host_threads": ts["threads"],
            "gpu_hit_ratio": float(h2.sum()) / float(n2.sum()),
            "tier_hit_ratio_of_gpu_misses": float(t2.sum()) / float((n2 - h2).sum()),
            "ms_per_batch_warm": 1e3 * (q2 - q1) / steps2,
            "store_rows_per_batch": float((n2 - h2 - t2).sum()) / steps2,
            "store_GBps": float((n2 - h2 - t2).sum()) * rb / (q1 - q0) / 1e9,
            "host_store_copy_ms_per_batch": ts["copy_ms"] / max(ts["batches"], 1),
            "note": "epoch from two empty levels; store = feature table in ordinary host memory",
        }
        c2.close()
        tier.close()
        del store

    if cfg.order == "po":
        # Proximity-aware ordering as the library computes it (once per epoch, outside the
        # timed region): 5 BFS sequences over the training set on the GPU, merged on the host.
        # (the epoch's seed batches above are the first batch x num_batches nodes of this order)
        train, roots, shifts = (w.order_draws[k] for k in ("train", "roots", "shifts"))
        B.order_proximity(graph, train, roots, shifts, len(train))          # warm-up
        o0 = time.perf_counter()
        order = B.order_proximity(graph, train, roots, shifts, len(train))
        o1 = time.perf_counter()
        result["ordering"] = {
            "call": "bgl_order_proximity", "sequences": cfg.po_sequences, "train_nodes": int(len(train)),
            "seconds": o1 - o0,
            "edges_traversed_per_s": cfg.po_sequences * w.num_edges / (o1 - o0),
        }
        if want_cpu:
            import oracle
            c0 = time.perf_counter()
            want = oracle.proximity_order(w.row_ptr, w.col, train, roots, shifts, len(train))
            result["ordering"]["oracle_seconds"] = time.perf_counter() - c0
            assert np.array_equal(order, want)
            assert np.array_equal(order[: w.seed_batches.size], w.seed_batches.reshape(-1))

    if want_cpu:
        # The CPU oracle on the batches the GPU leg has just run (a bounded sample: the first ones of them),
        # one core; its input counts and hit counts must be the GPU's.
        import oracle
        oc = oracle.Cache(cfg.cache_rows, w.features)
        nbat = min(steps, nb, args.cpu_batches)
        if args.steps_capped:                    # five configurations in one run: bound each one's share
            nbat = min(nbat, 100 if cfg.name == HEADLINE else 20)
        c0 = time.perf_counter()
        o_n, o_h = [], []
        for b in range(nbat):
            sg = oracle.sample_khop(w.row_ptr, w.col, w.seed_batches[b], cfg.fanouts, int(w.rng_seeds[b]))
            out, o_slot, o_miss, o_hit = oc.lookup_gather(sg.input_nodes)
            oc.insert_fifo(sg.input_nodes, o_miss, out)
            o_n.append(len(sg.input_nodes))
            o_h.append(o_hit)
        c1 = time.perf_counter()
        assert o_n == n_list[:nbat] and o_h == hit_list[:nbat], "the oracle's batches differ from the GPU's"
        result["cpu_baseline"] = {
            "value": nbat / (c1 - c0), "unit": "minibatches/s", "cores": 1, "kind": "oracle",
            "sample": f"the first {nbat} of the {steps} timed batches of this workload, same inputs, from an empty "
                      "cache (includes the Python/numpy marshalling around the C oracle); input and hit counts "
                      "per batch checked against the GPU run",
            "host_cores_available": os.cpu_count(),
        }
    if stage_ring is not None:
        stage_ring.close()
    cache.close()
    return result


ALL_CONFIGS = ("tiny", "mid", "bfs", "wide", "large")   # (small to large: see run order note in main)
HEADLINE = "large"       # the largest configuration that fits one GPU (Ogbn-papers shape)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2
    import gc
    import numpy as np
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    if args.calibrate_copy:
        a = torch.full((1 << 30,), 7, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": 1 << 30, "copies": 3}))
        return 0
    from paper_2112_08541_amd import binding as B
    torch.cuda.set_device(0)
    if args.hit_gather_sweep:
        print(json.dumps(hit_gather_sweep(torch, np, B)))
        return 0
    from paper_2112_08541_amd import inputs
    from paper_2112_08541_amd.pipeline import MinibatchPipeline

    # Run order, small to large: after the tens of gigabytes of page-locked memory of `large` and `wide` have
    # been allocated and freed, the host threads that pack `mid`'s miss rows were measured a third slower
    # (2.8 instead of 2.3 ms per batch), which says something about the host's memory, not about the path.
    names = ALL_CONFIGS if args.config == "all" else (args.config,)
    args.steps_capped = args.config == "all"     # one line for five epochs of different lengths
    results = {}
    for name in names:
        t0 = time.perf_counter()
        results[name] = run_config(inputs.CONFIGS[name], args, torch, np, B, inputs, MinibatchPipeline,
                                   want_cpu=not args.no_cpu_baseline)
        results[name]["config"]["wall_seconds_incl_input_generation"] = time.perf_counter() - t0
        gc.collect()
        torch.cuda.empty_cache()
    head = dict(results[HEADLINE if args.config == "all" else names[0]])
    if args.config == "all":
        # every configuration's figures beside the headline's (each one epoch, or `steps` batches of it,
        # from an empty cache, with its own oracle sample)
        def brief(r):
            out = {"name": r["config"]["name"], "workload": r["config"]["workload"],
                   "minibatches_per_s": r["value"], "ms_per_step": r["ms_per_step"], "steps": r["steps"],
                   "mean_input_nodes": r["config"]["mean_input_nodes"],
                   "hit_ratio_cumulative": r["config"]["hit_ratio_cumulative"],
                   "hit_ratio_steady_state": r["config"]["hit_ratio_steady_state"],
                   "gathered_feature_GBps": r["config"]["gathered_feature_GBps"],
                   "miss_path": r["config"]["miss_path"],
                   "host_copy_threads": r["config"]["host_copy_threads"],
                   "host_copy_ms_per_batch": r["config"]["host_copy_ms_per_batch"],
                   "map_bucket_lines_per_lookup": r["config"]["map_bucket_lines_per_lookup"]}
            if "roofline" in r:
                rf = r["roofline"]
                out["roofline"] = {k: rf[k] for k in ("kernel", "achieved", "frac", "frac_lines", "bytes_per_launch",
                                                      "avg_launch_us", "launches")}
                out["roofline_repeat_lookup_frac"] = r.get("roofline_repeat_lookup", {}).get("frac")
                hl = r["host_link"]
                out["host_link"] = {k: hl[k] for k in ("kernel", "achieved", "frac_of_nominal", "frac_of_measured",
                                                       "link_ms_per_step", "link_bound_ms_per_step")}
            out["sampling_only_ms_per_batch"] = r["sampling_only"]["ms_per_batch"]
            if "cpu_baseline" in r:
                out["cpu_baseline"] = {k: r["cpu_baseline"][k] for k in ("value", "cores", "sample")}
            if "ordering" in r:
                out["ordering"] = r["ordering"]
            return out
        head["configs"] = [brief(results[n]) for n in names]
    print(json.dumps(head))
    return 0


if __name__ == "__main__":
    sys.exit(main())
