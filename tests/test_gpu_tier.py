"""GPU parity for the two-level cache (GPU cache, then the FIFO tier in host
memory, then the feature store; Sec. 3.2.3) against the oracle's two-level
cache (oracle.TwoLevel: the second level sees the first one's misses, in order,
as its batch).  Bytes, slots, lists and both levels' states must be equal."""
import numpy as np
import pytest

from helpers import assert_state_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


@pytest.fixture(scope="module")
def B(torch_mod):
    from paper_2112_08541_amd import binding
    binding.lib()
    return binding


def assert_tier_state_equal(tier, oc2, what):
    s2n, tail, buf = tier.export_state(True)
    o_s2n = oc2.slot_to_node
    assert tail == oc2.tail, what
    assert np.array_equal(s2n, o_s2n), what
    live = o_s2n >= 0
    assert np.array_equal(buf[live], oc2.buffer[live]), what


def run_tiered_stream(B, torch, feats, cap1, cap2, batches, write_through, threads, side=True,
                      cache_has_store=False, early=None, copy_engine=False, spare=0, halves=False):
    import oracle
    N, rb = feats.shape[0], feats.shape[1] * feats.itemsize
    store = np.ascontiguousarray(feats.view(np.uint8).reshape(N, rb))      # ordinary host memory
    max_n = max(max((len(b) for b in batches), default=1), 1)
    # as in bench.py's staged miss path: the cache keeps its own page-locked table
    pinned = torch.from_numpy(store).pin_memory() if cache_has_store else None
    gc = B.Cache(cap1, pinned, num_nodes=N, row_bytes=rb)
    if spare:           # extra row positions in the cache buffer (with enough of them the one-pass output has no first pass)
        gc.set_spare_rows(spare)
    tier = B.HostTier(store, cap2, max_n, threads)
    if copy_engine:     # the packed rows cross the link as plain copies into device memory (2: assembled output)
        tier.set_copy_engine(copy_engine)
    # capacity 0: the tier keeps nothing (every miss row just passes through its ring)
    two = oracle.TwoLevel(cap1, cap2, feats)
    oc1, oc2 = two.level1, two.level2
    if write_through:
        gc.set_write_through(True)
    side_stream = torch.cuda.Stream() if side else None
    # early lookup: the map lookup and the lists run on a stream of their own ("own"), on the
    # one that also carries the map updates ("with_insert", as the benchmarked pipeline does), or only
    # every other call ("alternate")
    lookup_stream = torch.cuda.Stream() if early else None
    for bi, ids in enumerate(batches):
        n = len(ids)
        ids_t = (torch.tensor(ids, dtype=torch.int32, device="cuda") if n
                 else torch.empty(1, dtype=torch.int32, device="cuda"))
        out = torch.full((max(n, 1), rb), 0xCD, dtype=torch.uint8, device="cuda")
        out_slot = torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda")
        miss_pos = torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda")
        if lookup_stream is not None:
            lookup_stream.wait_stream(torch.cuda.current_stream())      # ids_t and the filled outputs
        # hold one of the streams up for a while (a spin kernel that ends by itself), a different one
        # each batch: a missing wait between the streams then shows as a wrong result
        streams = [st for st in (lookup_stream, torch.cuda.current_stream(), side_stream) if st is not None]
        if len(streams) > 1:
            with torch.cuda.stream(streams[bi % len(streams)]):
                torch.cuda._sleep(2_000_000)
        use_ls = lookup_stream if (early != "alternate" or bi % 2 == 1) else None
        h1, h2 = gc.lookup_gather_tiered(tier, ids_t, n, out, out_slot, miss_pos, side_stream=side_stream,
                                         lookup_stream=use_ls, begin_only=halves)
        gc.insert_fifo(ids_t, miss_pos, -1, out, stream=lookup_stream if early == "with_insert" else None)
        if halves:      # the call in two halves: the map update is enqueued between them, as the pipeline does
            if bi % 3 == 1:
                with torch.cuda.stream(streams[(bi + 1) % len(streams)]):
                    torch.cuda._sleep(1_000_000)
            gc.lookup_tiered_finish()
        gc.wait_rows()
        torch.cuda.synchronize()
        # oracle: level 1, then level 2 on level 1's misses, both updated first-in first-out
        o_out, o_slot, o_miss, o_hit, o2_hit = two.lookup_gather(ids)
        two.insert_fifo(ids, o_miss, o_out)
        what = f"batch {bi}"
        assert (h1, h2) == (o_hit, o2_hit), what
        assert np.array_equal(out_slot[:n].cpu().numpy(), o_slot), what
        assert np.array_equal(miss_pos[: n - h1].cpu().numpy(), o_miss), what
        assert np.array_equal(out[:n].cpu().numpy(), o_out), what
        assert np.array_equal(o_out, store[np.asarray(ids, dtype=np.int64)] if n else o_out), what  # the store's bytes
        assert_state_equal(gc, oc1, what)
        if oc2 is not None:
            assert_tier_state_equal(tier, oc2, what)
    st = tier.stats()
    if oc2 is not None:
        assert (st["lookups"], st["hits"]) == oc2.stats()
    else:
        total_miss = sum(len(b) for b in batches) - gc.stats()["hits"]
        passed = tier.export_state(True)[1]          # rows that went through the ring
        assert st["hits"] == 0 and passed == total_miss
    return gc, tier


def zipf_batches(rng, N, count, lo, hi, big=None):
    batches = []
    for b in range(count):
        size = int(rng.integers(lo, hi)) if b != 5 or big is None else big
        batches.append(list(dict.fromkeys((rng.zipf(1.2, size) % N).tolist())))
    batches.insert(3, [])
    batches.insert(8, batches[7])
    return batches


@pytest.mark.parametrize("dim,dtype", [(4, np.float32), (100, np.float32), (128, np.float32), (264, np.uint16)])
@pytest.mark.parametrize("write_through,early", [(False, None), (True, None), (True, "own"), (True, "with_insert"),
                                                 (True, "alternate")])
@pytest.mark.parametrize("copy_engine", [False, True, 2])
def test_tiered_random_streams(B, torch_mod, dim, dtype, write_through, early, copy_engine):
    rng = np.random.default_rng(100 + dim)
    N = 20000
    feats = (rng.standard_normal((N, dim)).astype(np.float32) if dtype == np.float32
             else rng.integers(0, 2**16, (N, dim), dtype=np.uint16))
    # batch 5 has more misses than either level has slots
    batches = zipf_batches(rng, N, 14, 1, 2500, big=9000)
    run_tiered_stream(B, torch_mod, feats, 1500, 4000, batches, write_through, threads=4, early=early,
                      copy_engine=copy_engine)


@pytest.mark.parametrize("cap2", [0, 4000])
@pytest.mark.parametrize("early", [None, "own", "with_insert"])
@pytest.mark.parametrize("copy_engine,spare", [(False, 0), (True, 0), (2, 0), (2, 9000)])
def test_tiered_lookup_in_two_halves(B, torch_mod, cap2, early, copy_engine, spare):
    """bgl_cache_lookup_tiered_begin / _finish with the batch's map update enqueued between them."""
    rng = np.random.default_rng(77 + cap2)
    N = 20000
    feats = rng.standard_normal((N, 100)).astype(np.float32)
    batches = zipf_batches(rng, N, 14, 1, 2500, big=9000)
    run_tiered_stream(B, torch_mod, feats, 1500, cap2, batches, True, threads=4, early=early,
                      copy_engine=copy_engine, spare=spare, halves=True)


def test_tiered_halves_refuse_what_does_not_fit_between_them(B, torch_mod):
    torch = torch_mod
    rng = np.random.default_rng(5)
    N = 4000
    feats = rng.standard_normal((N, 8)).astype(np.float32)
    store = np.ascontiguousarray(feats.view(np.uint8).reshape(N, 32))
    gc = B.Cache(500, None, num_nodes=N, row_bytes=32)
    tier = B.HostTier(store, 0, 1000, 2)
    ids = torch.arange(0, 300, dtype=torch.int32, device="cuda")
    out = torch.zeros((1000, 32), dtype=torch.uint8, device="cuda")
    slot = torch.zeros(1000, dtype=torch.int32, device="cuda")
    mp = torch.zeros(1000, dtype=torch.int32, device="cuda")
    with pytest.raises(B.BglError, match="no tiered lookup has been begun"):
        gc.lookup_tiered_finish()
    # without write-through mode the FIFO update needs the rows the second half brings in
    gc.lookup_gather_tiered(tier, ids, 300, out, slot, mp, begin_only=True)
    with pytest.raises(B.BglError, match="has been begun"):
        gc.insert_fifo(ids, mp, -1, out)
    with pytest.raises(B.BglError, match="has been begun"):
        gc.lookup_gather_tiered(tier, ids, 300, out, slot, mp)
    with pytest.raises(B.BglError, match="has been begun"):
        gc.set_write_through(True)
    gc.lookup_tiered_finish()
    gc.insert_fifo(ids, mp, -1, out)
    torch.cuda.synchronize()
    assert np.array_equal(out[:300].cpu().numpy(), store[:300])
    # and the pair still works after the refusals: everything hits now
    h1, h2 = gc.lookup_gather_tiered(tier, ids, 300, out, slot, mp, begin_only=True)
    gc.lookup_tiered_finish()
    gc.insert_fifo(ids, mp, -1, out)
    torch.cuda.synchronize()
    assert (h1, h2) == (300, 0)
    assert np.array_equal(out[:300].cpu().numpy(), store[:300])
    tier.close()
    gc.close()


@pytest.mark.parametrize("cap2", [0, 900_000])
def test_tiered_lookups_of_many_tiles(B, torch_mod, cap2):
    """More than 4096 tiles of 256 ids in both levels' list kernels (prefix sums from a scan kernel)."""
    rng = np.random.default_rng(78)
    N = 3_000_000
    feats = rng.integers(0, 2**31, (N, 4), dtype=np.int32).view(np.float32)      # 16-byte rows, compared as bytes
    perm = rng.permutation(N).astype(np.int32)
    batches = [perm[:1_300_000], perm[600_000:2_000_001], perm[:1_200_000]]
    run_tiered_stream(B, torch_mod, feats, 200_000, cap2, batches, True, threads=0, early="with_insert",
                      copy_engine=(2 if cap2 == 0 else False))


@pytest.mark.parametrize("cap1,cap2,threads", [(64, 300, 1), (1, 1, 3), (500, 100, 2), (3000, 18000, 0),
                                               (1500, 0, 0), (1, 0, 1)])
def test_tiered_capacity_corners(B, torch_mod, cap1, cap2, threads):
    """A tier smaller than a batch's misses (early rows never enter it; found rows are served
    although the same batch evicts them), single slots, a tier smaller than the GPU cache,
    a tier that ends up holding nearly the whole store."""
    rng = np.random.default_rng(cap1 * 7 + cap2)
    N = 20000
    feats = rng.standard_normal((N, 100)).astype(np.float32)
    batches = zipf_batches(rng, N, 12, 200, 3000)
    _, tier = run_tiered_stream(B, torch_mod, feats, cap1, cap2, batches, True, threads, side=(threads != 2),
                                early=("with_insert" if threads in (0, 3) else None),
                                copy_engine=(False if cap1 == 64 else 2 if cap2 == 0 else True))
    assert tier.stats()["threads"] == (threads or tier.stats()["threads"])


@pytest.mark.parametrize("write_through,early", [(False, None), (True, None), (True, "own"), (True, "with_insert"),
                                                 (True, "alternate")])
@pytest.mark.parametrize("side", [False, True])
@pytest.mark.parametrize("copy_engine", [False, True, 2])
def test_staging_only_large_batches(B, torch_mod, write_through, side, early, copy_engine):
    """Capacity 0 (every miss row passes through the ring) with batches of several chunks, hits
    that the same batch's insertions evict (small GPU cache), an empty batch, a repeat."""
    rng = np.random.default_rng(77)
    N = 200000
    feats = rng.integers(0, 2**32, (N, 25 * 4), dtype=np.uint32).view(np.float32)
    batches = [rng.permutation(N)[: int(k)].tolist() for k in (70000, 300, 90000, 26000, 60000, 24576, 24577, 80000)]
    batches.insert(2, [])
    batches.insert(5, batches[4])     # immediate repeat: hits everywhere the cache kept them
    run_tiered_stream(B, torch_mod, feats, 50000, 0, batches, write_through, 0, side=side, cache_has_store=True,
                      early=early, copy_engine=copy_engine, spare=(90000 if side else 0))


@pytest.mark.parametrize("dim,cap1", [(100, 6000), (128, 900), (256, 2500), (4, 1), (36, 40000)])
@pytest.mark.parametrize("early,spare", [(None, 0), ("with_insert", 0), (None, 45000), ("with_insert", 2500), ("own", 1)])
def test_assembled_output_corner_cases(B, torch_mod, dim, cap1, early, spare):
    """The one-pass output (copy-engine transport, mode 2) where its two launches split the work
    differently: no miss at all (nothing lands, the pass only gathers), only misses, hits that
    all sit in the slots the batch's own misses take (more misses than slots; a repeat of the
    previous batch in a cache that wraps), none of them there (few misses in a large cache),
    an empty batch, one id."""
    rng = np.random.default_rng(dim * 31 + cap1)
    N = 50000
    feats = rng.integers(0, 2**32, (N, dim), dtype=np.uint32).view(np.float32)
    a = rng.permutation(N)[:2000].tolist()
    b = rng.permutation(N)[:7000].tolist()
    few_new = a[:1900] + [x for x in rng.permutation(N)[:200].tolist() if x not in set(a)][:50]
    mixed = list(dict.fromkeys(b[:3000] + a[:500]))
    batches = [a, a, [], a[:1], few_new, b, b, a, mixed, rng.permutation(N)[:45000].tolist(), a]
    run_tiered_stream(B, torch_mod, feats, cap1, 0, batches, True, threads=3, cache_has_store=True,
                      early=early, copy_engine=2, spare=spare)


def test_tiered_uniform_ids_many_chunks(B, torch_mod):
    """Batches long enough for many host tasks and several fetch grid strides."""
    rng = np.random.default_rng(5)
    N = 300000
    feats = rng.integers(0, 2**32, (N, 25 * 4), dtype=np.uint32).view(np.float32)
    batches = [rng.permutation(N)[: int(rng.integers(60000, 90000))].tolist() for _ in range(5)]
    run_tiered_stream(B, torch_mod, feats, 40000, 120000, batches, True, threads=0)
    run_tiered_stream(B, torch_mod, feats, 40000, 120000, batches, True, threads=0, early="with_insert", copy_engine=True)


def test_tiered_argument_errors(B, torch_mod):
    torch = torch_mod
    N, rb = 1000, 64
    store = np.random.default_rng(1).integers(0, 255, (N, rb), dtype=np.uint8)
    gc = B.Cache(100, None, num_nodes=N, row_bytes=rb)
    tier = B.HostTier(store, 200, 50, 2)
    ids = torch.arange(60, dtype=torch.int32, device="cuda")
    out = torch.zeros((60, rb), dtype=torch.uint8, device="cuda")
    slot = torch.zeros(60, dtype=torch.int32, device="cuda")
    mp = torch.zeros(60, dtype=torch.int32, device="cuda")
    with pytest.raises(B.BglError) as e:      # the cache has no store of its own
        gc.lookup_gather(ids, 10, out, slot, mp)
    assert e.value.code == B.BGL_EINVAL
    with pytest.raises(B.BglError) as e:      # more ids than the tier was sized for
        gc.lookup_gather_tiered(tier, ids, 60, out, slot, mp)
    assert e.value.code == B.BGL_ECAPACITY
    other = B.HostTier(np.zeros((N, 32), dtype=np.uint8), 10, 50, 1)
    with pytest.raises(B.BglError) as e:      # row width differs
        gc.lookup_gather_tiered(other, ids, 10, out, slot, mp)
    assert e.value.code == B.BGL_EINVAL
    with pytest.raises(B.BglError) as e:      # early lookup needs write-through mode
        gc.lookup_gather_tiered(tier, ids, 10, out, slot, mp, lookup_stream=torch.cuda.Stream())
    assert e.value.code == B.BGL_EINVAL
    bad = ids.clone()
    bad[3] = N + 5
    with pytest.raises(B.BglError) as e:      # id out of range: nothing changes
        gc.lookup_gather_tiered(tier, bad, 10, out, slot, mp)
    assert e.value.code == B.BGL_EINVAL
    torch.cuda.synchronize()
    s2n, tail, _ = tier.export_state(False)
    assert tail == 0 and (s2n == -1).all()
    assert gc.export_state(False)[1] == 0
    # and the pair still works afterwards
    h1, h2 = gc.lookup_gather_tiered(tier, ids, 10, out, slot, mp)
    gc.insert_fifo(ids, mp, -1, out)
    gc.wait_rows()
    torch.cuda.synchronize()
    assert (h1, h2) == (0, 0)
    assert np.array_equal(out[:10].cpu().numpy(), store[:10])
    h1, h2 = gc.lookup_gather_tiered(tier, ids, 20, out, slot, mp)
    gc.insert_fifo(ids, mp, -1, out)
    torch.cuda.synchronize()
    assert (h1, h2) == (10, 0)


@pytest.mark.parametrize("tier_fraction,copy_engine", [(0.3, True), (0.0, True), (0.0, False), (0.0, 2)])
def test_tiered_pipeline_as_benchmarked_matches_oracle(torch_mod, B, tier_fraction, copy_engine):
    """The configurations `bench.py` times on the full-size mid workload (sampling ahead,
    tiered lookups on the chain stream, write-through GPU cache): a tier of 30 % of the nodes
    (`--two-level 0.3`) and the staging ring without a tier (the default miss path for
    400-byte rows).  Every batch's outputs and both levels' final states."""
    import oracle
    from helpers import OraclePipeline, assert_batch_equal
    from paper_2112_08541_amd import inputs
    from paper_2112_08541_amd.pipeline import MinibatchPipeline
    torch = torch_mod
    cfg = inputs.CONFIGS["mid"]
    staging_only = tier_fraction == 0.0
    w = inputs.make_workload(cfg, pinned=staging_only)      # (mid: random seed order)
    rb = cfg.row_bytes
    store = np.ascontiguousarray(w.features.view(np.uint8).reshape(cfg.num_nodes, rb))
    graph = B.Graph(w.row_ptr, w.col)
    # as in bench.py: the staging-only path keeps the cache's own page-locked table
    cache = B.Cache(cfg.cache_rows, w.features.ctypes.data if staging_only else None,
                    num_nodes=cfg.num_nodes, row_bytes=rb)
    tier_rows = int(tier_fraction * cfg.num_nodes)
    pipe = MinibatchPipeline(graph, cache, cfg.batch, cfg.fanouts, rb, write_through=True, tier=None)
    tier = B.HostTier(store, tier_rows, pipe.cap, 0)
    tier.set_copy_engine(copy_engine)
    pipe.tier = tier
    seeds_dev = torch.from_numpy(w.seed_batches).cuda()
    got = {}

    def grab(i, sb, n, p):
        torch.cuda.synchronize()
        c = p.samplers[i % 3].counts_host.numpy()
        K = len(cfg.fanouts)
        nf, nnz = c[: K + 1].astype(np.int64), c[B.BGL_MAX_HOPS + 1: B.BGL_MAX_HOPS + 1 + K].astype(np.int64)
        n_hit = n - int((p.out_slot[:n] < 0).sum())
        got[i] = dict(n_frontier=nf, nnz=nnz, n=n, n_hit=n_hit,
                      input_nodes=sb.input_nodes(n).cpu().numpy(),
                      row_ptr=[sb.row_ptr(h, int(nf[h])).cpu().numpy() for h in range(len(nnz))],
                      col_local=[sb.col_local(h, int(nnz[h])).cpu().numpy() for h in range(len(nnz))],
                      out_slot=p.out_slot[:n].cpu().numpy(), miss_pos=p.miss_pos[: n - n_hit].cpu().numpy(),
                      out_rows=p.out_rows[:n].cpu().numpy())

    steps = 6
    n_list, hit_list = pipe.run(seeds_dev, w.rng_seeds, steps, on_batch=grab)
    op = OraclePipeline(w, tier_rows=tier_rows)
    for b in range(steps):
        o = op.run_batch(w.seed_batches[b], w.rng_seeds[b])
        assert_batch_equal(got[b], o, f"tiered batch {b}")
        assert (n_list[b], hit_list[b], pipe.tier_hits[b]) == (o["n"], o["n_hit"], o["n_hit_tier"])
    assert_state_equal(cache, op.cache, "tiered pipeline")
    if op.tier is not None:
        assert_tier_state_equal(tier, op.tier, "tiered pipeline")


def test_tiered_random_cases_property(B, torch_mod):
    """Seeded random store sizes, row widths (any multiple of 16 bytes), capacities of both
    levels (the tier's may be 0), batch sequences and call modes (hypothesis draws them,
    derandomized): the pair of caches follows the two chained oracle caches."""
    from hypothesis import given, settings, strategies as st, HealthCheck

    @settings(max_examples=25, deadline=None, derandomize=True, suppress_health_check=list(HealthCheck))
    @given(st.integers(50, 5000), st.integers(1, 65), st.integers(1, 3000), st.sampled_from([0, 0, 1, 17, 300, 4000]),
           st.lists(st.integers(0, 2500), min_size=1, max_size=8), st.booleans(), st.booleans(),
           st.sampled_from([None, "own", "with_insert", "alternate"]), st.integers(1, 5), st.integers(0, 2**31),
           st.sampled_from([0, 1, 2]), st.sampled_from([0, 0, 3, 700, 2600]))
    def run(n_nodes, row_chunks, cap1, cap2, sizes, write_through, side, early, threads, seed, copy_engine, spare):
        rng = np.random.default_rng(seed)
        feats = rng.integers(0, 2**32, (n_nodes, row_chunks * 4), dtype=np.uint32)
        batches = [rng.permutation(n_nodes)[: min(k, n_nodes)].tolist() for k in sizes]
        if early is not None and not write_through:
            early = None                      # the library refuses early lookups there (tested elsewhere)
        run_tiered_stream(B, torch_mod, feats, cap1, cap2, batches, write_through, threads, side=side,
                          cache_has_store=(cap2 == 0), early=early, copy_engine=copy_engine, spare=spare)

    run()
