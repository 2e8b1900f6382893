"""GPU parity: the HIP library, called through its C ABI, against the CPU
oracle, bit for bit (sampled ids, CSR blocks, lookup results, feature bytes,
cache state).  Integer and byte work only, so the bar is exact equality."""
import dataclasses
import os

import numpy as np
import pytest

from helpers import GpuPipeline, OraclePipeline, assert_batch_equal, assert_state_equal, make_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


@pytest.fixture(scope="module")
def B(torch_mod):
    from paper_2112_08541_amd import binding
    binding.lib()  # must load: there is no fallback
    return binding


def _inputs():
    from paper_2112_08541_amd import inputs
    return inputs


# ------------------------------------------------------------------ sampling
def csr_from_adj(adj, dtype=np.int32):
    rp = np.zeros(len(adj) + 1, dtype=dtype)
    col = []
    for i, row in enumerate(adj):
        col.extend(row)
        rp[i + 1] = len(col)
    return rp, np.array(col if col else [0], dtype=np.int32)[: len(col)]


def gpu_sample(B, torch, rp, col, seeds, fanouts, rng_seed, placement=None):
    g = B.Graph(rp, col, B.BGL_DEVICE if placement is None else placement)
    s = B.Sampler(g, len(seeds), fanouts)
    sb = s.sample(torch.tensor(seeds, dtype=torch.int32, device="cuda"), rng_seed)
    torch.cuda.synchronize()
    nf, nnz = sb.sizes()
    K = len(fanouts)
    res = dict(n_frontier=nf, nnz=nnz, input_nodes=sb.input_nodes(int(nf[K])).cpu().numpy(),
               row_ptr=[sb.row_ptr(h, int(nf[h])).cpu().numpy() for h in range(K)],
               col_local=[sb.col_local(h, int(nnz[h])).cpu().numpy() for h in range(K)])
    return res


def assert_sample_equal(res, sg):
    assert res["n_frontier"].tolist() == sg.n_frontier.tolist()
    assert res["nnz"].tolist() == list(sg.nnz)
    assert np.array_equal(res["input_nodes"], sg.input_nodes)
    for h in range(len(sg.nnz)):
        assert np.array_equal(res["row_ptr"][h], sg.row_ptr[h])
        assert np.array_equal(res["col_local"][h], sg.col_local[h])


TINY_GRAPHS = {
    "path": [[1], [0, 2], [1, 3], [2, 4], [3]],
    "star": [[1, 2, 3, 4, 5, 6, 7], [0], [0], [0], [0], [0], [0], [0]],
    "clique6": [[j for j in range(6) if j != i] for i in range(6)],
    "two_components": [[1, 2], [0, 2], [0, 1], [4], [3, 5], [4]],
    "isolated": [[1], [0], [], [0, 1]],
    "multi_edges": [[1, 1, 1, 2], [0, 0], [2, 2, 0, 0, 1]],
}


@pytest.mark.parametrize("name", sorted(TINY_GRAPHS))
@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_sample_tiny_graphs(B, torch_mod, name, dtype):
    import oracle
    rp, col = csr_from_adj(TINY_GRAPHS[name], dtype)
    N = len(rp) - 1
    for fanouts in ([2], [1, 1], [2, 2, 2], [3, 1], [10, 10], [64]):
        for seed in range(3):
            seeds = [seed % N, (seed * 3 + 1) % N, seed % N]
            res = gpu_sample(B, torch_mod, rp, col, seeds, fanouts, 1000 + seed)
            assert_sample_equal(res, oracle.sample_khop(rp, col, seeds, fanouts, 1000 + seed))


@pytest.mark.parametrize("fanouts", [(1,), (3,), (4,), (5, 5), (8, 3), (15, 10, 5), (16,), (17,), (25, 10),
                                     (33, 2), (64, 1), (2, 2, 2, 2, 2, 2, 2, 2)])
def test_sample_random_graph_all_group_widths(B, torch_mod, fanouts):
    """Dense-ish random graph so that Floyd's algorithm (degree > fanout) runs for
    every lane-group width, several tiles and a ragged tail."""
    import oracle
    rng = np.random.default_rng(sum(fanouts))
    N = 3000
    deg = rng.integers(0, 120, N)
    deg[rng.integers(0, N, 50)] = 0
    rp = np.zeros(N + 1, dtype=np.int32)
    rp[1:] = np.cumsum(deg)
    col = rng.integers(0, N, rp[-1]).astype(np.int32)
    seeds = rng.integers(0, N, 777).astype(np.int32)  # with repeats
    for s in (1, 2**63 + 12345):
        res = gpu_sample(B, torch_mod, rp, col, seeds.tolist(), list(fanouts), s)
        assert_sample_equal(res, oracle.sample_khop(rp, col, seeds, list(fanouts), s))


def test_sample_random_cases_property(B, torch_mod):
    """Seeded random graphs, seed lists, fanout lists and call seeds (hypothesis draws them;
    derandomized, so every run sees the same cases): sampled ids, CSR blocks and sizes equal
    the oracle's."""
    import oracle
    from hypothesis import given, settings, strategies as st, HealthCheck

    @settings(max_examples=40, deadline=None, derandomize=True, suppress_health_check=list(HealthCheck))
    @given(st.integers(1, 400), st.integers(0, 30), st.lists(st.integers(1, 20), min_size=1, max_size=4),
           st.integers(1, 300), st.integers(0, 2**64 - 1), st.booleans(), st.integers(0, 2**31))
    def run(n_nodes, max_deg, fanouts, n_seeds, call_seed, wide_offsets, graph_seed):
        rng = np.random.default_rng(graph_seed)
        deg = rng.integers(0, max_deg + 1, n_nodes)
        rp = np.zeros(n_nodes + 1, dtype=np.int64 if wide_offsets else np.int32)
        rp[1:] = np.cumsum(deg)
        col = rng.integers(0, n_nodes, int(rp[-1])).astype(np.int32)       # may be empty
        seeds = rng.integers(0, n_nodes, n_seeds).astype(np.int32)
        res = gpu_sample(B, torch_mod, rp, col, seeds.tolist(), fanouts, call_seed)
        assert_sample_equal(res, oracle.sample_khop(rp, col, seeds, fanouts, call_seed))

    run()


@pytest.mark.parametrize("num_seeds", [16384, 16385, 511 * 32, 1])
def test_sample_stage_sizes_around_the_scan_threshold(B, torch_mod, num_seeds):
    """A stage of at most 512 tiles of 512 padded positions has its tile totals scanned inside the
    finalize kernel, a larger one by a launch of its own: 16,384 seeds x 16 lanes (fanout 10) are
    exactly 512 tiles, one seed more is 513; the second hop (fanout 3) is far beyond either way."""
    import oracle
    rng = np.random.default_rng(num_seeds)
    N = 40000
    deg = rng.integers(0, 25, N)
    rp = np.zeros(N + 1, dtype=np.int32)
    rp[1:] = np.cumsum(deg)
    col = rng.integers(0, N, rp[-1]).astype(np.int32)
    seeds = rng.permutation(N)[:num_seeds].astype(np.int32)
    res = gpu_sample(B, torch_mod, rp, col, seeds.tolist(), [10, 3], 4242)
    assert_sample_equal(res, oracle.sample_khop(rp, col, seeds, [10, 3], 4242))


def test_sample_high_degree_hub_and_host_pinned_graph(B, torch_mod):
    import oracle
    rng = np.random.default_rng(11)
    N = 5000
    deg = rng.integers(1, 8, N)
    deg[7] = 70000  # hub with degree far above 2^16
    rp = np.zeros(N + 1, dtype=np.int64)
    rp[1:] = np.cumsum(deg)
    col = rng.integers(0, N, rp[-1]).astype(np.int32)
    col[rp[100]: rp[101]] = 7  # make the hub reachable
    rp_t = torch_mod.from_numpy(rp).pin_memory()
    col_t = torch_mod.from_numpy(col).pin_memory()
    seeds = [100, 7, 3, 4000]
    for fan in ([15, 10], [64, 64]):
        for placement in (B.BGL_HOST_PINNED, B.BGL_HOST_PINNED_COL):
            res = gpu_sample(B, torch_mod, rp_t, col_t, seeds, fan, 99, placement)
            assert_sample_equal(res, oracle.sample_khop(rp, col, seeds, fan, 99))


def test_sample_is_deterministic_and_seed_sensitive(B, torch_mod):
    w = _inputs().make_workload(_inputs().CONFIGS["tiny"])
    a = gpu_sample(B, torch_mod, w.row_ptr, w.col, w.seed_batches[0].tolist(), [10, 5], 5)
    b = gpu_sample(B, torch_mod, w.row_ptr, w.col, w.seed_batches[0].tolist(), [10, 5], 5)
    c = gpu_sample(B, torch_mod, w.row_ptr, w.col, w.seed_batches[0].tolist(), [10, 5], 6)
    assert np.array_equal(a["input_nodes"], b["input_nodes"])
    assert all(np.array_equal(x, y) for x, y in zip(a["col_local"], b["col_local"]))
    assert not np.array_equal(a["input_nodes"], c["input_nodes"])


def test_sample_reports_out_of_range_seed(B, torch_mod):
    rp, col = csr_from_adj(TINY_GRAPHS["path"])
    g = B.Graph(rp, col)
    s = B.Sampler(g, 3, [2])
    sb = s.sample(torch_mod.tensor([0, 9, 1], dtype=torch_mod.int32, device="cuda"), 1)
    torch_mod.cuda.synchronize()
    with pytest.raises(B.BglError) as e:
        sb.sizes()
    assert e.value.code == B.BGL_EINVAL


# --------------------------------------------------------------------- cache
def run_cache_stream(B, torch, feats, cap, batches, device_n_miss=False, side=True, write_through=False,
                     early=None, spare=0):
    """Feed id batches through GPU cache and oracle cache; compare after every call.
    early: "own" / "with_insert" / "alternate" = map lookup and lists on a stream of their own,
    on the one that also carries the FIFO updates, or only in every other call."""
    import oracle
    N, rb = feats.shape[0], feats.shape[1] * feats.itemsize
    feat_t = torch.from_numpy(feats.view(np.uint8).reshape(N, rb)).pin_memory()
    gc = B.Cache(cap, feat_t, num_nodes=N, row_bytes=rb)
    if spare:      # extra row positions in the buffer: slots, lookups and exported state must not change
        gc.set_spare_rows(spare)
    oc = oracle.Cache(cap, feats)
    if write_through:
        gc.set_write_through(True)
        device_n_miss = True
    side_stream = torch.cuda.Stream() if side else None
    lookup_stream = torch.cuda.Stream() if early else None
    for bi, ids in enumerate(batches):
        n = len(ids)
        ids_t = torch.tensor(ids, dtype=torch.int32, device="cuda") if n else torch.empty(1, dtype=torch.int32, device="cuda")
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
        gc.lookup_gather(ids_t, n, out, out_slot, miss_pos, side_stream=side_stream, lookup_stream=use_ls)
        o_out, o_slot, o_miss, o_hit = oc.lookup_gather(ids)
        if device_n_miss:
            gc.insert_fifo(ids_t, miss_pos, -1, out, stream=lookup_stream if early == "with_insert" else None)
            torch.cuda.synchronize()
            n_hit = int(gc.n_hit_host[0])
        else:
            torch.cuda.synchronize()
            n_hit = int(gc.n_hit_host[0])
            gc.insert_fifo(ids_t, miss_pos, n - n_hit, out)
        oc.insert_fifo(ids, o_miss, o_out)
        assert n_hit == o_hit, f"batch {bi}"
        assert np.array_equal(out_slot[:n].cpu().numpy(), o_slot), f"batch {bi}"
        assert np.array_equal(miss_pos[: n - n_hit].cpu().numpy(), o_miss), f"batch {bi}"
        assert np.array_equal(out[:n].cpu().numpy(), o_out), f"batch {bi}"
        assert_state_equal(gc, oc, f"batch {bi}")
    return gc, oc


def test_cache_hand_worked_example(B, torch_mod, golden_dir):
    lines = [l.strip() for l in open(os.path.join(golden_dir, "fifo_worked_example.txt"))
             if l.strip() and not l.startswith("#")]
    cap = int(lines[0].split()[1])
    batches, expect = [], []
    for l in lines[1:]:
        if l.startswith("batch"):
            parts = [p.split() for p in l[len("batch"):].split("|")]
            batches.append([int(x) for x in parts[0]])
            expect.append(([int(x) for x in parts[2]], int(parts[3][0])))
    feats = np.random.default_rng(0).standard_normal((16, 4)).astype(np.float32)
    gc, _ = run_cache_stream(B, torch_mod, feats, cap, batches)
    s2n, tail, _ = gc.export_state(False)
    assert s2n.tolist() == expect[-1][0] and tail == expect[-1][1]
    assert gc.stats()["hits"] == 2 and gc.stats()["lookups"] == 13


@pytest.mark.parametrize("dim,dtype", [(4, np.float32), (100, np.float32), (128, np.float32),
                                       (512, np.uint16), (12, np.float32), (264, np.uint16)])
@pytest.mark.parametrize("device_n_miss,spare", [(False, 0), (True, 0), (True, 777), (False, 6000)])
def test_cache_random_streams(B, torch_mod, dim, dtype, device_n_miss, spare):
    rng = np.random.default_rng(dim)
    N, cap = 20000, 3000
    if dtype == np.float32:
        feats = rng.standard_normal((N, dim)).astype(np.float32)
    else:
        feats = rng.integers(0, 2**16, (N, dim), dtype=np.uint16)
    batches = []
    for b in range(12):
        size = int(rng.integers(1, 2500)) if b != 5 else 7000  # batch 5: more misses than slots
        hot = rng.zipf(1.2, size) % N
        batches.append(list(dict.fromkeys(hot.tolist())))
    batches.insert(3, [])          # empty lookup
    batches.insert(8, batches[7])  # immediate repeat: all hits unless evicted
    run_cache_stream(B, torch_mod, feats, cap, batches, device_n_miss=device_n_miss, spare=spare)


@pytest.mark.parametrize("dim,dtype", [(4, np.float32), (100, np.float32), (512, np.uint16), (264, np.uint16)])
@pytest.mark.parametrize("side,spare", [(True, 0), (False, 0), (True, 1), (False, 2900), (True, 10000)])
def test_cache_write_through_mode(B, torch_mod, dim, dtype, side, spare):
    """The miss fetch fills the cache buffer itself; same results as the default mode,
    including a batch with more misses than slots, an empty batch and tiny capacities."""
    rng = np.random.default_rng(dim + 1)
    N = 20000
    feats = (rng.standard_normal((N, dim)).astype(np.float32) if dtype == np.float32
             else rng.integers(0, 2**16, (N, dim), dtype=np.uint16))
    batches = []
    for b in range(12):
        size = int(rng.integers(1, 2500)) if b != 5 else 7000
        batches.append(list(dict.fromkeys((rng.zipf(1.2, size) % N).tolist())))
    batches.insert(3, [])
    batches.insert(8, batches[7])
    run_cache_stream(B, torch_mod, feats, 3000, batches, side=side, write_through=True, spare=spare)
    run_cache_stream(B, torch_mod, feats, 1, batches[:6], side=side, write_through=True, spare=spare)


@pytest.mark.parametrize("early", ["own", "with_insert", "alternate"])
@pytest.mark.parametrize("side", [True, False])
def test_cache_early_lookup(B, torch_mod, early, side):
    """bgl_cache_lookup_gather_early: the map lookup and the lists on another stream than the hit
    gather and the miss fetch.  Same results as the plain call, also when the two kinds of call
    alternate, with batches of more misses than slots and an empty batch."""
    rng = np.random.default_rng(91)
    N = 20000
    feats = rng.standard_normal((N, 100)).astype(np.float32)
    batches = []
    for b in range(12):
        size = int(rng.integers(1, 2500)) if b != 5 else 7000
        batches.append(list(dict.fromkeys((rng.zipf(1.2, size) % N).tolist())))
    batches.insert(3, [])
    batches.insert(8, batches[7])
    run_cache_stream(B, torch_mod, feats, 3000, batches, side=side, write_through=True, early=early)
    run_cache_stream(B, torch_mod, feats, 64, batches[:7], side=side, write_through=True, early=early)


def test_cache_early_lookup_needs_write_through(B, torch_mod):
    torch = torch_mod
    feats = torch.zeros((100, 64), dtype=torch.uint8).pin_memory()
    gc = B.Cache(10, feats, num_nodes=100, row_bytes=64)
    ids = torch.arange(8, dtype=torch.int32, device="cuda")
    out = torch.zeros((8, 64), dtype=torch.uint8, device="cuda")
    slot = torch.zeros(8, dtype=torch.int32, device="cuda")
    mp = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(B.BglError) as e:
        gc.lookup_gather(ids, 8, out, slot, mp, lookup_stream=torch.cuda.Stream())
    assert e.value.code == B.BGL_EINVAL


def test_cache_write_through_rejects_a_broken_call_sequence(B, torch_mod):
    feats = np.zeros((50, 4), dtype=np.float32)
    feat_t = torch_mod.from_numpy(feats.view(np.uint8).reshape(50, 16)).pin_memory()
    gc = B.Cache(8, feat_t, num_nodes=50, row_bytes=16)
    gc.set_write_through(True)
    ids = torch_mod.arange(5, dtype=torch_mod.int32, device="cuda")
    other = torch_mod.arange(5, dtype=torch_mod.int32, device="cuda")
    out = torch_mod.empty((5, 16), dtype=torch_mod.uint8, device="cuda")
    out_slot = torch_mod.empty(5, dtype=torch_mod.int32, device="cuda")
    miss_pos = torch_mod.empty(5, dtype=torch_mod.int32, device="cuda")
    with pytest.raises(B.BglError):
        gc.insert_fifo(ids, miss_pos, -1, out)               # no lookup before it
    gc.lookup_gather(ids, 5, out, out_slot, miss_pos)
    with pytest.raises(B.BglError):
        gc.lookup_gather(ids, 5, out, out_slot, miss_pos)    # second lookup without the insert
    with pytest.raises(B.BglError):
        gc.insert_fifo(ids, miss_pos, 3, out)                # explicit count
    with pytest.raises(B.BglError):
        gc.insert_fifo(other, miss_pos, -1, out)             # other ids
    with pytest.raises(B.BglError):
        gc.set_write_through(False)                          # mode change while an insert is owed
    gc.insert_fifo(ids, miss_pos, -1, out)
    gc.set_write_through(False)
    s2n, tail, _ = gc.export_state(False)
    assert tail == 5 and s2n[:5].tolist() == [0, 1, 2, 3, 4]


def test_cache_single_stream_and_tiny_capacity(B, torch_mod):
    rng = np.random.default_rng(3)
    feats = rng.standard_normal((500, 8)).astype(np.float32)
    batches = [rng.permutation(500)[: int(rng.integers(1, 200))].tolist() for _ in range(15)]
    run_cache_stream(B, torch_mod, feats, 1, batches, side=False)
    run_cache_stream(B, torch_mod, feats, 17, batches, side=False)
    run_cache_stream(B, torch_mod, feats, 500, batches)


@pytest.mark.parametrize("write_through,early", [(False, None), (True, "with_insert")])
def test_cache_lookups_of_many_tiles(B, torch_mod, write_through, early):
    """Lookups of more than 4096 tiles of 256 ids: the list kernel then takes the tiles' prefix
    sums from a scan kernel instead of summing its predecessors' counts in every workgroup."""
    rng = np.random.default_rng(77)
    N, cap = 3_000_000, 1_200_000
    feats = rng.integers(0, 2**31, (N, 4), dtype=np.int32).view(np.float32)      # 16-byte rows, compared as bytes
    perm = rng.permutation(N).astype(np.int32)
    batches = [perm[:1_300_000], perm[900_000:2_000_001], perm[:1_048_576], perm[5:1_048_576], rng.permutation(N)[:2_100_000]]
    run_cache_stream(B, torch_mod, feats, cap, batches, device_n_miss=True, write_through=write_through, early=early)


def test_cache_long_churn_keeps_map_exact(B, torch_mod):
    """Many times the capacity flows through a small cache: every eviction blanks a
    map word and every insertion reuses one; lookups must stay exact."""
    rng = np.random.default_rng(5)
    N, cap = 50000, 1500
    feats = rng.standard_normal((N, 4)).astype(np.float32)
    batches = [rng.permutation(N)[:1400].tolist() for _ in range(60)]
    gc, oc = run_cache_stream(B, torch_mod, feats, cap, batches, device_n_miss=True)
    # full map check: look up every node id
    ids = torch_mod.arange(N, dtype=torch_mod.int32, device="cuda")
    out = torch_mod.empty((N, 16), dtype=torch_mod.uint8, device="cuda")
    out_slot = torch_mod.empty(N, dtype=torch_mod.int32, device="cuda")
    miss_pos = torch_mod.empty(N, dtype=torch_mod.int32, device="cuda")
    gc.lookup_gather(ids, N, out, out_slot, miss_pos)
    torch_mod.cuda.synchronize()
    assert np.array_equal(out_slot.cpu().numpy(), oc.node_to_slot)
    assert np.array_equal(out.cpu().numpy(), feats.view(np.uint8).reshape(N, 16))


@pytest.mark.parametrize("write_through", [False, True])
def test_cache_map_lookups_stay_short_under_fifo_churn(B, torch_mod, write_through):
    spare = 12345 if write_through else 0        # (with spare row positions in the buffer as well)
    """More than 300 times the capacity flows through a cache whose map is at its highest load
    (15,360 x 2 slots over 4,096 buckets of 15 words: load 1/2).  The cache engine of the paper
    serves a whole training job, so the cost of a lookup must not grow with the number of
    evictions: the bucket lines read per looked-up id stay near one, no higher at the end than
    right after the cache has filled, while lookups and state stay equal to the oracle's."""
    import oracle
    torch = torch_mod
    rng = np.random.default_rng(20211208)
    cap, N, per_batch, turnovers = 30720, 200_000, 20_000, 310
    feats = rng.integers(0, 2**31, (N, 4), dtype=np.int32).view(np.float32)      # 16-byte rows, compared as bytes
    feat_t = torch.from_numpy(feats.view(np.uint8).reshape(N, 16)).pin_memory()
    gc = B.Cache(cap, feat_t, num_nodes=N, row_bytes=16)
    gc.set_spare_rows(spare)
    gc.set_write_through(write_through)
    oc = oracle.Cache(cap, feats)
    out = torch.empty((per_batch, 16), dtype=torch.uint8, device="cuda")
    out_slot = torch.empty(per_batch, dtype=torch.int32, device="cuda")
    miss_pos = torch.empty(per_batch, dtype=torch.int32, device="cuda")
    assert gc.map_stats()["num_buckets"] * 15 == 2 * cap
    marks, b = [], 0
    while oc.tail < turnovers * cap:
        ids = rng.choice(N, per_batch, replace=False).astype(np.int32)
        ids_t = torch.from_numpy(ids).cuda()
        gc.lookup_gather(ids_t, per_batch, out, out_slot, miss_pos)
        gc.insert_fifo(ids_t, miss_pos, -1, out)
        gc.wait_rows()
        o_out, o_slot, o_miss, o_hit = oc.lookup_gather(ids)
        oc.insert_fifo(ids, o_miss, o_out)
        torch.cuda.synchronize()
        assert int(gc.n_hit_host[0]) == o_hit, f"batch {b}"
        assert np.array_equal(out_slot.cpu().numpy(), o_slot), f"batch {b}"
        if b % 40 == 0:
            assert np.array_equal(out.cpu().numpy(), o_out), f"batch {b}"
            assert_state_equal(gc, oc, f"batch {b}")
            ms = gc.map_stats()
            marks.append((oc.tail / cap, ms["ids_looked_up"], ms["bucket_lines_read"], ms["buckets_passed"], ms["passes"]))
        b += 1
    assert_state_equal(gc, oc, "end")
    ms = gc.map_stats()
    marks.append((oc.tail / cap, ms["ids_looked_up"], ms["bucket_lines_read"], ms["buckets_passed"], ms["passes"]))
    assert oc.tail >= 300 * cap
    # lines per id over the whole run, and between consecutive marks
    assert ms["lines_per_id"] <= 1.2, ms
    per_span = [(t1, (l1 - l0) / (i1 - i0)) for (t0, i0, l0, _, _), (t1, i1, l1, _, _) in zip(marks, marks[1:])]
    early_spans = [x for t, x in per_span if 2 <= t <= 40]
    late_spans = [x for t, x in per_span if t >= 270]
    assert early_spans and late_spans
    assert max(late_spans) <= 1.2 and max(late_spans) <= 1.02 * max(early_spans), (early_spans, late_spans)
    # buckets that some live entry is pushed past: a few per cent, not growing
    assert marks[-1][3] <= 0.10 * ms["num_buckets"], marks[-1]
    # the whole map against the oracle's: every node id looked up
    ids = torch.arange(N, dtype=torch.int32, device="cuda")
    big_out = torch.empty((N, 16), dtype=torch.uint8, device="cuda")
    big_slot = torch.empty(N, dtype=torch.int32, device="cuda")
    big_miss = torch.empty(N, dtype=torch.int32, device="cuda")
    gc.set_write_through(False)
    gc.lookup_gather(ids, N, big_out, big_slot, big_miss)
    gc.wait_rows()
    torch.cuda.synchronize()
    assert np.array_equal(big_slot.cpu().numpy(), oc.node_to_slot)
    assert np.array_equal(big_out.cpu().numpy(), feats.view(np.uint8).reshape(N, 16))
    assert ms["passes"] >= ms["buckets_passed"]      # (every such bucket has at least one entry pushed past it)


def test_cache_flags_out_of_range_id(B, torch_mod):
    feats = np.zeros((10, 4), dtype=np.float32)
    feat_t = torch_mod.from_numpy(feats.view(np.uint8).reshape(10, 16)).pin_memory()
    gc = B.Cache(4, feat_t, num_nodes=10, row_bytes=16)
    ids = torch_mod.tensor([1, 10, 2], dtype=torch_mod.int32, device="cuda")
    out = torch_mod.full((3, 16), 0x55, dtype=torch_mod.uint8, device="cuda")
    out_slot = torch_mod.empty(3, dtype=torch_mod.int32, device="cuda")
    miss_pos = torch_mod.empty(3, dtype=torch_mod.int32, device="cuda")
    gc.lookup_gather(ids, 3, out, out_slot, miss_pos)
    gc.insert_fifo(ids, miss_pos, -1, out)
    assert gc.stats()["status"] == B.BGL_EINVAL
    assert out[1].cpu().tolist() == [0x55] * 16  # untouched row


# ------------------------------------------------------------ whole pipeline
def run_config(cfg, n_batches, device_n_miss=False, check_every=1, write_through=False, w=None):
    if w is None:
        w = make_workload(cfg)
    gp = GpuPipeline(w, device_n_miss=device_n_miss, write_through=write_through)
    op = OraclePipeline(w)
    hits = total = 0
    for b in range(n_batches):
        full = (b % check_every == 0) or b == n_batches - 1
        g = gp.run_batch(w.seed_batches[b], w.rng_seeds[b], fetch=full)
        o = op.run_batch(w.seed_batches[b], w.rng_seeds[b])
        if full:
            assert_batch_equal(g, o, f"{cfg.name} batch {b}")
        else:
            assert g["n"] == o["n"] and g["n_hit"] == o["n_hit"], f"{cfg.name} batch {b}"
        hits += o["n_hit"]
        total += o["n"]
    assert_state_equal(gp.cache, op.cache, cfg.name)
    return hits / max(total, 1)


def test_pipeline_tiny_config_all_batches():
    cfg = _inputs().CONFIGS["tiny"]
    run_config(cfg, cfg.num_batches)
    run_config(cfg, cfg.num_batches, device_n_miss=True)
    run_config(cfg, cfg.num_batches, write_through=True)


def test_pipeline_mid_config_full_size():
    cfg = _inputs().CONFIGS["mid"]
    run_config(cfg, 12, device_n_miss=True, check_every=4)


@pytest.mark.parametrize("write_through", [False, True])
def test_overlapped_pipeline_as_benchmarked_matches_oracle(torch_mod, B, write_through):
    """The launch configuration bench.py times (two sampling workspaces, next batch sampled
    while the misses are fetched on the side stream, device-side miss count) on the
    full-size mid workload: every batch's outputs and the final cache state."""
    inputs = _inputs()
    w = inputs.make_workload(inputs.CONFIGS["mid"], pinned=True)
    run_overlapped_against_oracle(torch_mod, B, w, 8, write_through)


@pytest.mark.parametrize("config,staged", [("tiny", False), ("mid", False), ("mid", True), ("mid", 2), ("bfs", 2)])
def test_native_pipeline_matches_oracle(torch_mod, B, config, staged):
    """bgl_pipeline_run, the overlapped loop as one call into the library: every batch's sampled
    blocks, lists and rows (read in the per-batch callback) and the final cache state."""
    from helpers import make_workload
    w = make_workload(_inputs().CONFIGS[config], pinned=True)
    run_overlapped_against_oracle(torch_mod, B, w, 10, staged=staged, native=True)


def run_overlapped_against_oracle(torch_mod, B, w, steps, write_through=True, staged=False, native=False):
    """MinibatchPipeline as bench.py sets it up for the workload's configuration (graph placement
    included; staged: miss rows packed by host threads into a page-locked ring and moved by the copy
    engine, bench.py's default for large batches); every batch's sampled blocks, lists and rows, and
    the final cache state."""
    from paper_2112_08541_amd.pipeline import MinibatchPipeline
    cfg = w.cfg
    placement = B.BGL_HOST_PINNED if cfg.graph_placement == "host_pinned" else B.BGL_DEVICE
    graph = B.Graph(w.row_ptr, w.col, placement)
    cache = B.Cache(cfg.cache_rows, w.features.ctypes.data, num_nodes=cfg.num_nodes, row_bytes=cfg.row_bytes)
    if native:      # the same loop as one call into the library (bgl_pipeline_run)
        from paper_2112_08541_amd.pipeline import NativePipeline
        pipe = NativePipeline(graph, cache, cfg.batch, cfg.fanouts, cfg.row_bytes)
    else:
        pipe = MinibatchPipeline(graph, cache, cfg.batch, cfg.fanouts, cfg.row_bytes, write_through=write_through)
    if staged:
        pipe.tier = B.HostTier(w.features.view(np.uint8).reshape(cfg.num_nodes, cfg.row_bytes), 0, pipe.cap, 0)
        pipe.tier.set_copy_engine(int(staged))        # True: landed rows scattered; 2: the whole output in one pass
    seeds_dev = torch_mod.from_numpy(w.seed_batches).cuda()
    got = {}

    def grab(i, sb, n, p):
        torch_mod.cuda.synchronize()
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

    n_list, hit_list = pipe.run(seeds_dev, w.rng_seeds, steps, on_batch=grab)
    op = OraclePipeline(w)
    for b in range(steps):
        o = op.run_batch(w.seed_batches[b], w.rng_seeds[b])
        assert_batch_equal(got[b], o, f"overlapped batch {b}")
        assert n_list[b] == o["n"] and hit_list[b] == o["n_hit"]
    assert_state_equal(cache, op.cache, "overlapped")


def test_native_pipeline_argument_errors_and_second_pass(torch_mod, B):
    """bgl_pipeline_create refuses buffers that are too small; a second run over the same seeds (first_step
    past the seed batches) samples differently, as the Python loop does, and both loops agree on it."""
    import ctypes as C
    from paper_2112_08541_amd.pipeline import MinibatchPipeline, NativePipeline
    inputs = _inputs()
    cfg = inputs.CONFIGS["tiny"]
    w = inputs.make_workload(cfg, pinned=True)
    graph = B.Graph(w.row_ptr, w.col)
    seeds_dev = torch_mod.from_numpy(w.seed_batches).cuda()
    runs = []
    for cls in (NativePipeline, MinibatchPipeline):
        cache = B.Cache(cfg.cache_rows, w.features.ctypes.data, num_nodes=cfg.num_nodes, row_bytes=cfg.row_bytes)
        pipe = cls(graph, cache, cfg.batch, cfg.fanouts, cfg.row_bytes)
        first = pipe.run(seeds_dev, w.rng_seeds, cfg.num_batches)
        second = pipe.run(seeds_dev, w.rng_seeds, 7, first_step=cfg.num_batches)
        rows = pipe.out_rows[: second[0][-1]].cpu().numpy()
        ids = pipe.last_ids[: second[0][-1]].cpu().numpy()
        assert np.array_equal(rows, w.features.view(np.uint8).reshape(cfg.num_nodes, cfg.row_bytes)[ids])
        runs.append((first, second, ids.tolist(), cache.export_state(True)))
        if cls is NativePipeline:
            # too few output rows, and a sampling workspace that is too small
            buf = B.PipelineBuffers()
            for k, smp in enumerate(pipe.samplers):
                buf.workspace[k] = smp.workspace.data_ptr()
                buf.counts_host[k] = smp.counts_host.data_ptr()
            buf.workspace_bytes = pipe.samplers[0].workspace_bytes
            buf.out_rows, buf.out_slot, buf.miss_pos = (pipe.out_rows.data_ptr(), pipe.out_slot.data_ptr(),
                                                        pipe.miss_pos.data_ptr())
            buf.cap_rows = pipe.cap - 1
            h = C.c_void_p()
            fan = np.ascontiguousarray(cfg.fanouts, dtype=np.int32)
            args = (graph._h, cache._h, None, cfg.batch, fan.ctypes.data, len(fan))
            assert B.lib().bgl_pipeline_create(*args, C.byref(buf), 0, None, C.byref(h)) == B.BGL_ECAPACITY
            buf.cap_rows = pipe.cap
            buf.workspace_bytes = 1024
            assert B.lib().bgl_pipeline_create(*args, C.byref(buf), 0, None, C.byref(h)) == B.BGL_ECAPACITY
            assert not h.value
    (f0, s0, ids0, st0), (f1, s1, ids1, st1) = runs
    assert f0 == f1 and s0 == s1 and ids0 == ids1
    assert s0[0] != f0[0][:7]                       # the second pass sampled other neighbors
    for a, b in zip(st0, st1):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("miss_path", ["zero_copy", "staged", "staged_kernel", "staged_assembled",
                                       "native_zero_copy", "native_staged_assembled"])
def test_overlapped_pipeline_full_epoch_counts_and_final_state(torch_mod, B, miss_path):
    """The whole benchmarked epoch (mid, 200 batches, overlapped, write-through) on both miss
    paths (staged = the ring of a host tier that keeps nothing, with the early lookup, as
    bench.py runs it): per-batch input and hit counts, the last batch's rows, and the cache
    state at the end."""
    from paper_2112_08541_amd.pipeline import MinibatchPipeline
    inputs = _inputs()
    cfg = inputs.CONFIGS["mid"]
    w = inputs.make_workload(cfg, pinned=True)
    graph = B.Graph(w.row_ptr, w.col)
    cache = B.Cache(cfg.cache_rows, w.features.ctypes.data, num_nodes=cfg.num_nodes, row_bytes=cfg.row_bytes)
    if miss_path.startswith("native_"):     # the loop as one call into the library (bgl_pipeline_run)
        from paper_2112_08541_amd.pipeline import NativePipeline
        pipe = NativePipeline(graph, cache, cfg.batch, cfg.fanouts, cfg.row_bytes)
        miss_path = miss_path[len("native_"):]
    else:
        pipe = MinibatchPipeline(graph, cache, cfg.batch, cfg.fanouts, cfg.row_bytes)
    if miss_path != "zero_copy":
        tier = B.HostTier(w.features.view(np.uint8).reshape(cfg.num_nodes, cfg.row_bytes), 0, pipe.cap, 0)
        tier.set_copy_engine({"staged": 1, "staged_kernel": 0, "staged_assembled": 2}[miss_path])
        pipe.tier = tier
    seeds_dev = torch_mod.from_numpy(w.seed_batches).cuda()
    steps = cfg.num_batches

    def jitter(i, sb, n, p):
        # shift the streams against each other now and then (spin kernels that end by themselves)
        if i % 7 == 3:
            with torch_mod.cuda.stream(p.chain):
                torch_mod.cuda._sleep(3_000_000)
        if i % 5 == 1:
            with torch_mod.cuda.stream(p.work):
                torch_mod.cuda._sleep(3_000_000)

    n_list, hit_list = pipe.run(seeds_dev, w.rng_seeds, steps, on_batch=jitter)
    last_rows = pipe.out_rows[: n_list[-1]].cpu().numpy()
    last_ids = pipe.last_ids[: n_list[-1]].cpu().numpy()
    op = OraclePipeline(w)
    for b in range(steps):
        o = op.run_batch(w.seed_batches[b], w.rng_seeds[b])
        assert (n_list[b], hit_list[b]) == (o["n"], o["n_hit"]), f"batch {b}"
    assert np.array_equal(last_ids, o["input_nodes"])
    assert np.array_equal(last_rows, o["out_rows"])
    assert_state_equal(cache, op.cache, "full epoch")


def test_pipeline_bfs_order_config_full_size_and_locality():
    """The `bfs` configuration at full size: its seed order comes from the library's
    bgl_order_proximity (checked against the oracle's order when the workload is made), every
    compared batch equals the oracle's, and with the cache at 10 % of the nodes the proximity-aware
    order beats random order over the same training set by a clear margin (paper Sec. 3.2.2: the
    order is there to raise the FIFO hit ratio).  Cumulative hit ratios from an empty cache."""
    inputs = _inputs()
    po = run_config(inputs.CONFIGS["bfs"], 12, check_every=4)
    rnd = run_config(dataclasses.replace(inputs.CONFIGS["bfs"], order="random_train", name="bfs-random"),
                     12, check_every=4)
    assert po > 2.0 * rnd and po > rnd + 0.2, (po, rnd)


def test_pipeline_large_shape_scaled():
    """Large config's shape (int64 offsets, CSR read in place from page-locked host
    memory, 512-byte rows) at 1/50 of the node count."""
    inputs = _inputs()
    cfg = inputs.scaled(inputs.CONFIGS["large"], 2_220_000, num_batches=6)
    run_config(cfg, 6, check_every=2)


def test_pipeline_wide_shape_scaled():
    """Wide config's shape (bf16 x 512 rows, 4096 seeds, fanout 25/10) at 1/10 of the nodes."""
    inputs = _inputs()
    cfg = inputs.scaled(inputs.CONFIGS["wide"], 3_000_000, num_batches=4)
    run_config(cfg, 4, check_every=2)


# ------------------------------------------------ full-size large / wide
SKIP_FULL = os.environ.get("BGL_SKIP_FULL_SIZE", "") not in ("", "0")


def run_full(cfg, n_batches, check_every, overlapped_steps, torch_mod, B, other_steps=None):
    """One batch after the other with a check of every output, then the overlapped pipeline
    as bench.py runs this configuration, on the same full-size workload."""
    other_steps = other_steps or max(2, overlapped_steps // 2)
    try:
        w = _inputs().make_workload(cfg, pinned=True)
        run_config(cfg, n_batches, device_n_miss=True, check_every=check_every, w=w)
    except MemoryError as e:  # the box cannot page-lock this much host memory
        pytest.skip(f"not enough page-locked host memory for {cfg.name}: {e}")
    run_overlapped_against_oracle(torch_mod, B, w, overlapped_steps, staged=2)       # bench.py's default for it
    run_overlapped_against_oracle(torch_mod, B, w, other_steps, staged=True)          # --miss-path staged
    run_overlapped_against_oracle(torch_mod, B, w, other_steps)                       # and with --miss-path zero_copy


@pytest.mark.skipif(SKIP_FULL, reason="BGL_SKIP_FULL_SIZE is set")
def test_pipeline_wide_config_full_size(torch_mod, B):
    """30 M nodes, ~600 M edges, bf16 x 512 rows, 4,096 seeds, fanout 25/10, 4.5 M-row cache
    (~33 GB of page-locked host memory).  The overlapped run is long enough (30 batches of about
    180 K misses) for the cache to fill and wrap around: every batch's outputs and the final state
    are compared, so evictions and slots on both sides of the buffer's 4 GiB offset are."""
    run_full(_inputs().CONFIGS["wide"], 4, 2, 30, torch_mod, B, other_steps=3)


@pytest.mark.skipif(SKIP_FULL, reason="BGL_SKIP_FULL_SIZE is set")
def test_pipeline_large_config_full_size(torch_mod, B):
    """111 M nodes, ~1.6 B edges (int64 offsets, CSR read in place from page-locked host
    memory), fp32 x 128 rows, 25 M-row cache (~64 GB of page-locked host memory, ~30 s)."""
    run_full(_inputs().CONFIGS["large"], 3, 1, 6, torch_mod, B)


# ------------------------------------------------------ argument errors on the GPU side
def test_sample_workspace_and_argument_errors(B, torch_mod):
    import ctypes as C
    rp, col = csr_from_adj(TINY_GRAPHS["path"])
    g = B.Graph(rp, col)
    s = B.Sampler(g, 4, [2, 2])
    seeds = torch_mod.tensor([0, 1, 2, 3], dtype=torch_mod.int32, device="cuda")
    L = B.lib()
    st = B.SubgraphStruct()
    fan = s.fanouts.ctypes.data
    ws, nbytes = s.workspace.data_ptr(), s.workspace_bytes
    call = lambda **kw: L.bgl_sample_khop(kw.get("g", g._h), kw.get("seeds", seeds.data_ptr()), kw.get("n", 4),
                                          kw.get("fan", fan), kw.get("hops", 2), 1, kw.get("ws", ws),
                                          kw.get("bytes", nbytes), C.byref(st), None, None)
    assert call() == B.BGL_OK
    assert call(bytes=nbytes - 1) == B.BGL_ECAPACITY
    assert call(ws=ws + 64) == B.BGL_EINVAL          # not 256-byte aligned
    assert call(ws=None) == B.BGL_EINVAL
    assert call(seeds=None) == B.BGL_EINVAL
    assert call(hops=0) == B.BGL_EINVAL and call(hops=9) == B.BGL_EINVAL
    assert call(n=0) == B.BGL_EINVAL
    big = np.array([65, 2], dtype=np.int32)
    assert call(fan=big.ctypes.data) == B.BGL_EUNSUPPORTED
    torch_mod.cuda.synchronize()


def test_cache_argument_errors_and_device_resident_store(B, torch_mod):
    import oracle
    rng = np.random.default_rng(21)
    feats = rng.standard_normal((4000, 32)).astype(np.float32)            # 128-byte rows
    pageable = np.zeros((8, 4), dtype=np.float32)
    with pytest.raises(B.BglError) as e:
        B.Cache(4, pageable)                                               # not page-locked
    assert e.value.code == B.BGL_EINVAL
    # a backing store in device memory is accepted: the "fetch" is then an HBM gather
    dev_feats = torch_mod.from_numpy(feats.view(np.uint8).reshape(4000, 128)).cuda()
    gc = B.Cache(500, dev_feats, num_nodes=4000, row_bytes=128)
    oc = oracle.Cache(500, feats)
    out = torch_mod.empty((1500, 128), dtype=torch_mod.uint8, device="cuda")
    out_slot = torch_mod.empty(1500, dtype=torch_mod.int32, device="cuda")
    miss_pos = torch_mod.empty(1500, dtype=torch_mod.int32, device="cuda")
    for b in range(6):
        ids = rng.permutation(4000)[: int(rng.integers(1, 1500))].astype(np.int32)
        ids_t = torch_mod.from_numpy(ids).cuda()
        gc.lookup_gather(ids_t, len(ids), out, out_slot, miss_pos)
        gc.insert_fifo(ids_t, miss_pos, -1, out)
        o_out, o_slot, o_miss, o_hit = oc.lookup_gather(ids)
        oc.insert_fifo(ids, o_miss, o_out)
        torch_mod.cuda.synchronize()
        assert int(gc.n_hit_host[0]) == o_hit
        assert np.array_equal(out[: len(ids)].cpu().numpy(), o_out)
    assert_state_equal(gc, oc, "device store")
    # misaligned output rows, pageable hit counter
    L = B.lib()
    ids_t = torch_mod.arange(4, dtype=torch_mod.int32, device="cuda")
    assert L.bgl_cache_lookup_gather(gc._h, ids_t.data_ptr(), 4, out.data_ptr() + 8, out_slot.data_ptr(),
                                     miss_pos.data_ptr(), None, None, None) == B.BGL_EINVAL
    word = np.zeros(1, dtype=np.int64)
    assert L.bgl_cache_lookup_gather(gc._h, ids_t.data_ptr(), 4, out.data_ptr(), out_slot.data_ptr(),
                                     miss_pos.data_ptr(), word.ctypes.data, None, None) == B.BGL_EINVAL
    assert L.bgl_cache_lookup_gather(gc._h, ids_t.data_ptr(), -1, out.data_ptr(), out_slot.data_ptr(),
                                     miss_pos.data_ptr(), None, None, None) == B.BGL_EINVAL
    assert L.bgl_cache_profile(gc._h, 17, None, None) == B.BGL_EINVAL
    torch_mod.cuda.synchronize()


def test_bench_line_contract_on_the_tiny_config():
    """bench.py prints ONE JSON line with the agreed fields (here on the small configuration;
    the benchmark itself defaults to `mid`)."""
    import json
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--config", "tiny", "--steps", "20",
                        "--warmup", "3", "--cpu-batches", "5"], capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    r = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "host_link"):
        assert key in r, key
    assert r["n_gpus"] == 1 and r["steps"] == 20 and r["warmup"] == 3 and r["unit"] == "minibatches/s"
    assert r["vs_baseline"] is None and r["data"] == "synthetic" and "workload" in r["config"]
    assert abs(r["value"] - 1e3 / r["ms_per_step"]) < 1e-6 * r["value"]
    roof = r["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12 and roof["achieved"] > 0
    cpu = r["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] == 1 and cpu["value"] > 0 and cpu["unit"] == r["unit"]
    assert 0.0 < r["config"]["hit_ratio_cumulative"] < 1.0
    assert roof["launches"] == 20 // 4           # the hit gather is timed in every 4th batch
    rep = r["roofline_repeat_lookup"]
    assert rep["launches"] == 5 and 0.0 < rep["frac"] < 1.0


def test_stage_timers_count_their_launches_and_leave_results_alone(B, torch_mod):
    """bgl_cache_set_profiling / _every / bgl_cache_profile: every timed stage reports one launch per
    call (or per `every`-th call), with a plausible duration, and the rows are the table's."""
    torch = torch_mod
    rng = np.random.default_rng(11)
    N, cap, rb = 50_000, 8_000, 64
    table = torch.from_numpy(rng.integers(0, 256, (N, rb), dtype=np.uint8)).pin_memory()
    cache = B.Cache(cap, table, num_nodes=N, row_bytes=rb)
    out = torch.empty((6_000, rb), dtype=torch.uint8, device="cuda")
    slot = torch.empty(6_000, dtype=torch.int32, device="cuda")
    mpos = torch.empty(6_000, dtype=torch.int32, device="cuda")

    def batches(count):
        for _ in range(count):
            ids = torch.from_numpy(rng.permutation(N)[:6_000].astype(np.int32)).cuda()
            cache.lookup_gather(ids, 6_000, out, slot, mpos)
            cache.insert_fifo(ids, mpos, -1, out)
            torch.cuda.synchronize()
            assert torch.equal(out.cpu(), table[ids.cpu().long()])

    cache.set_profiling(True)
    batches(6)
    prof = cache.profile()
    for stage in B.STAGE_NAMES[:6]:            # (the seventh times a host tier's copies)
        ms, launches = prof[stage]
        assert launches == 6, stage
        assert 0.0 < ms < 50.0, (stage, ms)
    # only some stages, the hit gather in every 3rd lookup only (lookups are counted from creation: 7 .. 12)
    cache.set_profiling(("gather_hit", "fetch_miss"))
    cache.set_profiling_every("gather_hit", 3)
    batches(6)
    prof = cache.profile()
    assert prof["gather_hit"][1] == 2 and prof["fetch_miss"][1] == 6
    assert prof["probe"][1] == 0 and prof["insert_map"][1] == 0
    cache.set_profiling(False)
    batches(2)
    assert all(cache.profile()[stage][1] == 0 for stage in B.STAGE_NAMES)
    with pytest.raises(B.BglError):
        cache.set_profiling_every("gather_hit", 0)
    rc = B.lib().bgl_cache_set_profiling_every(cache._h, 99, 1)
    assert rc == B.BGL_EINVAL
