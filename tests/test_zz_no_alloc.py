"""The lookup that allocates nothing (bgl_cache_lookup_gather_noalloc), through the C ABI, against
bgl_cache_lookup_gather on the same cache state and against the CPU oracle: out_slot, the miss list,
the hit count and every output byte equal, on calls in a row that share the library's fixed list
memory, the later ones with smaller inputs."""
import numpy as np
import pytest

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


def _both_lookups(B, torch, gc, ids_np, side):
    """The same ids through both entry points on the same cache state (a lookup changes nothing)."""
    n = len(ids_np)
    ids_t = torch.from_numpy(np.ascontiguousarray(ids_np, dtype=np.int32)).cuda() if n else \
        torch.empty(1, dtype=torch.int32, device="cuda")
    res = []
    for noalloc in (False, True):
        out = torch.full((max(n, 1), gc.row_bytes), 0xCD, dtype=torch.uint8, device="cuda")
        out_slot = torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda")
        miss_pos = torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda")
        gc.lookup_gather(ids_t, n, out, out_slot, miss_pos, side_stream=side, noalloc=noalloc)
        gc.wait_rows()
        torch.cuda.synchronize()
        n_hit = int(gc.n_hit_host[0])
        res.append((n_hit, out_slot[:n].cpu().numpy(), miss_pos[: n - n_hit].cpu().numpy(), out[:n].cpu().numpy(),
                    ids_t, out, miss_pos))
    return res


@pytest.mark.parametrize("dim,side", [(100, True), (128, False), (4, True)])
def test_noalloc_lookup_matches_the_allocating_one_and_the_oracle(B, torch_mod, dim, side):
    import oracle
    torch = torch_mod
    rng = np.random.default_rng(1000 + dim)
    N, cap = 60_000, 9_000
    feats = rng.standard_normal((N, dim)).astype(np.float32)
    rb = 4 * dim
    feat_t = torch.from_numpy(feats.view(np.uint8).reshape(N, rb)).pin_memory()
    gc = B.Cache(cap, feat_t, num_nodes=N, row_bytes=rb)
    oc = oracle.Cache(cap, feats)
    side_stream = torch.cuda.Stream() if side else None
    # sizes: large, smaller, empty, one id, several tiles with a ragged tail, more misses than slots, small again
    sizes = [7000, 1800, 0, 1, 2563, 12_000, 700]
    for bi, size in enumerate(sizes):
        ids = rng.permutation(N)[:size].astype(np.int32)
        if bi in (1, 4, 6) and size:                      # reuse ids of earlier batches: hits among the misses
            old = oc.slot_to_node[oc.slot_to_node >= 0]
            take = min(len(old), size // 2)
            ids[:take] = rng.permutation(old)[:take]
            ids = np.array(list(dict.fromkeys(ids.tolist())), dtype=np.int32)
        (h_a, slot_a, miss_a, out_a, *_), (h_b, slot_b, miss_b, out_b, ids_t, out_t, miss_t) = \
            _both_lookups(B, torch, gc, ids, side_stream)
        o_out, o_slot, o_miss, o_hit = oc.lookup_gather(ids)
        assert h_b == h_a == o_hit, f"batch {bi}"
        assert np.array_equal(slot_b, slot_a) and np.array_equal(slot_b, o_slot), f"batch {bi}"
        assert np.array_equal(miss_b, miss_a) and np.array_equal(miss_b, o_miss), f"batch {bi}"
        assert np.array_equal(out_b, out_a) and np.array_equal(out_b, o_out), f"batch {bi}"
        # the FIFO update follows the lookup that allocates nothing
        gc.insert_fifo(ids_t, miss_t, -1, out_t)
        oc.insert_fifo(ids, o_miss, o_out)
        torch.cuda.synchronize()
        s2n, tail, buf = gc.export_state(True)
        assert tail == oc.tail and np.array_equal(s2n, oc.slot_to_node), f"batch {bi}"
        occ = s2n >= 0
        assert np.array_equal(buf[occ], oc.buffer[occ]), f"batch {bi}"
    st = gc.stats()
    assert st["status"] == 0
    # both entry points count their lookups: every batch was looked up twice
    assert st["lookups"] == 2 * oc.stats()[0]


def test_noalloc_lookup_two_caches_share_the_list_memory(B, torch_mod):
    """Calls for two caches, one after the other on the same stream: the second overwrites the
    lists of the first, which by then has used them."""
    import oracle
    torch = torch_mod
    rng = np.random.default_rng(5)
    N = 20_000
    feats = rng.integers(0, 2**31, (N, 8), dtype=np.int32).view(np.float32)
    feat_t = torch.from_numpy(feats.view(np.uint8).reshape(N, 32)).pin_memory()
    caches = [(B.Cache(cap, feat_t, num_nodes=N, row_bytes=32), oracle.Cache(cap, feats)) for cap in (3000, 500)]
    bufs = [(torch.empty((4000, 32), dtype=torch.uint8, device="cuda"), torch.empty(4000, dtype=torch.int32, device="cuda"),
             torch.empty(4000, dtype=torch.int32, device="cuda")) for _ in caches]
    hits = torch.zeros(2, dtype=torch.int64).pin_memory()
    for bi in range(8):
        sizes = (int(rng.integers(1, 4000)), int(rng.integers(1, 4000)))
        idl = [rng.permutation(N)[:s].astype(np.int32) for s in sizes]
        idt = [torch.from_numpy(x).cuda() for x in idl]
        for k, (gc, _) in enumerate(caches):              # both calls enqueued before anything is read back
            out, slot, mp = bufs[k]
            gc.lookup_gather(idt[k], sizes[k], out, slot, mp, n_hit_ptr=hits.data_ptr() + 8 * k, noalloc=True)
            gc.insert_fifo(idt[k], mp, -1, out)
        torch.cuda.synchronize()
        for k, (gc, oc) in enumerate(caches):
            out, slot, mp = bufs[k]
            o_out, o_slot, o_miss, o_hit = oc.lookup_gather(idl[k])
            oc.insert_fifo(idl[k], o_miss, o_out)
            assert int(hits[k]) == o_hit, (bi, k)
            assert np.array_equal(slot[:sizes[k]].cpu().numpy(), o_slot), (bi, k)
            assert np.array_equal(mp[:sizes[k] - o_hit].cpu().numpy(), o_miss), (bi, k)
            assert np.array_equal(out[:sizes[k]].cpu().numpy(), o_out), (bi, k)


def test_noalloc_lookup_rejects_what_it_cannot_serve(B, torch_mod):
    torch = torch_mod
    feats = torch.zeros((100, 16), dtype=torch.uint8).pin_memory()
    gc = B.Cache(10, feats, num_nodes=100, row_bytes=16)
    n = B.BGL_NOALLOC_MAX_IDS + 1
    ids = torch.zeros(n, dtype=torch.int32, device="cuda")
    out = torch.empty((n, 16), dtype=torch.uint8, device="cuda")
    slot = torch.empty(n, dtype=torch.int32, device="cuda")
    mp = torch.empty(n, dtype=torch.int32, device="cuda")
    with pytest.raises(B.BglError) as e:
        gc.lookup_gather(ids, n, out, slot, mp, noalloc=True)
    assert e.value.code == B.BGL_ECAPACITY
    assert gc.stats()["lookups"] == 0                      # nothing was enqueued


def test_noalloc_lookup_at_its_maximum_size(B, torch_mod):
    """n = BGL_NOALLOC_MAX_IDS: more than 4,096 tiles, so the list kernel reads the tiles' prefix
    sums from the scan kernel, which live in the fixed array too."""
    import oracle
    torch = torch_mod
    rng = np.random.default_rng(9)
    n = B.BGL_NOALLOC_MAX_IDS
    N, cap = 2_000_000, 700_000
    feats = rng.integers(0, 2**31, (N, 4), dtype=np.int32).view(np.float32)
    feat_t = torch.from_numpy(feats.view(np.uint8).reshape(N, 16)).pin_memory()
    gc = B.Cache(cap, feat_t, num_nodes=N, row_bytes=16)
    oc = oracle.Cache(cap, feats)
    out = torch.empty((n, 16), dtype=torch.uint8, device="cuda")
    slot = torch.empty(n, dtype=torch.int32, device="cuda")
    mp = torch.empty(n, dtype=torch.int32, device="cuda")
    for size in (n, 300_001, n):
        ids = rng.permutation(N)[:size].astype(np.int32)
        ids_t = torch.from_numpy(ids).cuda()
        gc.lookup_gather(ids_t, size, out, slot, mp, noalloc=True)
        gc.insert_fifo(ids_t, mp, -1, out)
        torch.cuda.synchronize()
        o_out, o_slot, o_miss, o_hit = oc.lookup_gather(ids)
        oc.insert_fifo(ids, o_miss, o_out)
        assert int(gc.n_hit_host[0]) == o_hit
        assert np.array_equal(slot[:size].cpu().numpy(), o_slot)
        assert np.array_equal(mp[:size - o_hit].cpu().numpy(), o_miss)
        assert np.array_equal(out[:size].cpu().numpy(), o_out)
    s2n, tail, _ = gc.export_state(False)
    assert tail == oc.tail and np.array_equal(s2n, oc.slot_to_node)
