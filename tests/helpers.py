"""Shared drivers for the GPU-vs-oracle parity tests: run one minibatch through
the HIP library (via the binding, i.e. through the C ABI) and through the CPU
oracle, and compare everything bit for bit."""
import numpy as np


def proximity_order_checked(row_ptr, col, train_nodes, roots, shifts, num_out):
    """order_fn for inputs.make_workload: the proximity-aware seed order from the library's
    bgl_order_proximity (GPU), accepted only if it equals the oracle's."""
    import oracle
    from paper_2112_08541_amd import binding as B
    graph = B.Graph(row_ptr, col)
    got = B.order_proximity(graph, train_nodes, roots, shifts, num_out)
    graph.close()
    want = oracle.proximity_order(row_ptr, col, train_nodes, roots, shifts, num_out)
    assert np.array_equal(got, want), "bgl_order_proximity differs from the oracle's order"
    return got


def make_workload(cfg, pinned=True):
    """inputs.make_workload with the seed order of a proximity-ordered configuration computed by
    the library and checked against the oracle."""
    from paper_2112_08541_amd import inputs
    return inputs.make_workload(cfg, pinned=pinned, order_fn=proximity_order_checked if cfg.order == "po" else None)


class GpuPipeline:
    """sample_khop -> lookup_gather -> insert_fifo on the GPU for one workload."""

    def __init__(self, workload, cache_rows=None, placement=None, use_side_stream=True,
                 device_n_miss=False, write_through=False):
        import torch
        from paper_2112_08541_amd import binding as B
        self.torch, self.B = torch, B
        cfg = workload.cfg
        self.cfg = cfg
        if placement is None:
            placement = B.BGL_HOST_PINNED if cfg.graph_placement == "host_pinned" else B.BGL_DEVICE
        self.graph = B.Graph(workload.row_ptr, workload.col, placement)
        self.sampler = B.Sampler(self.graph, cfg.batch, cfg.fanouts)
        feats = workload.features
        self.feat_t = None
        for t in workload.keepalive:
            if t is not None and t.data_ptr() == feats.ctypes.data:
                self.feat_t = t
        if self.feat_t is None:  # not generated into pinned memory: make a pinned copy
            self.feat_t = torch.from_numpy(feats.view(np.uint8).reshape(feats.shape[0], -1)).pin_memory()
        self.cache = B.Cache(cache_rows or cfg.cache_rows, self.feat_t.data_ptr(),
                             num_nodes=cfg.num_nodes, row_bytes=cfg.row_bytes)
        K = len(cfg.fanouts)
        self.cap = int(min(cfg.num_nodes, cfg.batch * np.prod([1 + f for f in cfg.fanouts])))
        self.out_rows = torch.empty((self.cap, cfg.row_bytes), dtype=torch.uint8, device="cuda")
        self.out_slot = torch.empty(self.cap, dtype=torch.int32, device="cuda")
        self.miss_pos = torch.empty(self.cap, dtype=torch.int32, device="cuda")
        self.side = torch.cuda.Stream() if use_side_stream else None
        self.device_n_miss = device_n_miss or write_through
        if write_through:
            self.cache.set_write_through(True)

    def run_batch(self, seeds_np, rng_seed, fetch=True):
        torch = self.torch
        seeds = torch.from_numpy(np.ascontiguousarray(seeds_np, dtype=np.int32)).cuda()
        sb = self.sampler.sample(seeds, int(rng_seed))
        torch.cuda.current_stream().synchronize()
        nf, nnz = sb.sizes()
        n = int(nf[-1])
        ids = sb.input_nodes(self.cap)
        self.out_rows.fill_(0xAB)
        self.cache.lookup_gather(ids, n, self.out_rows, self.out_slot, self.miss_pos,
                                 side_stream=self.side)
        if self.device_n_miss:
            self.cache.insert_fifo(ids, self.miss_pos, -1, self.out_rows)
            self.cache.wait_rows()          # write-through mode: the insert does not wait for the fetch
            torch.cuda.current_stream().synchronize()
            n_hit = int(self.cache.n_hit_host[0])
        else:
            torch.cuda.current_stream().synchronize()
            n_hit = int(self.cache.n_hit_host[0])
            self.cache.insert_fifo(ids, self.miss_pos, n - n_hit, self.out_rows)
        res = dict(n_frontier=nf, nnz=nnz, n=n, n_hit=n_hit)
        if fetch:
            res["input_nodes"] = ids[:n].cpu().numpy()
            res["row_ptr"] = [sb.row_ptr(h, int(nf[h])).cpu().numpy() for h in range(len(nnz))]
            res["col_local"] = [sb.col_local(h, int(nnz[h])).cpu().numpy() for h in range(len(nnz))]
            res["out_slot"] = self.out_slot[:n].cpu().numpy()
            res["miss_pos"] = self.miss_pos[: n - n_hit].cpu().numpy()
            res["out_rows"] = self.out_rows[:n].cpu().numpy()
        return res


class OraclePipeline:
    """tier_rows > 0: a second cache level behind the first (oracle.TwoLevel)."""

    def __init__(self, workload, cache_rows=None, tier_rows=0):
        import oracle
        self.oracle = oracle
        self.w = workload
        self.two = oracle.TwoLevel(cache_rows or workload.cfg.cache_rows, tier_rows, workload.features)
        self.cache, self.tier = self.two.level1, self.two.level2

    def run_batch(self, seeds_np, rng_seed):
        cfg = self.w.cfg
        sg = self.oracle.sample_khop(self.w.row_ptr, self.w.col, seeds_np, cfg.fanouts, int(rng_seed))
        out, out_slot, miss_pos, n_hit, n_hit_tier = self.two.lookup_gather(sg.input_nodes)
        self.two.insert_fifo(sg.input_nodes, miss_pos, out)
        return dict(n_frontier=sg.n_frontier.astype(np.int64), nnz=np.array(sg.nnz, dtype=np.int64),
                    n=len(sg.input_nodes), n_hit=n_hit, n_hit_tier=n_hit_tier, input_nodes=sg.input_nodes,
                    row_ptr=sg.row_ptr, col_local=sg.col_local, out_slot=out_slot,
                    miss_pos=miss_pos, out_rows=out)


def assert_batch_equal(g, o, tag=""):
    assert g["n_frontier"].tolist() == o["n_frontier"].tolist(), tag
    assert g["nnz"].tolist() == o["nnz"].tolist(), tag
    assert np.array_equal(g["input_nodes"], o["input_nodes"]), tag
    for h in range(len(o["nnz"])):
        assert np.array_equal(g["row_ptr"][h], o["row_ptr"][h]), f"{tag} row_ptr hop {h}"
        assert np.array_equal(g["col_local"][h], o["col_local"][h]), f"{tag} col_local hop {h}"
    assert g["n_hit"] == o["n_hit"], tag
    assert np.array_equal(g["out_slot"], o["out_slot"]), tag
    assert np.array_equal(g["miss_pos"], o["miss_pos"]), tag
    assert np.array_equal(g["out_rows"], o["out_rows"]), tag


def assert_state_equal(gpu_cache, oracle_cache, tag=""):
    s2n, tail, buf = gpu_cache.export_state(True)
    assert tail == oracle_cache.tail, tag
    assert np.array_equal(s2n, oracle_cache.slot_to_node), tag
    occ = s2n >= 0
    assert np.array_equal(buf[occ], oracle_cache.buffer[occ]), tag
    st = gpu_cache.stats()
    lookups, hits = oracle_cache.stats()
    assert st["status"] == 0, tag
    assert (st["lookups"], st["hits"]) == (lookups, hits), tag
    assert st["inserts"] == tail
    assert st["evictions"] == max(0, tail - gpu_cache.capacity)
