"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments in the calls that touch no GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2112_08541_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2112_08541_amd import buildlib
        buildlib.build_hip()
    return binding.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "bgl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bgl_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(L):
    from paper_2112_08541_amd import binding
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_no_entry_point_lets_an_exception_out():
    """The header promises that nothing throws: every int-returning entry point is a
    function-try-block that ends in the library's catch-all."""
    csrc = os.path.join(ROOT, "paper_2112_08541_amd", "csrc")
    seen = 0
    for name in sorted(os.listdir(csrc)):
        if not name.endswith(".hip"):
            continue
        text = open(os.path.join(csrc, name)).read()
        for m in re.finditer(r'^extern "C" int (bgl_[a-z_]+)\([^;{]*?\)\n(\S+)', text, re.M):
            assert m.group(2) == "try", (name, m.group(1))
            end = text.index("\n}", m.end())
            assert text[end:end + 20].startswith("\n} BGL_NOTHROW_END"), (name, m.group(1))
            seen += 1
    assert seen == len(declared_symbols()) - 1      # all but bgl_last_error, which returns a pointer


def test_the_five_entry_points_are_declared():
    names = declared_symbols()
    for n in ("bgl_graph_load_csr", "bgl_sample_khop", "bgl_cache_create",
              "bgl_cache_lookup_gather", "bgl_cache_insert_fifo"):
        assert n in names


def _ws_bytes(L, num_seeds, fanouts, num_nodes):
    fan = np.asarray(fanouts, dtype=np.int32)
    out = C.c_size_t(0)
    rc = L.bgl_sample_workspace_bytes(num_seeds, fan.ctypes.data if len(fan) else None, len(fan),
                                      num_nodes, C.byref(out))
    return rc, out.value


def test_workspace_bytes_and_argument_errors(L):
    from paper_2112_08541_amd import binding as B
    rc, small = _ws_bytes(L, 512, [10, 5], 10_000)
    assert rc == B.BGL_OK and small > 0
    rc, big = _ws_bytes(L, 1024, [15, 10, 5], 2_450_000)
    assert rc == B.BGL_OK and big > small
    # at least the outputs must fit: frontier bound 1024*16*11*6 ints
    assert big >= 4 * 1024 * 16 * 11 * 6
    assert _ws_bytes(L, 0, [5], 100)[0] == B.BGL_EINVAL
    assert _ws_bytes(L, 4, [], 100)[0] == B.BGL_EINVAL
    assert _ws_bytes(L, 4, [1] * 9, 100)[0] == B.BGL_EINVAL
    assert _ws_bytes(L, 4, [0], 100)[0] == B.BGL_EINVAL
    assert _ws_bytes(L, 4, [-3], 100)[0] == B.BGL_EINVAL
    assert _ws_bytes(L, 4, [65], 100)[0] == B.BGL_EUNSUPPORTED
    assert _ws_bytes(L, 4, [5], 0)[0] == B.BGL_EINVAL
    assert b"fanouts" in L.bgl_last_error() or b"num_nodes" in L.bgl_last_error()


def test_null_handles_are_rejected_without_touching_the_gpu(L):
    from paper_2112_08541_amd import binding as B
    assert L.bgl_sample_khop(None, None, 1, None, 1, 0, None, 0, None, None, None) == B.BGL_EINVAL
    assert L.bgl_cache_lookup_gather(None, None, 0, None, None, None, None, None, None) == B.BGL_EINVAL
    assert L.bgl_cache_insert_fifo(None, None, None, 0, None, None) == B.BGL_EINVAL
    assert L.bgl_cache_lookup_gather_early(None, None, 0, None, None, None, None, None, None, None) == B.BGL_EINVAL
    assert L.bgl_cache_lookup_gather_noalloc(None, None, 0, None, None, None, None, None, None) == B.BGL_EINVAL
    assert L.bgl_cache_export_state(None, None, None, None) == B.BGL_EINVAL
    assert L.bgl_cache_stats(None, None, None, None, None, None) == B.BGL_EINVAL
    assert L.bgl_cache_map_stats(None, None, None, None, None, None) == B.BGL_EINVAL
    assert L.bgl_cache_profile(None, 0, None, None) == B.BGL_EINVAL
    assert L.bgl_graph_destroy(None) == B.BGL_OK
    assert L.bgl_cache_destroy(None) == B.BGL_OK
    h = C.c_void_p()
    # argument validation happens before any device work
    rp = np.array([0, 1, 2], dtype=np.int32)
    col = np.array([1, 0], dtype=np.int32)
    assert L.bgl_graph_load_csr(None, 32, col.ctypes.data, 2, 2, 0, C.byref(h)) == B.BGL_EINVAL
    assert L.bgl_graph_load_csr(rp.ctypes.data, 16, col.ctypes.data, 2, 2, 0, C.byref(h)) == B.BGL_EINVAL
    assert L.bgl_graph_load_csr(rp.ctypes.data, 32, col.ctypes.data, 2, 3, 0, C.byref(h)) == B.BGL_EINVAL
    bad_rp = np.array([0, 2, 1], dtype=np.int32)
    assert L.bgl_graph_load_csr(bad_rp.ctypes.data, 32, col.ctypes.data, 2, 1, 0, C.byref(h)) == B.BGL_EINVAL
    bad_col = np.array([1, 2], dtype=np.int32)
    assert L.bgl_graph_load_csr(rp.ctypes.data, 32, bad_col.ctypes.data, 2, 2, 0, C.byref(h)) == B.BGL_EINVAL
    assert L.bgl_graph_load_csr(rp.ctypes.data, 32, col.ctypes.data, 2, 2, 7, C.byref(h)) == B.BGL_EINVAL
    assert (B.BGL_DEVICE, B.BGL_HOST_PINNED, B.BGL_HOST_PINNED_COL) == (0, 1, 2)
    feats = np.zeros((4, 4), dtype=np.float32)
    assert L.bgl_cache_create(0, 16, feats.ctypes.data, 4, C.byref(h)) == B.BGL_EINVAL
    assert L.bgl_cache_create(4, 20, feats.ctypes.data, 4, C.byref(h)) == B.BGL_EINVAL
    assert L.bgl_cache_create(4, 16, feats.ctypes.data + 4, 4, C.byref(h)) == B.BGL_EINVAL   # misaligned
    # host tier
    assert L.bgl_host_tier_create(None, 4, 16, 4, 4, 1, C.byref(h)) == B.BGL_EINVAL
    assert L.bgl_host_tier_create(feats.ctypes.data, 4, 20, 4, 4, 1, C.byref(h)) == B.BGL_EINVAL
    assert L.bgl_host_tier_create(feats.ctypes.data, 4, 16, -1, 4, 1, C.byref(h)) == B.BGL_EINVAL
    assert L.bgl_host_tier_create(feats.ctypes.data, 4, 16, 4, 0, 1, C.byref(h)) == B.BGL_EINVAL
    assert L.bgl_host_tier_create(feats.ctypes.data, 4, 16, 2**31 - 2, 8, 1, C.byref(h)) == B.BGL_EINVAL
    assert L.bgl_host_tier_create(feats.ctypes.data, 4, 16, 4, 4, -1, C.byref(h)) == B.BGL_EINVAL
    assert L.bgl_host_tier_destroy(None) == B.BGL_OK
    assert L.bgl_host_tier_export_state(None, None, None, None) == B.BGL_EINVAL
    assert L.bgl_host_tier_stats(None, None, None, None, None, None) == B.BGL_EINVAL
    assert L.bgl_host_tier_set_copy_engine(None, 1) == B.BGL_EINVAL
    assert L.bgl_cache_lookup_gather_tiered(None, None, None, 0, None, None, None, None, None, None, None, 0) == B.BGL_EINVAL
    assert L.bgl_cache_create(4, 16, feats.ctypes.data, 0, C.byref(h)) == B.BGL_EINVAL
    assert L.bgl_cache_lookup_tiered_begin(None, None, None, 0, None, None, None, None, None, None, None, 0) == B.BGL_EINVAL
    assert L.bgl_cache_lookup_tiered_finish(None) == B.BGL_EINVAL
    # the overlapped loop
    fan = np.array([2], dtype=np.int32)
    buf = B.PipelineBuffers()
    assert L.bgl_pipeline_create(None, None, None, 4, fan.ctypes.data, 1, C.byref(buf), 0, None, C.byref(h)) == B.BGL_EINVAL
    assert b"handle is null" in L.bgl_last_error()
    assert L.bgl_pipeline_create(None, None, None, 4, fan.ctypes.data, 1, C.byref(buf), 0, None, None) == B.BGL_EINVAL
    assert L.bgl_pipeline_destroy(None) == B.BGL_OK
    assert L.bgl_pipeline_set_cache(None, None, 0) == B.BGL_EINVAL
    assert L.bgl_pipeline_set_tier(None, None) == B.BGL_EINVAL
    assert L.bgl_pipeline_streams(None, None, None) == B.BGL_EINVAL
    assert L.bgl_pipeline_last_batch(None, None, None) == B.BGL_EINVAL
    assert L.bgl_pipeline_run(None, None, 0, None, 0, 0, None, None, None, C.cast(None, B.BATCH_FN), None) == B.BGL_EINVAL


def test_binding_refuses_to_run_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    from paper_2112_08541_amd import binding as B
    rp = np.array([0, 1, 2], dtype=np.int32)
    col = np.array([1, 0], dtype=np.int32)
    with pytest.raises(RuntimeError):
        B.Graph(rp, col)


def test_input_generator_is_seeded_and_shaped():
    from paper_2112_08541_amd import inputs
    cfg = inputs.CONFIGS["tiny"]
    a = inputs.make_workload(cfg)
    b = inputs.make_workload(cfg)
    assert np.array_equal(a.row_ptr, b.row_ptr) and np.array_equal(a.col, b.col)
    assert np.array_equal(a.features, b.features) and np.array_equal(a.seed_batches, b.seed_batches)
    assert a.seed_batches.shape == (20, 512) and a.rng_seeds.dtype == np.uint64
    deg = np.diff(a.row_ptr)
    assert deg.min() >= cfg.dmin and 9.0 < deg.mean() < 11.5
    assert a.col.min() >= 0 and a.col.max() < cfg.num_nodes
    assert all(len(set(r.tolist())) == cfg.batch for r in a.seed_batches)
    assert abs(float(a.features.mean())) < 0.01 and abs(float(a.features.std()) - 1.0) < 0.01
    # power-law in-degree: a few hubs collect far more than the mean
    indeg = np.bincount(a.col, minlength=cfg.num_nodes)
    assert indeg.max() > 20 * indeg.mean()


def test_proximity_order_uses_each_training_node_once():
    from paper_2112_08541_amd import inputs
    import dataclasses
    cfg = dataclasses.replace(inputs.scaled(inputs.CONFIGS["bfs"], 50_000, num_batches=10), batch=64)
    import oracle
    rp, col, _ = inputs.make_graph(cfg)
    with pytest.raises(ValueError):
        inputs.make_seed_batches(cfg)                       # the order is the method's, not the generator's
    seeds, draws = inputs.make_seed_batches(
        cfg, lambda train, roots, shifts, num_out: oracle.proximity_order(rp, col, train, roots, shifts, num_out))
    assert seeds.shape == (10, 64)
    flat = seeds.reshape(-1)
    assert len(np.unique(flat)) == len(flat)
    assert set(flat.tolist()) <= set(draws["train"].tolist()) and len(draws["roots"]) == cfg.po_sequences


def test_generated_graph_has_the_locality_breadth_first_orders_need():
    """Short-range edges on the generator's hidden ring: a breadth-first traversal from one node needs
    many levels to reach the graph (an expander would need three or four), and ids carry no locality."""
    import dataclasses
    import scipy.sparse as sp
    import scipy.sparse.csgraph as csg
    from paper_2112_08541_amd import inputs
    cfg = dataclasses.replace(inputs.scaled(inputs.CONFIGS["mid"], 400_000, num_batches=4), num_hubs=2)
    rp, col, _ = inputs.make_graph(cfg)
    N = cfg.num_nodes
    g = sp.csr_matrix((np.ones(len(col), dtype=np.int8), col, rp), shape=(N, N))
    dist = csg.shortest_path(g, method="D", unweighted=True, indices=[12345])[0]
    reached = np.isfinite(dist)
    assert reached.mean() > 0.95
    assert np.percentile(dist[reached], 50) >= 6
    # neighbors are not close in id: the ring positions are hidden behind a permutation
    v = np.repeat(np.arange(N), np.diff(rp))[:200000]
    assert np.median(np.abs(col[:200000].astype(np.int64) - v)) > N / 20


def test_bench_refuses_more_than_one_gpu():
    """This build runs on exactly one GPU: bench.py --gpus N > 1 must say so and exit."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""
