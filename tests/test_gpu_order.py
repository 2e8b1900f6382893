"""GPU parity of the proximity-aware ordering calls against the CPU oracle:
the queue-order BFS sequence and the merged order are unique, so the comparison
is exact; the shuffling error is compared to 1e-12 (a mean of a few
hundred sums of ratios of integers, same operation order on both sides)."""
import os
import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2112_08541_amd import binding
    binding.lib()
    return binding


def random_graph(rng, N, max_deg, dtype=np.int32):
    deg = rng.integers(0, max_deg, N)
    rp = np.zeros(N + 1, dtype=dtype)
    rp[1:] = np.cumsum(deg)
    col = rng.integers(0, N, rp[-1]).astype(np.int32)
    return rp, col


def test_hand_worked_example(B, golden_dir):
    rp = np.array([0, 2, 3, 3, 4, 5, 5], dtype=np.int32)
    col = np.array([1, 2, 3, 0, 5], dtype=np.int32)
    g = B.Graph(rp, col)
    g2 = B.Graph(np.array([0, 2, 3, 3, 5, 5], dtype=np.int32), np.array([3, 1, 2, 4, 2], dtype=np.int32))
    for line in open(os.path.join(golden_dir, "po_worked_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        parts = [p.split() for p in line.split("|")]
        if parts[0][0] in ("bfs", "bfs2"):
            got = B.order_bfs_sequence(g if parts[0][0] == "bfs" else g2, [int(x) for x in parts[1]],
                                       int(parts[0][1]))
        else:
            got = B.order_proximity(g, list(range(6)), [int(x) for x in parts[0][2:]],
                                    [int(x) for x in parts[1][1:]], 6)
        assert got.tolist() == [int(x) for x in parts[2]]


@pytest.mark.parametrize("N,max_deg,dtype", [(7, 3, np.int32), (100, 2, np.int32), (1000, 3, np.int64),
                                             (5000, 8, np.int32), (70000, 4, np.int32), (33, 1, np.int32)])
def test_bfs_sequence_random_graphs(B, N, max_deg, dtype):
    """Sparse graphs: many components, isolated nodes, word-boundary sizes, restarts."""
    import oracle
    rng = np.random.default_rng(N)
    rp, col = random_graph(rng, N, max_deg, dtype)
    g = B.Graph(rp, col)
    for trial in range(3):
        train = rng.choice(N, max(1, N // (trial + 1)), replace=False)
        root = int(rng.integers(0, N))
        got = B.order_bfs_sequence(g, train, root)
        assert np.array_equal(got, oracle.bfs_sequence(rp, col, train, root))


def test_bfs_sequence_chain_of_open_components(B):
    """Several multi-node components that are only reachable by restarts, interleaved by id
    with closed singletons (the bulk restart must keep the sequential order)."""
    import oracle
    N = 40
    adj = [[] for _ in range(N)]
    adj[0] = [1]                      # root component {0,1}
    adj[5] = [30, 31]                 # open, reaches high ids
    adj[7] = [6]                      # open, reaches a smaller closed-looking id
    adj[6] = [1]                      # closed at first (points into the visited set)
    adj[20] = [21]; adj[21] = [22]; adj[22] = [20]   # a cycle
    adj[35] = [35]                    # self loop only: closed
    rp = np.zeros(N + 1, dtype=np.int32)
    rp[1:] = np.cumsum([len(a) for a in adj])
    col = np.array([u for a in adj for u in a], dtype=np.int32)
    g = B.Graph(rp, col)
    for root in (0, 22, 39):
        got = B.order_bfs_sequence(g, np.arange(N), root)
        assert got.tolist() == oracle.bfs_sequence(rp, col, np.arange(N), root).tolist()


def test_proximity_order_and_shuffling_error_mid_size(B):
    """The bfs configuration's graph at full size: 5 sequences over 204,800 training nodes."""
    import oracle
    from paper_2112_08541_amd import inputs
    cfg = inputs.CONFIGS["bfs"]
    rp, col, _ = inputs.make_graph(cfg)
    rng = np.random.default_rng(7)
    train = rng.choice(cfg.num_nodes, cfg.train_size, replace=False).astype(np.int32)
    roots = rng.integers(0, cfg.num_nodes, 5)
    shifts = rng.integers(0, len(train), 5)
    g = B.Graph(rp, col)
    t0 = time.perf_counter()
    got = B.order_proximity(g, train, roots, shifts, len(train))
    t_gpu = time.perf_counter() - t0
    t0 = time.perf_counter()
    want = oracle.proximity_order(rp, col, train, roots, shifts, len(train))
    t_cpu = time.perf_counter() - t0
    assert np.array_equal(got, want)
    print(f"proximity order, 5 sequences: GPU {t_gpu:.3f} s, oracle {t_cpu:.3f} s")
    labels = rng.integers(0, 47, cfg.num_nodes).astype(np.int32)
    gm, gx = B.order_shuffling_error(got, cfg.batch, labels, 47)
    om, ox = oracle.shuffling_error(want, cfg.batch, labels, 47)
    assert abs(gm - om) < 1e-12 and abs(gx - ox) < 1e-12


def test_host_pinned_graph_and_errors(B):
    import oracle
    import torch
    rng = np.random.default_rng(2)
    rp, col = random_graph(rng, 3000, 5, np.int64)
    g = B.Graph(torch.from_numpy(rp).pin_memory(), torch.from_numpy(col).pin_memory(), B.BGL_HOST_PINNED)
    train = rng.choice(3000, 500, replace=False)
    assert np.array_equal(B.order_bfs_sequence(g, train, 11), oracle.bfs_sequence(rp, col, train, 11))
    with pytest.raises(B.BglError):
        B.order_bfs_sequence(g, [1, 2, 2], 0)         # repeated id
    with pytest.raises(B.BglError):
        B.order_bfs_sequence(g, [1, 3000], 0)         # id out of range
    with pytest.raises(B.BglError):
        B.order_bfs_sequence(g, [1, 2], 3000)         # bad root
    with pytest.raises(B.BglError):
        B.order_proximity(g, [1, 2, 3], [0], [3], 3)  # shift out of range


def test_choose_sequences_matches_a_loop_over_the_oracle(B):
    import oracle
    rng = np.random.default_rng(12)
    N = 20000
    rp, col = random_graph(rng, N, 6)
    # labels follow the generation order of ids, so BFS from one root gives skewed batches
    labels = (np.arange(N) * 5 // N).astype(np.int32)
    train = rng.choice(N, 4000, replace=False).astype(np.int32)
    roots = rng.integers(0, N, 6)
    shifts = rng.integers(0, len(train), 6)
    g = B.Graph(rp, col)
    want_errs = []
    for s in range(1, 7):
        o = oracle.proximity_order(rp, col, train, roots[:s], shifts[:s], len(train))
        want_errs.append(oracle.shuffling_error(o, 100, labels, 5)[0])
    for threshold in (0.0, sorted(want_errs)[2], 1.0):
        chosen, errs, order = B.order_choose_sequences(g, train, roots, shifts, 100, labels, 5, threshold)
        expect = next((s for s in range(1, 7) if want_errs[s - 1] <= threshold), 6)
        assert chosen == expect
        assert np.allclose(errs, want_errs[:chosen], rtol=0, atol=1e-12)
        want = oracle.proximity_order(rp, col, train, roots[:chosen], shifts[:chosen], len(train))
        assert np.array_equal(order, want)
