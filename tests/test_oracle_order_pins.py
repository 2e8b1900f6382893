"""Pins of the proximity-aware-ordering part of the CPU oracle: a hand-worked
example, BFS levels against scipy's shortest paths, permutation and round-robin
properties, closed forms of the shuffling error.  CPU only."""
import os

import numpy as np
import pytest
import scipy.sparse as sp
from scipy.sparse.csgraph import breadth_first_order

import oracle

RP = np.array([0, 2, 3, 3, 4, 5, 5], dtype=np.int32)
COL = np.array([1, 2, 3, 0, 5], dtype=np.int32)
RP2 = np.array([0, 2, 3, 3, 5, 5], dtype=np.int32)     # 0->{3,1}, 1->{2}, 2->{}, 3->{4,2}, 4->{}
COL2 = np.array([3, 1, 2, 4, 2], dtype=np.int32)


def test_hand_worked_example(golden_dir):
    for line in open(os.path.join(golden_dir, "po_worked_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        parts = [p.split() for p in line.split("|")]
        if parts[0][0] in ("bfs", "bfs2"):
            rp, col = (RP, COL) if parts[0][0] == "bfs" else (RP2, COL2)
            got = oracle.bfs_sequence(rp, col, [int(x) for x in parts[1]], int(parts[0][1]))
            assert got.tolist() == [int(x) for x in parts[2]]
        else:
            roots = [int(x) for x in parts[0][2:]]
            shifts = [int(x) for x in parts[1][1:]]
            got = oracle.proximity_order(RP, COL, list(range(6)), roots, shifts, 6)
            assert got.tolist() == [int(x) for x in parts[2]]


def random_graph(rng, N, max_deg):
    deg = rng.integers(0, max_deg, N)
    rp = np.zeros(N + 1, dtype=np.int32)
    rp[1:] = np.cumsum(deg)
    col = rng.integers(0, N, rp[-1]).astype(np.int32)
    return rp, col


@pytest.mark.parametrize("seed", range(6))
def test_bfs_sequence_equals_scipy_breadth_first_order_run_by_run(seed):
    """Library special case: each traversal run must be scipy's breadth_first_order (the
    FIFO-queue traversal over CSR rows) from the run's root on the graph without the nodes
    of earlier runs; a new run starts at the smallest node not reached so far."""
    rng = np.random.default_rng(seed)
    N = int(rng.integers(30, 200))
    rp, col = random_graph(rng, N, 4)
    root = int(rng.integers(0, N))
    seq = oracle.bfs_sequence(rp, col, np.arange(N), root).tolist()
    assert sorted(seq) == list(range(N))
    done = np.zeros(N, dtype=bool)
    pos, start = 0, root
    while pos < N:
        # drop edges into nodes of earlier runs, keep row order, keep node numbering
        keep_e = ~done[col]
        rows = np.repeat(np.arange(N), np.diff(rp))
        rp2 = np.concatenate([[0], np.cumsum(np.bincount(rows[keep_e], minlength=N))]).astype(np.int32)
        A = sp.csr_matrix((np.ones(int(keep_e.sum())), col[keep_e], rp2), shape=(N, N))
        run = breadth_first_order(A, start, directed=True, return_predecessors=False).tolist()
        assert seq[pos: pos + len(run)] == run
        done[run] = True
        pos += len(run)
        if pos < N:
            start = int(np.nonzero(~done)[0][0])


def test_bfs_sequence_records_only_training_nodes_in_the_same_relative_order():
    rng = np.random.default_rng(9)
    rp, col = random_graph(rng, 300, 5)
    full = oracle.bfs_sequence(rp, col, np.arange(300), 17).tolist()
    train = rng.choice(300, 80, replace=False)
    part = oracle.bfs_sequence(rp, col, train, 17).tolist()
    tset = set(train.tolist())
    assert part == [v for v in full if v in tset]
    rp64 = rp.astype(np.int64)
    assert oracle.bfs_sequence(rp64, col, train, 17).tolist() == part


def test_proximity_order_properties():
    rng = np.random.default_rng(3)
    N = 500
    rp, col = random_graph(rng, N, 6)
    train = rng.choice(N, 200, replace=False)
    roots = [5, 77, 400]
    shifts = [0, 13, 199]
    order = oracle.proximity_order(rp, col, train, roots, shifts, 200)
    assert sorted(order.tolist()) == sorted(train.tolist())          # every training node once
    # one sequence, no shift: the merge is the sequence itself
    one = oracle.proximity_order(rp, col, train, [5], [0], 200)
    assert one.tolist() == oracle.bfs_sequence(rp, col, train, 5).tolist()
    # a shift is a rotation
    rot = oracle.proximity_order(rp, col, train, [5], [31], 200)
    assert rot.tolist() == np.roll(one, -31).tolist()
    # turn t comes from sequence t mod S: element 0 is sequence 0's first, element 1 is sequence 1's
    seqs = [np.roll(oracle.bfs_sequence(rp, col, train, r), -s) for r, s in zip(roots, shifts)]
    assert order[0] == seqs[0][0]
    firsts = [x for x in seqs[1] if x != order[0]]
    assert order[1] == firsts[0]
    # a prefix request is the prefix of the full order
    assert oracle.proximity_order(rp, col, train, roots, shifts, 64).tolist() == order[:64].tolist()


def test_shuffling_error_closed_forms():
    labels = np.array([0, 1] * 50, dtype=np.int32)           # node i has label i % 2
    order = np.arange(100, dtype=np.int32)
    # every batch of 10 holds 5 of each label: identical to the global distribution
    assert oracle.shuffling_error(order, 10, labels, 2) == (0.0, 0.0)
    # sorted by label: each batch is pure, global is (1/2, 1/2): TV = 1/2
    by_label = np.concatenate([np.arange(0, 100, 2), np.arange(1, 100, 2)]).astype(np.int32)
    m, x = oracle.shuffling_error(by_label, 10, labels, 2)
    assert abs(m - 0.5) < 1e-12 and abs(x - 0.5) < 1e-12
    # k equally likely labels, pure batches: TV = 1 - 1/k
    k = 5
    labels = (np.arange(100) % k).astype(np.int32)
    pure = np.concatenate([np.arange(c, 100, k) for c in range(k)]).astype(np.int32)
    m, x = oracle.shuffling_error(pure, 20, labels, k)
    assert abs(m - (1 - 1 / k)) < 1e-12
    # a random order sits in between and the mean is below the maximum
    rng = np.random.default_rng(0)
    m, x = oracle.shuffling_error(rng.permutation(100).astype(np.int32), 20, labels, k)
    assert 0.0 < m <= x < 1 - 1 / k
