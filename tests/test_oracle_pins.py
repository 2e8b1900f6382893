"""Pins of the CPU oracle against things other than itself: published vectors,
closed forms, exhaustive enumeration, brute-force invariants, textbook special
cases and an independently written FIFO model.  CPU only."""
import collections
import itertools
import math
import os

import numpy as np
import pytest

import oracle

M64 = 2**64 - 1


# --------------------------------------------------------------------------- RNG
def test_mix64_published_splitmix64_vectors(golden_dir):
    G = 0x9E3779B97F4A7C15
    n = 0
    for line in open(os.path.join(golden_dir, "splitmix64_vectors.txt")):
        if line.startswith("#") or not line.strip():
            continue
        vals = [int(x) for x in line.split()]
        state = vals[0]
        for expect in vals[1:]:
            state = (state + G) & M64
            assert oracle.mix64(state) == expect
            n += 1
    assert n == 6


def _unxorshift(z, s):
    x = z
    for _ in range(64 // s + 1):
        x = z ^ (x >> s)
    return x


def test_mix64_is_a_bijection_via_independent_inverse():
    # Inverse built from number theory (modular inverses of the odd multipliers,
    # inverse xor-shifts), not from the forward code.
    inv1 = pow(0xBF58476D1CE4E5B9, -1, 2**64)
    inv2 = pow(0x94D049BB133111EB, -1, 2**64)
    rng = np.random.default_rng(1)
    xs = [0, 1, M64, 2**63] + [int(x) for x in rng.integers(0, 2**64, 2000, dtype=np.uint64)]
    for x in xs:
        z = oracle.mix64(x)
        z = _unxorshift(z, 31)
        z = (z * inv2) & M64
        z = _unxorshift(z, 27)
        z = (z * inv1) & M64
        z = _unxorshift(z, 30)
        assert z == x


def test_mix64_avalanche():
    rng = np.random.default_rng(2)
    flips = []
    for x in rng.integers(0, 2**64, 300, dtype=np.uint64):
        x = int(x)
        b = int(rng.integers(0, 64))
        flips.append(bin(oracle.mix64(x) ^ oracle.mix64(x ^ (1 << b))).count("1"))
    assert 29.0 < np.mean(flips) < 35.0


def test_mulhi64_closed_form():
    rng = np.random.default_rng(3)
    xs = [0, 1, M64, 2**63, 2**32 - 1, 2**32] + [int(x) for x in rng.integers(0, 2**64, 500, dtype=np.uint64)]
    ms = [1, 2, 3, 15, 16, 2**31, 2**31 - 1, 2**32 + 7, 2**63, M64]
    for x in xs:
        for m in ms:
            assert oracle.mulhi64(x, m) == (x * m) >> 64
            assert oracle.mulhi64(x, m) < m


def test_draw_depends_on_every_key_component():
    base = oracle.draw(42, 1, 1000, 3)
    assert base != oracle.draw(43, 1, 1000, 3)
    assert base != oracle.draw(42, 2, 1000, 3)
    assert base != oracle.draw(42, 1, 1001, 3)
    assert base != oracle.draw(42, 1, 1000, 4)
    # hop and slot must not be interchangeable, nor node and slot
    assert oracle.draw(42, 1, 5, 2) != oracle.draw(42, 2, 5, 1)
    assert oracle.draw(42, 0, 7, 9) != oracle.draw(42, 0, 9, 7)
    seen = set()
    for hop in range(3):
        for node in range(40):
            for slot in range(25):
                seen.add(oracle.draw(7, hop, node, slot))
    assert len(seen) == 3 * 40 * 25


@pytest.mark.parametrize("vary", ["slot", "node", "hop_seed"])
def test_draw_top_bits_uniform(vary):
    # chi-square of the top 4 bits over 16,000 draws, 15 dof: 99.99% quantile ~ 44.3
    counts = np.zeros(16)
    for i in range(16000):
        if vary == "slot":
            w = oracle.draw(99, 0, 12345, i)
        elif vary == "node":
            w = oracle.draw(99, 1, i, 0)
        else:
            w = oracle.draw(i, i % 3, 77, 2)
        counts[w >> 60] += 1
    chi2 = ((counts - 1000.0) ** 2 / 1000.0).sum()
    assert chi2 < 44.3


# ------------------------------------------------------------------------- Floyd
@pytest.mark.parametrize("d,k", [(4, 2), (5, 3), (6, 2), (6, 5), (7, 3)])
def test_floyd_exhaustive_every_subset_equally_often(d, k):
    ranges = [range(d - k + s + 1) for s in range(k)]
    total = math.prod(len(r) for r in ranges)
    counts = collections.Counter()
    for t in itertools.product(*ranges):
        pos = oracle.floyd_from_t(d, k, list(t))
        assert len(set(pos.tolist())) == k
        assert pos.min() >= 0 and pos.max() < d
        counts[frozenset(pos.tolist())] += 1
    n_subsets = math.comb(d, k)
    assert len(counts) == n_subsets
    assert set(counts.values()) == {total // n_subsets}


def test_floyd_slot_order_rule():
    # d=10, k=3: J = 7, 8, 9.  t = [4, 4, 4] -> 4, then 4 is taken -> 8, then -> 9.
    assert oracle.floyd_from_t(10, 3, [4, 4, 4]).tolist() == [4, 8, 9]
    assert oracle.floyd_from_t(10, 3, [7, 8, 9]).tolist() == [7, 8, 9]
    assert oracle.floyd_from_t(10, 3, [0, 0, 8]).tolist() == [0, 8, 9]


def test_sample_positions_small_degree_keeps_row_in_order():
    for d in range(0, 8):
        pos = oracle.sample_positions(5, 0, 11, d, 7)
        assert pos.tolist() == list(range(d))


def test_sample_positions_validity_brute_force():
    rng = np.random.default_rng(4)
    for _ in range(400):
        d = int(rng.integers(1, 300))
        k = int(rng.integers(1, 30))
        pos = oracle.sample_positions(int(rng.integers(0, 2**63)), int(rng.integers(0, 3)),
                                      int(rng.integers(0, 10**6)), d, k)
        assert len(pos) == min(k, d)
        assert len(set(pos.tolist())) == len(pos)
        assert pos.min() >= 0 and pos.max() < d


@pytest.mark.parametrize("d,k", [(6, 5), (10, 5), (97, 15), (30, 15)])
def test_sample_positions_uniform_inclusion(d, k):
    trials = 20000
    counts = np.zeros(d)
    for s in range(trials):
        counts[oracle.sample_positions(s * 2654435761 + 17, 1, 31337, d, k)] += 1
    p = k / d
    # per-position binomial z-scores; 5.0 sigma over <= 97 positions
    z = (counts - trials * p) / math.sqrt(trials * p * (1 - p))
    assert np.abs(z).max() < 5.0
    if d == k + 1:
        left_out = trials - counts
        chi2 = ((left_out - trials / d) ** 2 / (trials / d)).sum()
        assert chi2 < 30.0  # 5 dof, far tail


# --------------------------------------------------------------------- k-hop
def csr_from_adj(adj, dtype=np.int32):
    rp = np.zeros(len(adj) + 1, dtype=dtype)
    col = []
    for i, row in enumerate(adj):
        col.extend(row)
        rp[i + 1] = len(col)
    return rp, np.array(col, dtype=np.int32)


def check_khop_invariants(rp, col, seeds, fanouts, sg):
    K = len(fanouts)
    uniq_seeds = list(dict.fromkeys(int(s) for s in seeds))
    nf = sg.n_frontier
    assert sg.input_nodes[: nf[0]].tolist() == uniq_seeds
    assert len(set(sg.input_nodes.tolist())) == len(sg.input_nodes) == nf[K]
    frontier_so_far = uniq_seeds
    for h in range(K):
        n_dst = nf[h]
        rph, cl, cg = sg.row_ptr[h], sg.col_local[h], sg.col_global[h]
        assert rph[0] == 0 and rph[-1] == sg.nnz[h] == len(cl)
        stream = list(frontier_so_far)
        for i in range(n_dst):
            v = int(sg.input_nodes[i])
            row = col[rp[v]: rp[v + 1]].tolist()
            got = cg[rph[i]: rph[i + 1]].tolist()
            assert len(got) == min(fanouts[h], len(row))
            # distinct edge positions => multiset inclusion in the CSR row
            need = collections.Counter(got)
            have = collections.Counter(row)
            assert all(have[u] >= c for u, c in need.items())
            stream.extend(got)
        # next frontier = order-preserving unique of (frontier ++ neighbors)
        frontier_so_far = list(dict.fromkeys(stream))
        assert sg.input_nodes[: nf[h + 1]].tolist() == frontier_so_far
        assert np.array_equal(sg.input_nodes[cl], cg)


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
def test_khop_invariants_tiny_graphs(name, dtype):
    rp, col = csr_from_adj(TINY_GRAPHS[name], dtype)
    N = len(rp) - 1
    for fanouts in ([2], [1, 1], [2, 2, 2], [3, 1], [10, 10]):
        for seed in range(6):
            seeds = [seed % N, (seed * 3 + 1) % N, seed % N]
            sg = oracle.sample_khop(rp, col, seeds, fanouts, 1000 + seed)
            check_khop_invariants(rp, col, seeds, fanouts, sg)


def test_khop_complete_graph_full_fanout_is_the_adjacency():
    adj = TINY_GRAPHS["clique6"]
    rp, col = csr_from_adj(adj)
    sg = oracle.sample_khop(rp, col, [0, 1, 2, 3, 4, 5], [5], 9)
    assert sg.row_ptr[0].tolist() == rp.tolist()
    assert sg.col_global[0].tolist() == col.tolist()
    assert sg.input_nodes.tolist() == [0, 1, 2, 3, 4, 5]
    assert sg.col_local[0].tolist() == col.tolist()


def test_khop_random_graphs_invariants_and_reachability_independence():
    rng = np.random.default_rng(5)
    for trial in range(30):
        N = int(rng.integers(5, 60))
        adj = [rng.integers(0, N, int(rng.integers(0, 12))).tolist() for _ in range(N)]
        rp, col = csr_from_adj(adj)
        fanouts = [int(f) for f in rng.integers(1, 6, int(rng.integers(1, 4)))]
        seeds = rng.integers(0, N, int(rng.integers(1, 8))).tolist()
        s = int(rng.integers(0, 2**62))
        sg = oracle.sample_khop(rp, col, seeds, fanouts, s)
        check_khop_invariants(rp, col, seeds, fanouts, sg)
        # the sample of (node, hop) does not depend on who else is in the batch
        a = seeds[0]
        alone = oracle.sample_khop(rp, col, [a], fanouts[:1], s)
        i = sg.input_nodes.tolist().index(a)
        assert (sg.col_global[0][sg.row_ptr[0][i]: sg.row_ptr[0][i + 1]].tolist()
                == alone.col_global[0].tolist())


def test_khop_neighbor_frequencies_uniform():
    # node 0 has 12 distinct neighbors, fanout 4: each is picked with probability 1/3
    adj = [list(range(1, 13))] + [[0]] * 12
    rp, col = csr_from_adj(adj)
    trials = 9000
    counts = np.zeros(13)
    for s in range(trials):
        sg = oracle.sample_khop(rp, col, [0], [4], s * 7919 + 3)
        counts[sg.col_global[0]] += 1
    assert counts[0] == 0
    z = (counts[1:] - trials / 3) / math.sqrt(trials * (1 / 3) * (2 / 3))
    assert np.abs(z).max() < 4.5


def test_khop_fanout_list_applies_front_to_back():
    # star centre as the seed: hop 0 uses fanouts[0]
    rp, col = csr_from_adj(TINY_GRAPHS["star"])
    sg = oracle.sample_khop(rp, col, [0], [3, 1], 1)
    assert sg.nnz[0] == 3 and sg.n_frontier[:2].tolist() == [1, 4]
    # hop 1 samples all 4 frontier nodes (the centre again, and the 3 leaves) with fanout 1;
    # the centre's fresh draw may or may not reach a new leaf
    assert sg.nnz[1] == 4 and sg.n_frontier[2] in (4, 5)
    # reversed list: 1 edge at the seed, then 2 nodes with fanout 3 (leaf has degree 1)
    sg = oracle.sample_khop(rp, col, [0], [1, 3], 1)
    assert sg.nnz[0] == 1 and sg.nnz[1] == 3 + 1


def test_khop_rejects_bad_arguments():
    rp, col = csr_from_adj(TINY_GRAPHS["path"])
    with pytest.raises(ValueError):
        oracle.sample_khop(rp, col, [7], [2], 1)
    with pytest.raises(ValueError):
        oracle.sample_khop(rp, col, [0], [0], 1)


# ----------------------------------------------------------------------- cache
def _features(N, dim, seed=0, dtype=np.float32):
    return np.random.default_rng(seed).standard_normal((N, dim)).astype(dtype)


def check_cache_invariants(c, total_inserted):
    s2n, n2s = c.slot_to_node, c.node_to_slot
    occ = s2n[s2n >= 0]
    assert len(set(occ.tolist())) == len(occ)
    assert len(occ) == min(c.tail, c.capacity)
    for s, v in enumerate(s2n):
        if v >= 0:
            assert n2s[v] == s
    assert (n2s >= 0).sum() == len(occ)
    assert set(occ.tolist()) == set(total_inserted[-min(c.tail, c.capacity):]) if total_inserted else True
    feats = c._features.view(np.uint8).reshape(c.num_nodes, -1)
    buf = c.buffer
    for s, v in enumerate(s2n):
        if v >= 0:
            assert np.array_equal(buf[s], feats[v])


def test_fifo_hand_worked_example(golden_dir):
    lines = [l.strip() for l in open(os.path.join(golden_dir, "fifo_worked_example.txt"))
             if l.strip() and not l.startswith("#")]
    cap = int(lines[0].split()[1])
    feats = _features(16, 4)
    fbytes = feats.view(np.uint8).reshape(16, -1)
    c = oracle.Cache(cap, feats)
    hits = lookups = 0
    for l in lines[1:]:
        if l.startswith("hits"):
            w = l.split()
            assert hits == int(w[1]) and lookups == int(w[3])
            continue
        parts = [p.split() for p in l[len("batch"):].split("|")]
        ids = [int(x) for x in parts[0]]
        out, out_slot, miss_pos, n_hit = c.lookup_gather(ids)
        assert out_slot.tolist() == [int(x) for x in parts[1]]
        assert np.array_equal(out, fbytes[ids])
        c.insert_fifo(ids, miss_pos, out)
        assert c.slot_to_node.tolist() == [int(x) for x in parts[2]]
        assert c.tail == int(parts[3][0])
        hits += n_hit
        lookups += len(ids)
    assert c.stats() == (13, 2)


class DequeFifo:
    """Independent FIFO model: a bounded queue of node ids plus a membership set."""

    def __init__(self, cap):
        self.cap, self.q, self.members = cap, collections.deque(), set()

    def batch(self, ids):
        hit = [i in self.members for i in ids]  # lookup sees the state at entry
        for i, h in zip(ids, hit):
            if not h:
                if len(self.q) == self.cap:
                    self.members.discard(self.q.popleft())
                self.q.append(i)
                self.members.add(i)
        return hit


@pytest.mark.parametrize("cap,N,batch", [(4, 12, 5), (50, 200, 40), (64, 100, 90), (7, 300, 30)])
def test_fifo_matches_independent_deque_model(cap, N, batch):
    rng = np.random.default_rng(cap)
    feats = _features(N, 8, seed=cap)
    fbytes = feats.view(np.uint8).reshape(N, -1)
    c = oracle.Cache(cap, feats)
    model = DequeFifo(cap)
    inserted = []
    for b in range(25):
        # zipf-ish popularity so that hits happen
        ids = list(dict.fromkeys((rng.zipf(1.3, batch) % N).tolist()))
        out, out_slot, miss_pos, n_hit = c.lookup_gather(ids)
        expect_hit = model.batch(ids)
        assert (out_slot >= 0).tolist() == expect_hit
        assert n_hit == sum(expect_hit)
        assert miss_pos.tolist() == [i for i, h in enumerate(expect_hit) if not h]
        assert np.array_equal(out, fbytes[ids])  # plain definition of the result
        c.insert_fifo(ids, miss_pos, out)
        inserted.extend(ids[i] for i in miss_pos)
        assert c.tail == len(inserted)
        check_cache_invariants(c, inserted)
        assert sorted(model.members) == sorted(c.slot_to_node[c.slot_to_node >= 0].tolist())


def test_fifo_closed_form_when_everything_fits():
    # capacity >= number of distinct ids: every distinct id misses exactly once
    rng = np.random.default_rng(8)
    N = 500
    feats = _features(N, 4)
    c = oracle.Cache(N, feats)
    total = hits = 0
    distinct = set()
    for b in range(40):
        ids = np.unique(rng.integers(0, N, 60)).tolist()
        rng.shuffle(ids)
        out, out_slot, miss_pos, n_hit = c.lookup_gather(ids)
        c.insert_fifo(ids, miss_pos, out)
        total += len(ids)
        hits += n_hit
        distinct.update(ids)
    assert hits == total - len(distinct)
    assert c.tail == len(distinct)


def test_fifo_slot_is_insertion_index_mod_capacity():
    feats = _features(40, 4)
    c = oracle.Cache(6, feats)
    order = []
    for ids in ([3, 9, 1], [9, 20, 21, 22], [30, 1, 31, 32, 33, 34, 35, 36, 37]):
        out, out_slot, miss_pos, _ = c.lookup_gather(ids)
        c.insert_fifo(ids, miss_pos, out)
        order.extend(ids[i] for i in miss_pos)
    s2n = c.slot_to_node
    for r, v in enumerate(order):
        if r >= len(order) - 6:
            assert s2n[r % 6] == v


def test_gather_bf16_sized_rows_and_bad_id():
    feats = np.random.default_rng(0).integers(0, 2**16, (30, 24), dtype=np.uint16)
    c = oracle.Cache(5, feats)
    ids = [7, 0, 29]
    out, _, miss_pos, _ = c.lookup_gather(ids)
    assert out.shape == (3, 48)
    assert np.array_equal(out.view(np.uint16), feats[ids])
    with pytest.raises(ValueError):
        c.lookup_gather([30])


# ---------------------------------------------------------------- key schedule
def _published_splitmix64(golden_dir):
    """(state seed, outputs) pairs of the published SplitMix64 check values."""
    out = []
    for line in open(os.path.join(golden_dir, "splitmix64_vectors.txt")):
        if line.startswith("#") or not line.strip():
            continue
        vals = [int(x) for x in line.split()]
        out.append((vals[0], vals[1:]))
    return out


def test_key_schedule_steps_are_published_splitmix64_outputs(golden_dir):
    """The hop key is output number hop+1 of SplitMix64 seeded with the call seed and a draw is
    output number slot+1 of SplitMix64 seeded with the node key: with the published seed both
    must reproduce the published outputs one by one (an off-by-one in either counter, or a
    constant other than the generator's increment, gives other numbers)."""
    G = 0x9E3779B97F4A7C15
    for seed, outputs in _published_splitmix64(golden_dir):
        for k, expect in enumerate(outputs):
            assert oracle.hop_key(seed, k) == expect
            assert oracle.slot_draw(seed, k) == expect
    seed, outputs = _published_splitmix64(golden_dir)[0]
    # the node key mixes (hop key XOR node) once: choose hop keys that land on the published states
    for node in (0, 1, 0x7FFFFFFF, 123456789):
        for k, expect in enumerate(outputs):
            state = (seed + (k + 1) * G) & M64
            assert oracle.node_key(state ^ node, node) == expect
    # xor, not addition: a node id that overlaps set bits of the key
    state = (seed + G) & M64
    node = int(state & 0x7FFFFFFF) | 1
    assert oracle.node_key(state ^ node, node) == outputs[0]
    assert oracle.node_key((state - node) & M64, node) != outputs[0]
    # and draw() is the three steps chained
    for key in ((1234567, 0, 0, 0), (1234567, 2, 99, 14), (2**64 - 1, 7, 2**31 - 1, 63)):
        s, h, v, sl = key
        assert oracle.draw(*key) == oracle.slot_draw(oracle.node_key(oracle.hop_key(s, h), v), sl)
    # seed 1234567, hop 0 and 1: the first two published outputs
    assert oracle.hop_key(1234567, 0) == 6457827717110365317
    assert oracle.hop_key(1234567, 1) == 3203168211198807973


def test_draw_golden_values(golden_dir):
    """Regression lock on the composed key schedule: values written by tests/golden/make_draw_golden.py
    (which calls only the oracle), checked here with Python integers."""
    G = 0x9E3779B97F4A7C15

    def mix(z):
        z ^= z >> 30
        z = (z * 0xBF58476D1CE4E5B9) & M64
        z ^= z >> 27
        z = (z * 0x94D049BB133111EB) & M64
        return z ^ (z >> 31)

    n = 0
    for line in open(os.path.join(golden_dir, "draw_values.txt")):
        if line.startswith("#") or not line.strip():
            continue
        seed, hop, node, slot, value = (int(x) for x in line.split())
        assert oracle.draw(seed, hop, node, slot) == value
        assert mix((mix(mix((seed + G * (hop + 1)) & M64) ^ node) + G * (slot + 1)) & M64) == value
        n += 1
    assert n >= 12


# ------------------------------------------------------------------ two levels
def test_lookup_rejects_a_repeated_id():
    feats = _features(20, 4)
    c = oracle.Cache(5, feats)
    with pytest.raises(ValueError, match="repeated"):
        c.lookup_gather([3, 4, 3])
    assert c.stats() == (0, 0)
    out, _, miss_pos, n_hit = c.lookup_gather([3, 4])       # the next call starts afresh
    assert n_hit == 0 and miss_pos.tolist() == [0, 1]
    c.insert_fifo([3, 4], miss_pos, out)
    assert c.lookup_gather([4, 3])[3] == 2


def test_two_level_hand_worked_example(golden_dir):
    lines = [l.strip() for l in open(os.path.join(golden_dir, "two_level_worked_example.txt"))
             if l.strip() and not l.startswith("#")]
    c1, c2 = (int(x) for x in lines[0].split()[1:])
    feats = _features(16, 4)
    fbytes = feats.view(np.uint8).reshape(16, -1)
    t = oracle.TwoLevel(c1, c2, feats)
    for l in lines[1:]:
        if not l.startswith("batch"):
            continue
        ids, slots, h2, s1, t1, s2, t2 = ([int(x) for x in p.split()] for p in l[len("batch"):].split("|"))
        out, out_slot, miss_pos, n_hit1, n_hit2 = t.lookup_gather(ids)
        assert out_slot.tolist() == slots
        assert n_hit1 == sum(s >= 0 for s in slots) and n_hit2 == h2[0]
        assert np.array_equal(out, fbytes[ids])
        t.insert_fifo(ids, miss_pos, out)
        assert t.level1.slot_to_node.tolist() == s1 and t.level1.tail == t1[0]
        assert t.level2.slot_to_node.tolist() == s2 and t.level2.tail == t2[0]
    tot = [int(x) for x in lines[-1].replace("hits", "").replace("lookups", "").split()]
    assert t.level1.stats() == (tot[2], tot[0]) and t.level2.stats() == (tot[3], tot[1])


@pytest.mark.parametrize("c1,c2,N,batch", [(4, 9, 40, 12), (30, 80, 400, 60), (50, 20, 300, 70), (1, 1, 10, 6)])
def test_two_level_matches_chained_deque_models(c1, c2, N, batch):
    """Two independent queue models chained the way Sec. 3.2.3 describes: the second one sees what
    the first one missed, in that order."""
    rng = np.random.default_rng(c1 * 1000 + c2)
    feats = _features(N, 8, seed=c2)
    fbytes = feats.view(np.uint8).reshape(N, -1)
    t = oracle.TwoLevel(c1, c2, feats)
    m1, m2 = DequeFifo(c1), DequeFifo(c2)
    for b in range(30):
        ids = list(dict.fromkeys((rng.zipf(1.3, batch) % N).tolist()))
        out, out_slot, miss_pos, n_hit1, n_hit2 = t.lookup_gather(ids)
        hit1 = m1.batch(ids)
        missed = [i for i, h in zip(ids, hit1) if not h]
        hit2 = m2.batch(missed)
        assert (out_slot >= 0).tolist() == hit1
        assert (n_hit1, n_hit2) == (sum(hit1), sum(hit2))
        assert np.array_equal(out, fbytes[ids])
        t.insert_fifo(ids, miss_pos, out)
        assert sorted(m1.members) == sorted(t.level1.slot_to_node[t.level1.slot_to_node >= 0].tolist())
        assert sorted(m2.members) == sorted(t.level2.slot_to_node[t.level2.slot_to_node >= 0].tolist())


def test_two_level_without_second_level_is_the_one_level_cache():
    feats = _features(60, 4)
    t, c = oracle.TwoLevel(7, 0, feats), oracle.Cache(7, feats)
    rng = np.random.default_rng(4)
    for b in range(10):
        ids = rng.permutation(60)[:15].tolist()
        out, out_slot, miss_pos, h1, h2 = t.lookup_gather(ids)
        o2, s2, m2, hh = c.lookup_gather(ids)
        assert h2 == 0 and h1 == hh and np.array_equal(out, o2) and np.array_equal(out_slot, s2)
        t.insert_fifo(ids, miss_pos, out)
        c.insert_fifo(ids, m2, o2)
    assert np.array_equal(t.level1.slot_to_node, c.slot_to_node)
