"""Pins of the oracle's policy definitions (oracle/policies.py) against a hand-worked example,
closed forms and textbook special cases, and of the product's fast simulators against them.
CPU only."""
import os

import numpy as np
import pytest

import oracle
from oracle import policies as P


def _golden(golden_dir):
    cap = nodes = None
    col = hottest = None
    batches, expect = [], []
    for line in open(os.path.join(golden_dir, "policies_worked_example.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, rest = line.split(None, 1)
        if key == "capacity":
            cap = int(rest)
        elif key == "nodes":
            nodes = int(rest)
        elif key == "col":
            col = [int(x) for x in rest.split()]
        elif key == "hottest":
            hottest = [int(x) for x in rest.split()]
        elif key == "batch":
            ids, hits = rest.split("|")
            batches.append([int(x) for x in ids.split()])
            expect.append([int(x) for x in hits.split()])
    return cap, nodes, col, hottest, batches, np.array(expect)


def test_policies_hand_worked_example(golden_dir):
    cap, nodes, col, hottest, batches, expect = _golden(golden_dir)
    assert P.hottest_by_in_degree(col, nodes) == hottest
    assert P.static_hits(batches, cap, hottest) == expect[:, 0].tolist()
    assert P.fifo_hits(batches, cap) == expect[:, 1].tolist()
    assert P.lru_hits(batches, cap) == expect[:, 2].tolist()
    assert P.lfu_hits(batches, cap) == expect[:, 3].tolist()


def test_in_degree_order_equals_a_library_count():
    rng = np.random.default_rng(3)
    col = rng.zipf(1.5, 5000) % 300
    order = P.hottest_by_in_degree(col.tolist(), 300)
    deg = np.bincount(col, minlength=300)
    assert order == np.lexsort((np.arange(300), -deg)).tolist()


@pytest.mark.parametrize("policy", [P.fifo_hits, P.lru_hits, P.lfu_hits])
def test_dynamic_policies_closed_forms(policy):
    rng = np.random.default_rng(11)
    N = 400
    batches = [np.unique(rng.integers(0, N, 50)).tolist() for _ in range(40)]
    total = sum(len(b) for b in batches)
    distinct = len(set(v for b in batches for v in b))
    # everything fits: every distinct id misses exactly once, whatever the policy
    assert sum(policy(batches, N)) == total - distinct
    # a stream that never repeats an id never hits
    fresh = [list(range(k * 30, (k + 1) * 30)) for k in range(20)]
    assert sum(policy(fresh, 50)) == 0
    # one id asked for again and again hits every time but the first
    assert policy([[7]] * 9, 1) == [0] + [1] * 8


def test_lru_is_the_stack_distance_rule_on_single_accesses():
    """Textbook characterisation: with one id per batch, an access hits in an LRU cache of capacity c
    iff fewer than c distinct other ids were accessed since the same id's previous access."""
    rng = np.random.default_rng(5)
    stream = (rng.zipf(1.4, 3000) % 60).tolist()
    for cap in (1, 3, 10, 59):
        expect, last = [], {}
        for t, v in enumerate(stream):
            if v in last:
                expect.append(1 if len(set(stream[last[v] + 1:t])) < cap else 0)
            else:
                expect.append(0)
            last[v] = t
        assert P.lru_hits([[v] for v in stream], cap) == expect


def test_fifo_definition_equals_the_oracle_cache():
    """The FIFO hit counter of the policy definitions and the oracle's FIFO feature cache are two
    independent statements of the same rule."""
    rng = np.random.default_rng(8)
    N = 300
    feats = rng.standard_normal((N, 4)).astype(np.float32)
    for cap in (1, 5, 40, 299):
        batches = [list(dict.fromkeys((rng.zipf(1.3, 70) % N).tolist())) for _ in range(30)]
        c = oracle.Cache(cap, feats)
        hits = []
        for ids in batches:
            out, _, miss_pos, n_hit = c.lookup_gather(ids)
            c.insert_fifo(ids, miss_pos, out)
            hits.append(n_hit)
        assert hits == P.fifo_hits(batches, cap)


def test_lfu_keeps_the_often_used_id_lru_the_recent_one():
    # ids 1 (used often, long ago) and 2 (used once, recently); 3 arrives in a cache of two
    warm = [[1]] * 5 + [[2]]
    assert P.lfu_hits(warm + [[3], [1]], 2)[-1] == 1 and P.lfu_hits(warm + [[3], [2]], 2)[-1] == 0
    assert P.lru_hits(warm + [[3], [1]], 2)[-1] == 0 and P.lru_hits(warm + [[3], [2]], 2)[-1] == 1


@pytest.mark.parametrize("cap", [1, 7, 50, 400])
def test_product_simulators_match_the_definitions(cap):
    from paper_2112_08541_amd.policy_study import PolicySim
    rng = np.random.default_rng(cap)
    N = 500
    batches = [list(dict.fromkeys((rng.zipf(1.3, 60) % N).tolist())) for _ in range(80)]
    col = (rng.zipf(1.4, 4000) % N).astype(np.int32)
    hottest = np.array(P.hottest_by_in_degree(col.tolist(), N), dtype=np.int32)
    for kind, definition in (("lru", P.lru_hits), ("lfu", P.lfu_hits)):
        sim = PolicySim(kind, N, cap)
        assert [sim.batch(np.array(b, dtype=np.int32)) for b in batches] == definition(batches, cap)
    sim = PolicySim("static", N, cap, hottest)
    assert [sim.batch(np.array(b, dtype=np.int32)) for b in batches] == P.static_hits(batches, cap, hottest)


def test_static_simulator_counts_members_only():
    from paper_2112_08541_amd.policy_study import PolicySim
    sim = PolicySim("static", 100, 3, hottest=np.array([5, 9, 2, 77], dtype=np.int32))
    assert sim.batch(np.array([5, 77, 2, 1], dtype=np.int32)) == 2
    assert sim.batch(np.array([9], dtype=np.int32)) == 1
