"""The LRU / LFU / static simulators of the policy study against straightforward
Python models (CPU only)."""
import collections

import numpy as np
import pytest

from paper_2112_08541_amd.policy_study import PolicySim


def py_lru(batches, cap):
    od, hits = collections.OrderedDict(), 0
    for ids in batches:
        hits += sum(1 for v in ids if v in od)
        for v in ids:
            if v in od:
                od.move_to_end(v)
            else:
                if len(od) == cap:
                    od.popitem(last=False)
                od[v] = True
    return hits


def py_lfu(batches, cap):
    freq, last, hits, clock = {}, {}, 0, 0
    for ids in batches:
        hits += sum(1 for v in ids if v in freq)
        for v in ids:
            clock += 1
            if v in freq:
                freq[v] += 1
            else:
                if len(freq) == cap:
                    victim = min(freq, key=lambda u: (freq[u], last[u]))
                    del freq[victim], last[victim]
                freq[v] = 1
            last[v] = clock
    return hits


@pytest.mark.parametrize("cap", [1, 7, 50, 400])
def test_lru_and_lfu_match_python_models(cap):
    rng = np.random.default_rng(cap)
    N = 500
    batches = [list(dict.fromkeys((rng.zipf(1.3, 60) % N).tolist())) for _ in range(80)]
    for kind, model in (("lru", py_lru), ("lfu", py_lfu)):
        sim = PolicySim(kind, N, cap)
        assert sum(sim.batch(np.array(b, dtype=np.int32)) for b in batches) == model(batches, cap)


def test_static_counts_members_only():
    sim = PolicySim("static", 100, 3, hottest=np.array([5, 9, 2, 77], dtype=np.int32))
    assert sim.batch(np.array([5, 77, 2, 1], dtype=np.int32)) == 2
    assert sim.batch(np.array([9], dtype=np.int32)) == 1
