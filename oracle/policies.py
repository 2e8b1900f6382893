"""Plain definitions of the cache policies the BGL paper compares its FIFO cache with
(Sec. 2.3: the static cache of PaGraph, which holds the nodes of highest degree and never
changes; Sec. 3.2.1: the dynamic policies LRU and LFU, and FIFO itself), as hit counters over a
stream of batches of distinct node ids.

TEST INFRASTRUCTURE ONLY, like the rest of this package: pure Python, one dictionary or list per
policy, no attempt at speed.  The product's simulators (csrc/policy_sim.c) and its GPU cache are
checked against these.

Common reading (the paper compares hit ratios per minibatch and says no more): a batch is looked
up against the cache as it is when the batch arrives; then the batch's ids update the cache one
after the other, in batch order.  That is the rule of the FIFO cache (lookup, then insertion of
the misses), applied to every policy alike.
"""
from __future__ import annotations

import collections
from typing import Iterable, List, Sequence


def hottest_by_in_degree(col: Sequence[int], num_nodes: int) -> List[int]:
    """Node ids by falling in-degree (how often a node appears as a neighbor in the CSR's column
    array), ties by rising id: the order in which a static degree-based cache (Sec. 2.3) is filled."""
    deg = [0] * num_nodes
    for u in col:
        deg[int(u)] += 1
    return sorted(range(num_nodes), key=lambda v: (-deg[v], v))


def static_hits(batches: Iterable[Sequence[int]], capacity: int, hottest: Sequence[int]) -> List[int]:
    """Static cache: the first `capacity` ids of `hottest`, fixed for the whole run."""
    members = set(int(v) for v in hottest[:capacity])
    return [sum(1 for v in ids if int(v) in members) for ids in batches]


def fifo_hits(batches: Iterable[Sequence[int]], capacity: int) -> List[int]:
    """First in, first out: a miss enters at the back of a queue of `capacity` ids, the id at
    the front leaves; a hit changes nothing (Sec. 3.2.1)."""
    queue, members, out = collections.deque(), set(), []
    for ids in batches:
        hit = [int(v) in members for v in ids]
        out.append(sum(hit))
        for v, h in zip(ids, hit):
            if h:
                continue
            if len(queue) == capacity:
                members.discard(queue.popleft())
            queue.append(int(v))
            members.add(int(v))
    return out


def lru_hits(batches: Iterable[Sequence[int]], capacity: int) -> List[int]:
    """Least recently used: every access, hit or miss, makes the id the most recent one; when a
    new id needs room the least recent one leaves."""
    order, out = collections.OrderedDict(), []          # oldest first
    for ids in batches:
        out.append(sum(1 for v in ids if int(v) in order))
        for v in ids:
            v = int(v)
            if v in order:
                order.move_to_end(v)
            else:
                if len(order) == capacity:
                    order.popitem(last=False)
                order[v] = True
    return out


def lfu_hits(batches: Iterable[Sequence[int]], capacity: int) -> List[int]:
    """Least frequently used: every cached id counts its accesses since it entered; when a new id
    needs room the id with the fewest leaves, among equals the one accessed longest ago.  A new id
    enters with a count of one."""
    count, last, clock, out = {}, {}, 0, []
    for ids in batches:
        out.append(sum(1 for v in ids if int(v) in count))
        for v in ids:
            v = int(v)
            clock += 1
            if v in count:
                count[v] += 1
            else:
                if len(count) == capacity:
                    victim = min(count, key=lambda u: (count[u], last[u]))
                    del count[victim], last[victim]
                count[v] = 1
            last[v] = clock
    return out
