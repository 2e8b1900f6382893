"""The policy study's GPU leg against the oracle: its seed orders (bgl_order_proximity), its streams
of input nodes (bgl_sample_khop), its FIFO columns (the library's GPU cache) and its simulator columns
(static, LRU, LFU), every count compared with the oracle's definitions on a small workload."""
import dataclasses

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_policy_study_every_column_matches_the_oracle():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import oracle
    from oracle import policies as P
    from paper_2112_08541_amd import inputs, policy_study
    cfg = dataclasses.replace(inputs.CONFIGS["tiny"], batch=128, train_size=2048, po_sequences=3)
    row_ptr, col, _keep = inputs.make_graph(cfg)
    nb, fractions = 14, (0.02, 0.1, 0.3)
    r = policy_study.run_study(cfg, row_ptr, col, nb, fractions)
    N = cfg.num_nodes
    # the seed orders: random is a permutation of training nodes, proximity-aware is the oracle's order
    assert np.array_equal(r["order_po"].reshape(-1),
                          oracle.proximity_order(row_ptr, col, r["train"], r["roots"], r["shifts"], nb * cfg.batch))
    assert len(set(r["order_random"].reshape(-1).tolist())) == nb * cfg.batch
    assert set(r["order_random"].reshape(-1).tolist()) <= set(r["train"].tolist())
    # the streams: the input nodes of every batch, as the oracle samples them
    for name, seeds in (("random", r["order_random"]), ("po", r["order_po"])):
        assert len(r["streams"][name]) == nb
        for b in range(nb):
            sg = oracle.sample_khop(row_ptr, col, seeds[b], cfg.fanouts, int(r["rng_seeds"][b]))
            assert np.array_equal(r["streams"][name][b], sg.input_nodes), (name, b)
    # the static cache's content
    hottest = P.hottest_by_in_degree(col.tolist(), N)
    assert r["hottest"].tolist() == hottest
    assert r["capacities"] == [max(1, int(round(f * N))) for f in fractions]
    rand = [s.tolist() for s in r["streams"]["random"]]
    po = [s.tolist() for s in r["streams"]["po"]]
    feats = np.zeros((N, 4), dtype=np.float32)
    for cap in r["capacities"]:
        row = r["hits"][cap]
        assert row["static"] == sum(P.static_hits(rand, cap, hottest)), cap
        assert row["lru"] == sum(P.lru_hits(rand, cap)), cap
        assert row["lfu"] == sum(P.lfu_hits(rand, cap)), cap
        assert row["lru_po"] == sum(P.lru_hits(po, cap)), cap
        # the FIFO columns: the oracle's feature cache, and the policy definition beside it
        for column, stream in (("fifo_random", rand), ("fifo_po", po)):
            oc = oracle.Cache(cap, feats)
            for ids in stream:
                out, _, miss_pos, _ = oc.lookup_gather(ids)
                oc.insert_fifo(ids, miss_pos, out)
            assert row[column] == oc.stats()[1] == sum(P.fifo_hits(stream, cap)), (cap, column)
    # and the counts are not degenerate: hits happen, and grow with the cache
    small, large = r["hits"][r["capacities"][0]], r["hits"][r["capacities"][-1]]
    for c in policy_study.COLUMNS:
        assert 0 < large[c] and small[c] <= large[c], c
        assert all(r["overhead_ms"][cap][c] > 0 for cap in r["capacities"]), c
