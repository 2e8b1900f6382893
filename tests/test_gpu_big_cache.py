"""GPU parity where the two largest configurations live: cache buffers of more than 4 GiB
(1,024-byte rows x 4.5 M slots: the `wide` shape; 512-byte rows x 9.5 M slots: the row width of
`large`), filled, wrapped around several times and evicted from by million-id batches, compared
with the CPU oracle after every call and byte by byte at the end, on both sides of the 4 GiB
offset.  The batches take turns through the five ways a miss row gets into the buffer: the FIFO
update's row copy, the write-through fetch from the page-locked table, the write-through
scatter of packed rows (landed by the copy engine, or read over the link), and the one pass that
writes the whole output and the landed miss rows' slots."""
import os

import numpy as np
import pytest

from helpers import assert_state_equal

pytestmark = pytest.mark.gpu

SKIP_FULL = os.environ.get("BGL_SKIP_FULL_SIZE", "") not in ("", "0")
MODES = ("row_copy", "write_through", "write_through_landed", "write_through_packed_over_link",
         "write_through_assembled")
TRANSPORT = {"write_through_landed": 1, "write_through_packed_over_link": 0, "write_through_assembled": 2}


@pytest.mark.skipif(SKIP_FULL, reason="BGL_SKIP_FULL_SIZE is set")
@pytest.mark.parametrize("row_bytes,cap,num_nodes,fresh,hits,turns,spare", [
    (1024, 4_500_000, 6_000_000, 800_000, 200_000, 4.2, 0),
    (512, 9_500_000, 12_000_000, 1_000_000, 250_000, 3.2, 1_250_000),   # spare row positions: slot != position
])
def test_cache_buffer_beyond_4gib_wraps_and_evicts(row_bytes, cap, num_nodes, fresh, hits, turns, spare):
    import torch
    import oracle
    from paper_2112_08541_amd import binding as B, inputs
    assert cap * row_bytes > (4 << 30) + (256 << 20)
    first_slot_past_4gib = (4 << 30) // row_bytes
    dim = row_bytes // 4
    cfg = inputs.Config("big-cache", num_nodes, 1.0, 4, dim, "f32", 1, (1,), cap, 1, "random_all", 0, seed=row_bytes)
    try:
        feats, keep = inputs.make_features(cfg, pinned=True)          # page-locked table of cheap synthetic rows
    except MemoryError as e:
        pytest.skip(f"not enough page-locked host memory: {e}")
    fb = feats.view(np.uint8).reshape(num_nodes, row_bytes)
    rng = np.random.default_rng(cap)
    gc = B.Cache(cap, feats.ctypes.data, num_nodes=num_nodes, row_bytes=row_bytes)
    gc.set_spare_rows(spare)
    oc = oracle.Cache(cap, feats)
    n_max = fresh + hits
    tier = B.HostTier(fb, 0, n_max, 0)                               # keeps nothing: the staging ring
    out = torch.empty((n_max, row_bytes), dtype=torch.uint8, device="cuda")
    out_slot = torch.empty(n_max, dtype=torch.int32, device="cuda")
    miss_pos = torch.empty(n_max, dtype=torch.int32, device="cuda")
    sweep = rng.permutation(num_nodes).astype(np.int32)              # ids not in the cache when their turn comes
    wrote_past_4gib = {m: False for m in MODES}
    b = past = 0
    while oc.tail < turns * cap:
        take = (np.arange(fresh, dtype=np.int64) + b * fresh) % num_nodes
        ids = sweep[take]
        held = oc.slot_to_node[oc.slot_to_node >= 0]
        if len(held):                                                 # ids the cache holds: hits, from every part of the buffer
            ids = np.concatenate([ids, rng.choice(held, size=min(hits, len(held)), replace=False)])
            ids = ids[rng.permutation(len(ids))]
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        n = len(ids)
        ids_t = torch.from_numpy(ids).cuda()
        # the modes take turns, separately over the batches whose insertions reach beyond 4 GiB (the swept ids
        # all miss, the held ones all hit, so where a batch's insertions go is known beforehand) and the others
        e0, e1 = oc.tail % cap, (oc.tail + fresh - 1) % cap
        if e1 < e0 or e1 >= first_slot_past_4gib:
            mode = MODES[past % len(MODES)]
            past += 1
        else:
            mode = MODES[b % len(MODES)]
        gc.set_write_through(mode != "row_copy")
        if mode in ("row_copy", "write_through"):
            gc.lookup_gather(ids_t, n, out, out_slot, miss_pos)
            gc.insert_fifo(ids_t, miss_pos, -1, out)
            gc.wait_rows()
            torch.cuda.synchronize()
            n_hit = int(gc.n_hit_host[0])
        else:
            tier.set_copy_engine(TRANSPORT[mode])
            n_hit, _ = gc.lookup_gather_tiered(tier, ids_t, n, out, out_slot, miss_pos)
            gc.insert_fifo(ids_t, miss_pos, -1, out)
            gc.wait_rows()
            torch.cuda.synchronize()
        o_out, o_slot, o_miss, o_hit = oc.lookup_gather(ids)
        tail0 = oc.tail
        oc.insert_fifo(ids, o_miss, o_out)
        assert n_hit == o_hit, f"batch {b} ({mode})"
        assert np.array_equal(out_slot[:n].cpu().numpy(), o_slot), f"batch {b} ({mode})"
        assert np.array_equal(miss_pos[: n - n_hit].cpu().numpy(), o_miss), f"batch {b} ({mode})"
        assert np.array_equal(out[:n].cpu().numpy(), o_out), f"batch {b} ({mode})"
        if tail0 >= cap:                                               # full: some of the hits came from beyond 4 GiB
            assert int(o_slot.max()) >= first_slot_past_4gib
        # which slots this batch's insertions went to
        s0, s1 = tail0 % cap, (oc.tail - 1) % cap
        if s1 < s0 or s1 >= first_slot_past_4gib:
            wrote_past_4gib[mode] = True
        b += 1
    assert all(wrote_past_4gib.values()), wrote_past_4gib
    assert oc.tail > 3 * cap                                           # wrapped around three times and more
    tier.close()
    # slot_to_node, tail, counters, and every byte of the buffer (all slots are occupied by now)
    assert (oc.slot_to_node >= 0).all()
    assert_state_equal(gc, oc, "end")
