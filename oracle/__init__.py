"""ctypes wrapper around the plain-C CPU oracle (``bgl_oracle.c``).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product package never does.
It shares nothing with the HIP library.  Citations of the paper sit on the C
functions; this file only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bgl_oracle.c")
_LIB = os.path.join(_HERE, "libbgl_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no OpenMP, no vectorising flags)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        u64, i64, i32, vp = C.c_uint64, C.c_int64, C.c_int32, C.c_void_p
        L.bglo_mix64.restype = u64
        L.bglo_mix64.argtypes = [u64]
        L.bglo_draw.restype = u64
        L.bglo_draw.argtypes = [u64, i32, i32, i32]
        L.bglo_hop_key.restype = u64
        L.bglo_hop_key.argtypes = [u64, i32]
        L.bglo_node_key.restype = u64
        L.bglo_node_key.argtypes = [u64, i32]
        L.bglo_slot_draw.restype = u64
        L.bglo_slot_draw.argtypes = [u64, i32]
        L.bglo_mulhi64.restype = u64
        L.bglo_mulhi64.argtypes = [u64, u64]
        L.bglo_floyd_from_t.restype = None
        L.bglo_floyd_from_t.argtypes = [i64, i32, vp, vp]
        L.bglo_sample_positions.restype = i32
        L.bglo_sample_positions.argtypes = [u64, i32, i32, i64, i32, vp]
        L.bglo_sample_khop.restype = C.c_int
        L.bglo_sample_khop.argtypes = [vp, C.c_int, vp, i64, vp, i32, vp, i32, u64,
                                       vp, i64, vp, vp, vp, vp, vp, vp]
        L.bglo_cache_create.restype = vp
        L.bglo_cache_create.argtypes = [i64, i32, vp, i64]
        L.bglo_cache_destroy.restype = None
        L.bglo_cache_destroy.argtypes = [vp]
        L.bglo_cache_lookup_gather.restype = i64
        L.bglo_cache_lookup_gather.argtypes = [vp, vp, i64, vp, vp, vp]
        L.bglo_cache_insert_fifo.restype = None
        L.bglo_cache_insert_fifo.argtypes = [vp, vp, vp, i64, vp]
        L.bglo_cache_tail.restype = u64
        L.bglo_cache_tail.argtypes = [vp]
        for name in ("bglo_cache_slot_to_node", "bglo_cache_node_to_slot", "bglo_cache_buffer"):
            getattr(L, name).restype = vp
            getattr(L, name).argtypes = [vp]
        L.bglo_cache_stats.restype = None
        L.bglo_cache_stats.argtypes = [vp, vp, vp]
        L.bglo_bfs_sequence.restype = i64
        L.bglo_bfs_sequence.argtypes = [vp, C.c_int, vp, i64, vp, i64, vp]
        L.bglo_po_merge.restype = C.c_int
        L.bglo_po_merge.argtypes = [vp, i64, i32, vp, i64, i64, vp]
        L.bglo_shuffling_error.restype = C.c_int
        L.bglo_shuffling_error.argtypes = [vp, i64, i32, vp, i32, vp, vp]
        _lib = L
    return _lib


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def mix64(z: int) -> int:
    return int(lib().bglo_mix64(z & (2**64 - 1)))


def draw(rng_seed: int, hop: int, node: int, slot: int) -> int:
    return int(lib().bglo_draw(rng_seed & (2**64 - 1), hop, node, slot))


def hop_key(rng_seed: int, hop: int) -> int:
    return int(lib().bglo_hop_key(rng_seed & (2**64 - 1), hop))


def node_key(hop_key_: int, node: int) -> int:
    return int(lib().bglo_node_key(hop_key_ & (2**64 - 1), node))


def slot_draw(node_key_: int, slot: int) -> int:
    return int(lib().bglo_slot_draw(node_key_ & (2**64 - 1), slot))


def mulhi64(x: int, m: int) -> int:
    return int(lib().bglo_mulhi64(x, m))


def floyd_from_t(d: int, k: int, t) -> np.ndarray:
    t = np.ascontiguousarray(t, dtype=np.int64)
    pos = np.zeros(k, dtype=np.int64)
    lib().bglo_floyd_from_t(d, k, _ptr(t), _ptr(pos))
    return pos


def sample_positions(rng_seed: int, hop: int, node: int, d: int, fanout: int) -> np.ndarray:
    pos = np.zeros(max(fanout, min(d, fanout), 1), dtype=np.int64)
    c = lib().bglo_sample_positions(rng_seed & (2**64 - 1), hop, node, d, fanout, _ptr(pos))
    return pos[:c].copy()


def frontier_bounds(num_seeds: int, fanouts, num_nodes: int):
    """Upper bounds |frontier_h| <= min(N, B * prod(1+f)) and per-hop edge bounds."""
    nf = [min(num_seeds, num_nodes)]
    ne = []
    for f in fanouts:
        ne.append(nf[-1] * f)
        nf.append(min(num_nodes, nf[-1] * (1 + f)))
    return nf, ne


class Subgraph:
    """Result of :func:`sample_khop` (numpy arrays trimmed to their real sizes)."""

    def __init__(self):
        self.input_nodes = None
        self.n_frontier = None
        self.row_ptr = []
        self.col_local = []
        self.col_global = []
        self.nnz = []


def sample_khop(row_ptr: np.ndarray, col: np.ndarray, seeds, fanouts, rng_seed: int) -> Subgraph:
    row_ptr = np.ascontiguousarray(row_ptr)
    assert row_ptr.dtype in (np.int32, np.int64)
    bits = 64 if row_ptr.dtype == np.int64 else 32
    col = np.ascontiguousarray(col, dtype=np.int32)
    seeds = np.ascontiguousarray(seeds, dtype=np.int32)
    fan = np.ascontiguousarray(fanouts, dtype=np.int32)
    K = len(fan)
    N = len(row_ptr) - 1
    nf, ne = frontier_bounds(len(seeds), [int(f) for f in fan], N)
    input_nodes = np.empty(max(nf[-1], 1), dtype=np.int32)
    n_frontier = np.zeros(K + 1, dtype=np.int32)
    rps = [np.zeros(nf[h] + 1, dtype=np.int32) for h in range(K)]
    cls = [np.empty(max(ne[h], 1), dtype=np.int32) for h in range(K)]
    cgs = [np.empty(max(ne[h], 1), dtype=np.int32) for h in range(K)]
    PtrArr = C.c_void_p * K
    cap_edges = np.array(ne, dtype=np.int64)
    nnz = np.zeros(K, dtype=np.int64)
    rc = lib().bglo_sample_khop(
        _ptr(row_ptr), bits, _ptr(col), N, _ptr(seeds), len(seeds), _ptr(fan), K,
        rng_seed & (2**64 - 1), _ptr(input_nodes), nf[-1], _ptr(n_frontier),
        C.cast(PtrArr(*[_ptr(a) for a in rps]), C.c_void_p),
        C.cast(PtrArr(*[_ptr(a) for a in cls]), C.c_void_p),
        C.cast(PtrArr(*[_ptr(a) for a in cgs]), C.c_void_p),
        _ptr(cap_edges), _ptr(nnz))
    if rc != 0:
        raise ValueError(f"bglo_sample_khop failed with status {rc}")
    sg = Subgraph()
    sg.n_frontier = n_frontier
    sg.input_nodes = input_nodes[: n_frontier[K]].copy()
    for h in range(K):
        e = int(nnz[h])
        sg.row_ptr.append(rps[h][: n_frontier[h] + 1].copy())
        sg.col_local.append(cls[h][:e].copy())
        sg.col_global.append(cgs[h][:e].copy())
        sg.nnz.append(e)
    return sg


class Cache:
    """FIFO feature cache over a host feature table given as a 2-D byte view."""

    def __init__(self, capacity_rows: int, features: np.ndarray):
        feats = features if features.flags.c_contiguous else np.ascontiguousarray(features)
        self._features = feats  # keep alive
        self.num_nodes = feats.shape[0]
        self.row_bytes = feats.strides[0]
        self.capacity = capacity_rows
        self._h = lib().bglo_cache_create(capacity_rows, self.row_bytes, _ptr(feats), self.num_nodes)
        if not self._h:
            raise ValueError("bglo_cache_create failed")

    def __del__(self):
        if getattr(self, "_h", None):
            lib().bglo_cache_destroy(self._h)
            self._h = None

    def lookup_gather(self, ids):
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        n = len(ids)
        out = np.empty((n, self.row_bytes), dtype=np.uint8)
        out_slot = np.empty(n, dtype=np.int32)
        miss_pos = np.empty(max(n, 1), dtype=np.int32)
        n_hit = lib().bglo_cache_lookup_gather(self._h, _ptr(ids), n, _ptr(out), _ptr(out_slot), _ptr(miss_pos))
        if n_hit == -2:
            raise ValueError("repeated id in one lookup: the ids of a call must be distinct")
        if n_hit < 0:
            raise ValueError("node id out of range")
        return out, out_slot, miss_pos[: n - n_hit].copy(), int(n_hit)

    def insert_fifo(self, ids, miss_pos, out_rows):
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        miss_pos = np.ascontiguousarray(miss_pos, dtype=np.int32)
        out_rows = np.ascontiguousarray(out_rows)
        lib().bglo_cache_insert_fifo(self._h, _ptr(ids), _ptr(miss_pos), len(miss_pos), _ptr(out_rows))

    @property
    def tail(self) -> int:
        return int(lib().bglo_cache_tail(self._h))

    def _view(self, fn, dtype, shape):
        p = getattr(lib(), fn)(self._h)
        n = int(np.prod(shape))
        buf = (C.c_uint8 * (n * np.dtype(dtype).itemsize)).from_address(p)
        return np.frombuffer(buf, dtype=dtype).reshape(shape).copy()

    @property
    def slot_to_node(self) -> np.ndarray:
        return self._view("bglo_cache_slot_to_node", np.int32, (self.capacity,))

    @property
    def node_to_slot(self) -> np.ndarray:
        return self._view("bglo_cache_node_to_slot", np.int32, (self.num_nodes,))

    @property
    def buffer(self) -> np.ndarray:
        return self._view("bglo_cache_buffer", np.uint8, (self.capacity, self.row_bytes))

    def stats(self):
        a, b = C.c_uint64(0), C.c_uint64(0)
        lib().bglo_cache_stats(self._h, C.addressof(a), C.addressof(b))
        return a.value, b.value


class TwoLevel:
    """The two cache levels of the paper's Sec. 3.2.3: a GPU cache, behind it a CPU cache with
    the same (FIFO) policy, behind that the feature store.  Reading taken where the paper omits
    the details: the second level sees the first level's misses of one call, in miss order, as
    one FIFO batch of its own: they are looked up against the second level's state at entry,
    then the ones it does not hold are inserted in that order (the rule of `Cache.insert_fifo`);
    a hit in either level does not renew anything.  The first level is updated by the caller
    afterwards, as in the one-level workflow.  capacity2 = 0: no second level."""

    def __init__(self, capacity1: int, capacity2: int, features: np.ndarray):
        self.level1 = Cache(capacity1, features)
        self.level2 = Cache(capacity2, features) if capacity2 > 0 else None

    def lookup_gather(self, ids):
        """Returns (rows, out_slot, miss_pos, hits in level 1, hits in level 2 among level 1's
        misses).  Level 2 is updated; level 1 is not (see insert_fifo)."""
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        out, out_slot, miss_pos, n_hit1 = self.level1.lookup_gather(ids)
        n_hit2 = 0
        if self.level2 is not None:
            missed = ids[miss_pos]
            rows2, _, miss2, n_hit2 = self.level2.lookup_gather(missed)
            self.level2.insert_fifo(missed, miss2, rows2)
            out[miss_pos] = rows2          # what level 2 or the store returned for level 1's misses
        return out, out_slot, miss_pos, n_hit1, n_hit2

    def insert_fifo(self, ids, miss_pos, out_rows):
        self.level1.insert_fifo(ids, miss_pos, out_rows)


def bfs_sequence(row_ptr: np.ndarray, col: np.ndarray, train_nodes, root: int) -> np.ndarray:
    """Training nodes in canonical BFS order from `root`: first-in first-out queue order, a
    node's neighbors entering the queue in the order of its CSR row, restart at the smallest
    unvisited id."""
    row_ptr = np.ascontiguousarray(row_ptr)
    bits = 64 if row_ptr.dtype == np.int64 else 32
    col = np.ascontiguousarray(col, dtype=np.int32)
    N = len(row_ptr) - 1
    is_train = np.zeros(N, dtype=np.uint8)
    is_train[np.asarray(train_nodes, dtype=np.int64)] = 1
    seq = np.empty(int(is_train.sum()), dtype=np.int32)
    n = lib().bglo_bfs_sequence(_ptr(row_ptr), bits, _ptr(col), N, _ptr(is_train), int(root), _ptr(seq))
    if n != len(seq):
        raise ValueError("bglo_bfs_sequence failed")
    return seq


def proximity_order(row_ptr, col, train_nodes, roots, shifts, num_out: int) -> np.ndarray:
    train_nodes = np.asarray(train_nodes, dtype=np.int32)
    seqs = np.concatenate([bfs_sequence(row_ptr, col, train_nodes, r) for r in roots]).astype(np.int32)
    shifts = np.ascontiguousarray(shifts, dtype=np.int64)
    order = np.empty(num_out, dtype=np.int32)
    rc = lib().bglo_po_merge(_ptr(seqs), len(train_nodes), len(roots), _ptr(shifts), len(row_ptr) - 1,
                             num_out, _ptr(order))
    if rc != 0:
        raise ValueError(f"bglo_po_merge failed with status {rc}")
    return order


def shuffling_error(order, batch: int, labels, num_classes: int):
    order = np.ascontiguousarray(order, dtype=np.int32)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    a, b = C.c_double(0), C.c_double(0)
    rc = lib().bglo_shuffling_error(_ptr(order), len(order), batch, _ptr(labels), num_classes,
                                    C.addressof(a), C.addressof(b))
    if rc != 0:
        raise ValueError("bglo_shuffling_error failed")
    return a.value, b.value
