"""Seeded synthetic workloads shaped like the paper's datasets (Table 2 of the
paper: node/edge counts and feature widths of Ogbn-products and Ogbn-papers;
batch size and fanouts of its Sec. 5.1).  None of those datasets is used: the
graphs here are generated power-law graphs with the same shapes.

This module only produces *inputs* (graphs, feature tables, seed lists, one
64-bit RNG seed per batch).  It contains nothing of the sampling or caching
method, so both the HIP library's tests and the CPU oracle's tests can be fed
from it.  It imports neither of them.
"""
from __future__ import annotations

import ctypes as C
import dataclasses
import os
import subprocess
from typing import Callable, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csrc", "gen_inputs.c")
_LIB = os.path.join(_HERE, "libbgl_gen.so")


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _gen() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        L = C.CDLL(_LIB)
        i64, i32, u64, vp, dbl = C.c_int64, C.c_int32, C.c_uint64, C.c_void_p, C.c_double
        L.bglgen_degrees.restype = i64
        L.bglgen_degrees.argtypes = [i64, dbl, i64, i64, u64, vp]
        L.bglgen_row_ptr.restype = i64
        L.bglgen_row_ptr.argtypes = [i64, vp, vp, C.c_int]
        L.bglgen_permutation.restype = None
        L.bglgen_permutation.argtypes = [i64, u64, vp, vp]
        L.bglgen_edges.restype = C.c_int
        L.bglgen_edges.argtypes = [i64, vp, C.c_int, vp, u64, i64, dbl, dbl, i64, vp, vp]
        L.bglgen_features.restype = C.c_int
        L.bglgen_features.argtypes = [i64, i32, i32, u64, vp]
        _lib = L
    return _lib


@dataclasses.dataclass(frozen=True)
class Config:
    """One benchmark/parity configuration (tiny, mid, bfs, large, wide)."""
    name: str
    num_nodes: int
    mean_degree: float
    dmax: int
    feat_dim: int
    feat_dtype: str            # "f32" | "bf16"
    batch: int
    fanouts: tuple
    cache_rows: int
    num_batches: int
    order: str                 # "random_all" | "random_train" | "po"
    train_size: int
    row_ptr_bits: int = 32
    graph_placement: str = "device"   # "device" | "host_pinned"
    seed: int = 20211208
    reach: int = 2000          # mean distance of a short-range edge on the generator's hidden ring
    p_local: float = 0.97      # share of short-range edges; the others go to hubs
    beta: float = 0.75         # Zipf exponent over the hub ranks
    num_hubs: int = 0          # 0: one hub per 16,384 nodes, at least 16
    po_sequences: int = 5
    dmin: int = 1

    @property
    def elem_bytes(self) -> int:
        return 4 if self.feat_dtype == "f32" else 2

    @property
    def row_bytes(self) -> int:
        return self.feat_dim * self.elem_bytes


CONFIGS = {
    "tiny": Config("tiny", 10_000, 10.0, 1_000, 100, "f32", 512, (10, 5), 2_000, 20,
                   "random_all", 0, seed=20211208, dmin=2),
    "mid": Config("mid", 2_450_000, 50.2, 20_000, 100, "f32", 1024, (15, 10, 5), 490_000, 200,
                  "random_train", 204_800, seed=20211209, dmin=5),
    "bfs": Config("bfs", 2_450_000, 50.2, 20_000, 100, "f32", 1024, (15, 10, 5), 245_000, 200,
                  "po", 204_800, seed=20211209, dmin=5),
    "large": Config("large", 111_000_000, 14.4, 50_000, 128, "f32", 1024, (15, 10, 5), 25_000_000, 200,
                    "random_train", 1_200_000, row_ptr_bits=64, graph_placement="host_pinned",
                    seed=20211211, dmin=3),
    "wide": Config("wide", 30_000_000, 20.0, 20_000, 512, "bf16", 4096, (25, 10), 4_500_000, 100,
                   "random_train", 409_600, seed=20211212, dmin=4),
}


def scaled(cfg: Config, num_nodes: int, num_batches: Optional[int] = None) -> Config:
    """Same shape at a smaller node count: cache fraction, training fraction and
    degree distribution are kept; used where the full size does not fit."""
    f = num_nodes / cfg.num_nodes
    return dataclasses.replace(
        cfg, name=f"{cfg.name}@{num_nodes}", num_nodes=num_nodes,
        dmax=max(4 * cfg.dmin, int(cfg.mean_degree * 4), min(cfg.dmax, num_nodes // 4)),
        cache_rows=max(16, int(round(cfg.cache_rows * f))),
        train_size=(max(cfg.batch * (num_batches or cfg.num_batches),
                        int(round(cfg.train_size * f))) if cfg.train_size else 0),
        num_batches=num_batches or cfg.num_batches)


class PinnedBuffer:
    """Page-locked host memory of exactly the requested size (hipHostMalloc through
    ctypes; a framework allocator may round large requests up to a power of two,
    which the 50+ GB feature table cannot afford)."""

    _hip = None

    def __init__(self, nbytes: int):
        if PinnedBuffer._hip is None:
            PinnedBuffer._hip = C.CDLL("libamdhip64.so")
            PinnedBuffer._hip.hipHostMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t, C.c_uint]
            PinnedBuffer._hip.hipHostFree.argtypes = [C.c_void_p]
        p = C.c_void_p()
        rc = PinnedBuffer._hip.hipHostMalloc(C.byref(p), max(int(nbytes), 1), 0)
        if rc != 0 or not p.value:
            raise MemoryError(f"hipHostMalloc of {nbytes} bytes failed with status {rc}")
        self.ptr, self.nbytes = p.value, int(nbytes)

    def data_ptr(self) -> int:
        return self.ptr

    def array(self, shape, dtype) -> np.ndarray:
        buf = (C.c_uint8 * max(self.nbytes, 1)).from_address(self.ptr)
        return np.frombuffer(buf, dtype=dtype, count=int(np.prod(shape))).reshape(shape)

    def __del__(self):
        hip = getattr(type(self), "_hip", None) if type is not None else None
        if getattr(self, "ptr", None) and hip is not None:
            hip.hipHostFree(self.ptr)
            self.ptr = None


def _alloc(shape, dtype, pinned: bool):
    """numpy array, optionally backed by page-locked memory (needs a GPU runtime).
    Returns (array, owner); keep `owner` alive as long as the array is in use."""
    if pinned:
        import torch
        if torch.cuda.is_available():
            n = int(np.prod(shape)) * np.dtype(dtype).itemsize
            buf = PinnedBuffer(n)
            return buf.array(shape, dtype), buf
    return np.empty(shape, dtype=dtype), None


@dataclasses.dataclass
class Workload:
    cfg: Config
    row_ptr: np.ndarray          # int32 or int64 [N+1]
    col: np.ndarray              # int32 [E]
    features: np.ndarray         # float32 [N, dim] or uint16 (bf16 bits) [N, dim]
    seed_batches: np.ndarray     # int32 [num_batches, batch]
    rng_seeds: np.ndarray        # uint64 [num_batches], one per sampling call
    keepalive: list = dataclasses.field(default_factory=list)
    order_draws: Optional[dict] = None   # proximity-aware order: training set, roots, shifts it was computed from

    @property
    def num_edges(self) -> int:
        return int(self.row_ptr[-1])

    def feature_bytes(self) -> np.ndarray:
        return self.features.view(np.uint8).reshape(self.features.shape[0], -1)


def make_graph(cfg: Config, pinned: bool = False):
    g = _gen()
    N = cfg.num_nodes
    deg = np.empty(N, dtype=np.int32)
    E = g.bglgen_degrees(N, float(cfg.mean_degree), int(cfg.dmin), int(cfg.dmax), cfg.seed, deg.ctypes.data)
    if E < 0:
        raise ValueError("bad degree parameters")
    if cfg.row_ptr_bits == 32 and E >= 2**31:
        raise ValueError("edge count needs 64-bit row offsets")
    keep = []
    rp, t = _alloc(N + 1, np.int64 if cfg.row_ptr_bits == 64 else np.int32, pinned)
    keep.append(t)
    g.bglgen_row_ptr(N, deg.ctypes.data, rp.ctypes.data, cfg.row_ptr_bits)
    del deg
    col, t = _alloc(max(E, 1), np.int32, pinned)
    keep.append(t)
    perm = np.empty(N, dtype=np.int32)
    inv = np.empty(N, dtype=np.int32)
    g.bglgen_permutation(N, cfg.seed + 1, perm.ctypes.data, inv.ctypes.data)
    rc = g.bglgen_edges(N, rp.ctypes.data, cfg.row_ptr_bits, col.ctypes.data, cfg.seed + 2,
                        cfg.reach, cfg.p_local, cfg.beta, cfg.num_hubs or max(16, N // 16384),
                        perm.ctypes.data, inv.ctypes.data)
    if rc != 0:
        raise ValueError("edge generation failed")
    return rp, col[:E], keep


def make_features(cfg: Config, pinned: bool = False):
    dt = np.float32 if cfg.feat_dtype == "f32" else np.uint16
    feats, t = _alloc((cfg.num_nodes, cfg.feat_dim), dt, pinned)
    rc = _gen().bglgen_features(cfg.num_nodes, cfg.feat_dim, cfg.elem_bytes, cfg.seed + 3, feats.ctypes.data)
    if rc != 0:
        raise ValueError("feature generation failed")
    return feats, [t]


def make_seed_batches(cfg: Config, order_fn: Optional[Callable] = None):
    """Seed batches [num_batches, batch] and, for the proximity-aware order, the random draws that
    order was given.  The proximity-aware order of the paper's Sec. 3.2.2 is part of the method, not
    of the inputs: this module only draws the training set, the BFS roots and the shifts, and
    `order_fn(train_nodes, roots, shifts, num_out) -> order` (the library's bgl_order_proximity, or
    the oracle's) turns them into the order."""
    rng = np.random.default_rng(cfg.seed + 4)
    N, B, nb = cfg.num_nodes, cfg.batch, cfg.num_batches
    if cfg.order == "random_all":
        return np.stack([rng.choice(N, size=B, replace=False) for _ in range(nb)]).astype(np.int32), None
    train = rng.choice(N, size=cfg.train_size, replace=False).astype(np.int32)
    if B * nb > len(train):
        raise ValueError("training set smaller than one epoch of batches")
    if cfg.order == "random_train":
        return rng.permutation(train)[: B * nb].reshape(nb, B).astype(np.int32), None
    if cfg.order == "po":
        draws = dict(train=train, roots=rng.integers(0, N, cfg.po_sequences).astype(np.int64),
                     shifts=rng.integers(0, len(train), cfg.po_sequences).astype(np.int64), num_out=B * nb)
        if order_fn is None:
            raise ValueError("the proximity-aware order needs order_fn (the library's or the oracle's ordering call)")
        order = np.asarray(order_fn(draws["train"], draws["roots"], draws["shifts"], draws["num_out"]), dtype=np.int32)
        return order.reshape(nb, B), draws
    raise ValueError(cfg.order)


def make_workload(cfg: Config, pinned: bool = False, order_fn: Optional[Callable] = None) -> Workload:
    """Generate everything one configuration needs.  `pinned` places the feature
    table (and, for host-resident graphs, the CSR) in page-locked memory.
    order_fn(row_ptr, col, train_nodes, roots, shifts, num_out) -> order: needed for a configuration
    with proximity-aware seed order (see make_seed_batches); the draws it got are kept in
    `Workload.order_draws`."""
    rp, col, keep = make_graph(cfg, pinned and cfg.graph_placement == "host_pinned")
    feats, keep2 = make_features(cfg, pinned)
    fn = (lambda train, roots, shifts, num_out: order_fn(rp, col, train, roots, shifts, num_out)) if order_fn else None
    seeds, draws = make_seed_batches(cfg, fn)
    rng = np.random.default_rng(cfg.seed + 5)
    rng_seeds = rng.integers(0, 2**64, size=cfg.num_batches, dtype=np.uint64)
    return Workload(cfg, rp, col, feats, seeds, rng_seeds, keep + keep2, draws)
