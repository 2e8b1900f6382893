"""Thin ctypes binding over libbgl.so (the C ABI declared in include/bgl.h).

Argument marshalling only: every step of sampling and of the cache workflow runs
in the library's HIP kernels.  PyTorch supplies device memory, page-locked host
memory and streams.  There is no fallback: importing this module without a built
library, or calling it without a GPU, raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbgl.so")

BGL_OK, BGL_EINVAL, BGL_ENOMEM, BGL_EHIP, BGL_ECAPACITY, BGL_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
BGL_MAX_HOPS = 8
BGL_MAX_FANOUT = 64
BGL_COUNTS_LEN = 2 * BGL_MAX_HOPS + 2
BGL_NOALLOC_MAX_IDS = 1310720
BGL_DEVICE, BGL_HOST_PINNED, BGL_HOST_PINNED_COL = 0, 1, 2
(STAGE_PROBE, STAGE_MISS_LIST, STAGE_GATHER_HIT, STAGE_FETCH_MISS,
 STAGE_INSERT_MAP, STAGE_INSERT_ROWS, STAGE_LINK_COPY, STAGE_ASSEMBLE_PRE, STAGE_ASSEMBLE) = range(9)
STAGE_NAMES = ["probe", "miss_list", "gather_hit", "fetch_miss", "insert_map", "insert_rows", "link_copy",
               "assemble_pre", "assemble"]

EXPORTS = [
    "bgl_last_error", "bgl_graph_load_csr", "bgl_graph_destroy", "bgl_sample_workspace_bytes",
    "bgl_sample_khop", "bgl_cache_create", "bgl_cache_destroy", "bgl_cache_lookup_gather",
    "bgl_cache_lookup_gather_early", "bgl_cache_lookup_gather_noalloc",
    "bgl_cache_insert_fifo", "bgl_cache_set_write_through", "bgl_cache_wait_rows", "bgl_cache_wait_lists", "bgl_cache_export_state", "bgl_cache_stats",
    "bgl_cache_map_stats", "bgl_cache_set_spare_rows",
    "bgl_cache_set_profiling", "bgl_cache_profile", "bgl_cache_set_profiling_every",
    "bgl_host_tier_create", "bgl_host_tier_destroy", "bgl_host_tier_set_copy_engine", "bgl_cache_lookup_gather_tiered",
    "bgl_cache_lookup_tiered_begin", "bgl_cache_lookup_tiered_finish",
    "bgl_host_tier_export_state", "bgl_host_tier_stats",
    "bgl_order_bfs_sequence", "bgl_order_proximity", "bgl_order_choose_sequences",
    "bgl_order_shuffling_error",
    "bgl_pipeline_create", "bgl_pipeline_destroy", "bgl_pipeline_set_cache", "bgl_pipeline_set_tier", "bgl_pipeline_streams", "bgl_pipeline_last_batch", "bgl_pipeline_run",
]


class BglError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"bgl status {code}: {msg}")
        self.code = code


class SubgraphStruct(C.Structure):
    _fields_ = [
        ("num_hops", C.c_int32),
        ("input_nodes", C.c_void_p),
        ("row_ptr", C.c_void_p * BGL_MAX_HOPS),
        ("col_local", C.c_void_p * BGL_MAX_HOPS),
        ("cap_nodes", C.c_int64 * (BGL_MAX_HOPS + 1)),
        ("cap_edges", C.c_int64 * BGL_MAX_HOPS),
        ("counts", C.c_void_p),
    ]


class PipelineBuffers(C.Structure):
    _fields_ = [
        ("workspace", C.c_void_p * 3),
        ("workspace_bytes", C.c_size_t),
        ("counts_host", C.c_void_p * 3),
        ("out_rows", C.c_void_p),
        ("out_slot", C.c_void_p),
        ("miss_pos", C.c_void_p),
        ("cap_rows", C.c_int64),
    ]


BATCH_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_int64, C.c_int32, C.POINTER(SubgraphStruct), C.c_int64)


def load_library(path: str = LIB_PATH) -> C.CDLL:
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2112_08541_amd.buildlib`")
    L = C.CDLL(path)
    i64, i32, u64, vp, ci = C.c_int64, C.c_int32, C.c_uint64, C.c_void_p, C.c_int
    L.bgl_last_error.restype = C.c_char_p
    L.bgl_last_error.argtypes = []
    L.bgl_graph_load_csr.argtypes = [vp, ci, vp, i64, i64, ci, C.POINTER(vp)]
    L.bgl_graph_destroy.argtypes = [vp]
    L.bgl_sample_workspace_bytes.argtypes = [i32, vp, i32, i64, C.POINTER(C.c_size_t)]
    L.bgl_sample_khop.argtypes = [vp, vp, i32, vp, i32, u64, vp, C.c_size_t,
                                  C.POINTER(SubgraphStruct), vp, vp]
    L.bgl_cache_create.argtypes = [i64, i32, vp, i64, C.POINTER(vp)]
    L.bgl_cache_destroy.argtypes = [vp]
    L.bgl_cache_lookup_gather.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp, vp]
    L.bgl_cache_lookup_gather_noalloc.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp, vp]
    L.bgl_cache_lookup_gather_early.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp, vp, vp]
    L.bgl_cache_insert_fifo.argtypes = [vp, vp, vp, i64, vp, vp]
    L.bgl_cache_set_write_through.argtypes = [vp, ci]
    L.bgl_cache_set_spare_rows.argtypes = [vp, i64]
    L.bgl_cache_wait_rows.argtypes = [vp, vp]
    L.bgl_cache_wait_lists.argtypes = [vp, vp]
    L.bgl_host_tier_create.argtypes = [vp, i64, i32, i64, i64, i32, C.POINTER(vp)]
    L.bgl_host_tier_destroy.argtypes = [vp]
    L.bgl_host_tier_set_copy_engine.argtypes = [vp, ci]
    L.bgl_cache_lookup_gather_tiered.argtypes = [vp, vp, vp, i64, vp, vp, vp, C.POINTER(i64), vp, vp, vp, ci]
    L.bgl_cache_lookup_tiered_begin.argtypes = L.bgl_cache_lookup_gather_tiered.argtypes
    L.bgl_cache_lookup_tiered_finish.argtypes = [vp]
    L.bgl_host_tier_export_state.argtypes = [vp, vp, C.POINTER(C.c_uint64), vp]
    L.bgl_host_tier_stats.argtypes = [vp, C.POINTER(u64), C.POINTER(u64), C.POINTER(C.c_double), C.POINTER(u64), C.POINTER(i32)]
    L.bgl_cache_export_state.argtypes = [vp, vp, C.POINTER(u64), vp]
    L.bgl_cache_stats.argtypes = [vp, C.POINTER(u64), C.POINTER(u64), C.POINTER(u64),
                                  C.POINTER(u64), C.POINTER(i32)]
    L.bgl_cache_map_stats.argtypes = [vp] + [C.POINTER(u64)] * 5
    L.bgl_cache_set_profiling.argtypes = [vp, ci]
    L.bgl_cache_profile.argtypes = [vp, ci, C.POINTER(C.c_double), C.POINTER(i64)]
    L.bgl_cache_set_profiling_every.argtypes = [vp, ci, ci]
    L.bgl_order_bfs_sequence.argtypes = [vp, vp, i64, i64, vp, vp]
    L.bgl_order_proximity.argtypes = [vp, vp, i64, i32, vp, vp, i64, vp, vp]
    L.bgl_order_choose_sequences.argtypes = [vp, vp, i64, i32, vp, vp, i32, vp, i32, C.c_double,
                                             C.POINTER(i32), vp, vp, vp]
    L.bgl_order_shuffling_error.argtypes = [vp, i64, i32, vp, i64, i32, C.POINTER(C.c_double),
                                            C.POINTER(C.c_double)]
    L.bgl_pipeline_create.argtypes = [vp, vp, vp, i32, vp, i32, C.POINTER(PipelineBuffers), ci, vp, C.POINTER(vp)]
    L.bgl_pipeline_destroy.argtypes = [vp]
    L.bgl_pipeline_set_cache.argtypes = [vp, vp, ci]
    L.bgl_pipeline_set_tier.argtypes = [vp, vp]
    L.bgl_pipeline_streams.argtypes = [vp, C.POINTER(vp), C.POINTER(vp)]
    L.bgl_pipeline_last_batch.argtypes = [vp, C.POINTER(vp), C.POINTER(i64)]
    L.bgl_pipeline_run.argtypes = [vp, vp, i64, vp, i64, i64, vp, vp, vp, BATCH_FN, vp]
    for name in EXPORTS:
        if name != "bgl_last_error":
            getattr(L, name).restype = ci
    return L


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = load_library()
    return _lib


def _check(rc: int) -> None:
    if rc != BGL_OK:
        raise BglError(rc, lib().bgl_last_error().decode())


def _require_gpu() -> None:
    if not torch.cuda.is_available():
        raise RuntimeError("paper_2112_08541_amd needs a GPU: there is no CPU path")


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dev_ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _host_ptr(x) -> int:
    if isinstance(x, torch.Tensor):
        if x.is_cuda or not x.is_contiguous():
            raise ValueError("expected a contiguous host tensor")
        return x.data_ptr()
    if not x.flags.c_contiguous:
        raise ValueError("expected a C-contiguous array")
    return x.ctypes.data


class Graph:
    """bgl_graph_load_csr / bgl_graph_destroy."""

    def __init__(self, row_ptr, col_idx, placement: int = BGL_DEVICE):
        _require_gpu()
        rp_dtype = row_ptr.dtype
        bits = 64 if rp_dtype in (np.int64, torch.int64) else 32
        if bits == 32 and rp_dtype not in (np.int32, torch.int32):
            raise ValueError("row_ptr must be int32 or int64")
        self.num_nodes = int(row_ptr.shape[0]) - 1
        self.num_edges = int(col_idx.shape[0])
        self.placement = placement
        self._keep = (row_ptr, col_idx) if placement != BGL_DEVICE else None
        h = C.c_void_p()
        _check(lib().bgl_graph_load_csr(_host_ptr(row_ptr), bits, _host_ptr(col_idx), self.num_nodes,
                                        self.num_edges, placement, C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None) and lib is not None:
            lib().bgl_graph_destroy(self._h)
            self._h = None

    __del__ = close


class SampledBatch:
    """Device-side result of one bgl_sample_khop call (views into the sampler's workspace)."""

    def __init__(self, sampler: "Sampler", st: SubgraphStruct):
        self._s = sampler
        self.struct = st
        self.num_hops = st.num_hops

    def counts(self) -> np.ndarray:
        """Host copy of the counts block; the stream must have been synchronised."""
        return self._s.counts_host.numpy().copy()

    def sizes(self):
        c = self.counts()
        K = self.num_hops
        status = int(c[BGL_COUNTS_LEN - 1])
        if status != 0:
            raise BglError(status, "sampling reported an error on the device (seed id out of range?)")
        return c[: K + 1].astype(np.int64), c[BGL_MAX_HOPS + 1: BGL_MAX_HOPS + 1 + K].astype(np.int64)

    def _view(self, ptr: int, n: int) -> torch.Tensor:
        off = ptr - self._s.workspace.data_ptr()
        return self._s.workspace[off: off + 4 * n].view(torch.int32)

    def input_nodes(self, n: Optional[int] = None) -> torch.Tensor:
        """int32 device view of frontier_K (first n entries; default: the upper bound)."""
        K = self.num_hops
        return self._view(self.struct.input_nodes, int(self.struct.cap_nodes[K]) if n is None else n)

    def row_ptr(self, h: int, n_dst: int) -> torch.Tensor:
        return self._view(self.struct.row_ptr[h], n_dst + 1)

    def col_local(self, h: int, nnz: int) -> torch.Tensor:
        return self._view(self.struct.col_local[h], nnz)


class Sampler:
    """Owns the device workspace for bgl_sample_khop at a fixed (num_seeds, fanouts)."""

    def __init__(self, graph: Graph, num_seeds: int, fanouts: Sequence[int]):
        _require_gpu()
        self.graph = graph
        self.num_seeds = int(num_seeds)
        self.fanouts = np.ascontiguousarray(fanouts, dtype=np.int32)
        nbytes = C.c_size_t(0)
        _check(lib().bgl_sample_workspace_bytes(self.num_seeds, self.fanouts.ctypes.data,
                                                len(self.fanouts), graph.num_nodes, C.byref(nbytes)))
        self.workspace_bytes = int(nbytes.value)
        self.workspace = torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device="cuda")
        pad = (-self.workspace.data_ptr()) % 256
        self.workspace = self.workspace[pad: pad + self.workspace_bytes]
        self.counts_host = torch.zeros(BGL_COUNTS_LEN, dtype=torch.int32).pin_memory()

    def sample(self, seeds: torch.Tensor, rng_seed: int, stream=None) -> SampledBatch:
        if seeds.numel() != self.num_seeds:
            raise ValueError("seed count differs from the one the workspace was sized for")
        st = SubgraphStruct()
        _check(lib().bgl_sample_khop(self.graph._h, _dev_ptr(seeds, torch.int32), self.num_seeds,
                                     self.fanouts.ctypes.data, len(self.fanouts),
                                     int(rng_seed) & (2**64 - 1), self.workspace.data_ptr(),
                                     self.workspace_bytes, C.byref(st), self.counts_host.data_ptr(),
                                     _stream_handle(stream)))
        return SampledBatch(self, st)


class Cache:
    """bgl_cache_* calls on one cache handle."""

    def __init__(self, capacity_rows: int, features, num_nodes: Optional[int] = None,
                 row_bytes: Optional[int] = None):
        _require_gpu()
        if features is None:           # misses are served through a HostTier only
            if num_nodes is None or row_bytes is None:
                raise ValueError("num_nodes and row_bytes are required without a backing store")
            nn, rb, ptr = num_nodes, row_bytes, None
        elif isinstance(features, int):  # raw address of page-locked or device memory
            if num_nodes is None or row_bytes is None:
                raise ValueError("num_nodes and row_bytes are required with a raw address")
            nn, rb, ptr = num_nodes, row_bytes, features
        elif isinstance(features, torch.Tensor):
            nn = features.shape[0]
            rb = features.stride(0) * features.element_size()
            ptr = features.data_ptr()
        else:
            nn = features.shape[0]
            rb = features.strides[0]
            ptr = features.ctypes.data
        self.num_nodes = int(num_nodes if num_nodes is not None else nn)
        self.row_bytes = int(row_bytes if row_bytes is not None else rb)
        self.capacity = int(capacity_rows)
        self._features = features
        h = C.c_void_p()
        _check(lib().bgl_cache_create(self.capacity, self.row_bytes, ptr, self.num_nodes, C.byref(h)))
        self._h = h
        self.n_hit_host = torch.zeros(1, dtype=torch.int64).pin_memory()

    def close(self):
        if getattr(self, "_h", None) and lib is not None:
            lib().bgl_cache_destroy(self._h)
            self._h = None

    __del__ = close

    def lookup_gather(self, ids: torch.Tensor, n: int, out_rows: torch.Tensor, out_slot: torch.Tensor,
                      miss_pos: torch.Tensor, main_stream=None, side_stream=None,
                      n_hit_ptr: Optional[int] = None, lookup_stream=None, noalloc: bool = False) -> None:
        """n_hit_ptr: address of a page-locked int64 for the hit count (default: self.n_hit_host).
        lookup_stream: run the map lookup and the lists there (bgl_cache_lookup_gather_early).
        noalloc: bgl_cache_lookup_gather_noalloc (the call that allocates nothing)."""
        if n > 0 and (ids.numel() < n or out_slot.numel() < n or miss_pos.numel() < n or
                      out_rows.numel() * out_rows.element_size() < n * self.row_bytes):
            raise ValueError("an argument is smaller than n")
        args = (self._h, _dev_ptr(ids, torch.int32), n, _dev_ptr(out_rows), _dev_ptr(out_slot, torch.int32),
                _dev_ptr(miss_pos, torch.int32),
                self.n_hit_host.data_ptr() if n_hit_ptr is None else n_hit_ptr, _stream_handle(main_stream),
                None if side_stream is None else int(side_stream.cuda_stream))
        if noalloc:
            if lookup_stream is not None:
                raise ValueError("the call that allocates nothing has no early form")
            _check(lib().bgl_cache_lookup_gather_noalloc(*args))
        elif lookup_stream is None:
            _check(lib().bgl_cache_lookup_gather(*args))
        else:
            _check(lib().bgl_cache_lookup_gather_early(*args, _stream_handle(lookup_stream)))

    def lookup_gather_tiered(self, tier: "HostTier", ids: torch.Tensor, n: int, out_rows: torch.Tensor,
                             out_slot: torch.Tensor, miss_pos: torch.Tensor, main_stream=None,
                             side_stream=None, lookup_stream=None, begin_only: bool = False):
        """Returns (hits in this cache, hits in the tier).  lookup_stream: run the map lookup and
        the lists there (early lookup; write-through mode only).  begin_only: the first half alone
        (bgl_cache_lookup_tiered_begin); lookup_tiered_finish() is the second."""
        if n > 0 and (ids.numel() < n or out_slot.numel() < n or miss_pos.numel() < n or
                      out_rows.numel() * out_rows.element_size() < n * self.row_bytes):
            raise ValueError("an argument is smaller than n")
        n_hit = (C.c_int64 * 2)(0, 0)
        call = lib().bgl_cache_lookup_tiered_begin if begin_only else lib().bgl_cache_lookup_gather_tiered
        _check(call(
            self._h, tier._h, _dev_ptr(ids, torch.int32), n, _dev_ptr(out_rows),
            _dev_ptr(out_slot, torch.int32), _dev_ptr(miss_pos, torch.int32), n_hit,
            _stream_handle(main_stream), None if side_stream is None else int(side_stream.cuda_stream),
            None if lookup_stream is None else _stream_handle(lookup_stream), 0 if lookup_stream is None else 1))
        return int(n_hit[0]), int(n_hit[1])

    def lookup_tiered_finish(self) -> None:
        _check(lib().bgl_cache_lookup_tiered_finish(self._h))

    def insert_fifo(self, ids: torch.Tensor, miss_pos: torch.Tensor, n_miss: int,
                    out_rows: torch.Tensor, stream=None) -> None:
        _check(lib().bgl_cache_insert_fifo(self._h, _dev_ptr(ids, torch.int32),
                                           _dev_ptr(miss_pos, torch.int32), n_miss, _dev_ptr(out_rows),
                                           _stream_handle(stream)))

    def set_spare_rows(self, spare_rows: int) -> None:
        """bgl_cache_set_spare_rows: extra row positions in the buffer (before the first insertion)."""
        _check(lib().bgl_cache_set_spare_rows(self._h, int(spare_rows)))

    def set_write_through(self, enable: bool) -> None:
        _check(lib().bgl_cache_set_write_through(self._h, 1 if enable else 0))

    def wait_lists(self, stream=None) -> None:
        _check(lib().bgl_cache_wait_lists(self._h, _stream_handle(stream)))

    def wait_rows(self, stream=None) -> None:
        _check(lib().bgl_cache_wait_rows(self._h, _stream_handle(stream)))

    def export_state(self, with_buffer: bool = True):
        s2n = np.empty(self.capacity, dtype=np.int32)
        tail = C.c_uint64(0)
        buf = np.empty((self.capacity, self.row_bytes), dtype=np.uint8) if with_buffer else None
        _check(lib().bgl_cache_export_state(self._h, s2n.ctypes.data, C.byref(tail),
                                            buf.ctypes.data if with_buffer else None))
        return s2n, int(tail.value), buf

    def stats(self):
        vals = [C.c_uint64(0) for _ in range(4)]
        status = C.c_int32(0)
        _check(lib().bgl_cache_stats(self._h, *[C.byref(v) for v in vals], C.byref(status)))
        return dict(lookups=vals[0].value, hits=vals[1].value, inserts=vals[2].value,
                    evictions=vals[3].value, status=status.value)

    def map_stats(self):
        """bgl_cache_map_stats: what the map's lookups have cost so far and how many buckets
        a lookup would walk past right now."""
        vals = [C.c_uint64(0) for _ in range(5)]
        _check(lib().bgl_cache_map_stats(self._h, *[C.byref(v) for v in vals]))
        ids, lines, nb, passed, passes = (v.value for v in vals)
        return dict(ids_looked_up=ids, bucket_lines_read=lines, num_buckets=nb, buckets_passed=passed,
                    passes=passes, lines_per_id=(lines / ids if ids else 0.0))

    def set_profiling(self, stages=True) -> None:
        """stages: False/True (none/all) or an iterable of stage names to bracket with events."""
        if stages is True:
            mask = (1 << len(STAGE_NAMES)) - 1
        elif not stages:
            mask = 0
        else:
            mask = sum(1 << STAGE_NAMES.index(s) for s in stages)
        _check(lib().bgl_cache_set_profiling(self._h, mask))

    def set_profiling_every(self, stage: str, every: int) -> None:
        """Time `stage` only in every `every`-th call (counted from the cache's creation, from 1)."""
        _check(lib().bgl_cache_set_profiling_every(self._h, STAGE_NAMES.index(stage), int(every)))

    def profile(self):
        out = {}
        for s, name in enumerate(STAGE_NAMES):
            ms, n = C.c_double(0), C.c_int64(0)
            _check(lib().bgl_cache_profile(self._h, s, C.byref(ms), C.byref(n)))
            out[name] = (ms.value, n.value)
        ms, n = C.c_double(0), C.c_int64(0)
        _check(lib().bgl_cache_profile(self._h, 100, C.byref(ms), C.byref(n)))
        out["event_overhead"] = (ms.value, 1)
        return out


class HostTier:
    """bgl_host_tier_* calls: FIFO cache level in page-locked host memory in front of `store`
    (a C-contiguous numpy array of num_nodes rows, ordinary host memory)."""

    def __init__(self, store: np.ndarray, capacity_rows: int, max_batch_rows: int, num_threads: int = 0):
        _require_gpu()
        if not store.flags["C_CONTIGUOUS"]:
            raise ValueError("store must be C-contiguous")
        self._store = store
        self.num_nodes = int(store.shape[0])
        self.row_bytes = int(store.strides[0])
        self.capacity = int(capacity_rows)
        h = C.c_void_p()
        _check(lib().bgl_host_tier_create(store.ctypes.data, self.num_nodes, self.row_bytes, self.capacity,
                                          int(max_batch_rows), int(num_threads), C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None) and lib is not None:
            lib().bgl_host_tier_destroy(self._h)
            self._h = None

    __del__ = close

    def set_copy_engine(self, mode) -> None:
        """Packed rows cross the link as plain copies into device memory (then scattered by kernels)
        instead of being read over the link by the kernels themselves.  mode: False/0, True/1, or
        2 = as 1, with the cache writing its whole output in one pass where it can."""
        _check(lib().bgl_host_tier_set_copy_engine(self._h, int(mode)))

    def export_state(self, with_buffer: bool = True):
        s2n = np.empty(self.capacity, dtype=np.int32)
        tail = C.c_uint64(0)
        buf = np.empty((self.capacity, self.row_bytes), dtype=np.uint8) if with_buffer else None
        _check(lib().bgl_host_tier_export_state(self._h, s2n.ctypes.data, C.byref(tail),
                                                buf.ctypes.data if with_buffer else None))
        return s2n, int(tail.value), buf

    def stats(self):
        lk, ht, nb, th, ms = C.c_uint64(0), C.c_uint64(0), C.c_uint64(0), C.c_int32(0), C.c_double(0)
        _check(lib().bgl_host_tier_stats(self._h, C.byref(lk), C.byref(ht), C.byref(ms), C.byref(nb), C.byref(th)))
        return dict(lookups=lk.value, hits=ht.value, copy_ms=ms.value, batches=nb.value, threads=th.value)


def order_bfs_sequence(graph: Graph, train_nodes, root: int, stream=None) -> np.ndarray:
    """bgl_order_bfs_sequence: the training nodes in canonical BFS order from `root`."""
    train = np.ascontiguousarray(train_nodes, dtype=np.int32)
    seq = np.empty(len(train), dtype=np.int32)
    _check(lib().bgl_order_bfs_sequence(graph._h, train.ctypes.data, len(train), int(root),
                                        seq.ctypes.data, _stream_handle(stream)))
    return seq


def order_proximity(graph: Graph, train_nodes, roots, shifts, num_out: int, stream=None) -> np.ndarray:
    """bgl_order_proximity: the first num_out nodes of the proximity-aware order."""
    train = np.ascontiguousarray(train_nodes, dtype=np.int32)
    roots = np.ascontiguousarray(roots, dtype=np.int64)
    shifts = np.ascontiguousarray(shifts, dtype=np.int64)
    if len(roots) != len(shifts):
        raise ValueError("one shift per root")
    order = np.empty(max(num_out, 1), dtype=np.int32)
    _check(lib().bgl_order_proximity(graph._h, train.ctypes.data, len(train), len(roots),
                                     roots.ctypes.data, shifts.ctypes.data, int(num_out),
                                     order.ctypes.data, _stream_handle(stream)))
    return order[:num_out]


def order_shuffling_error(order, batch: int, labels, num_classes: int):
    """bgl_order_shuffling_error: (mean, max) total variation distance over the batches."""
    order = np.ascontiguousarray(order, dtype=np.int32)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    a, b = C.c_double(0), C.c_double(0)
    _check(lib().bgl_order_shuffling_error(order.ctypes.data, len(order), int(batch), labels.ctypes.data,
                                           len(labels), int(num_classes), C.byref(a), C.byref(b)))
    return a.value, b.value


def order_choose_sequences(graph: Graph, train_nodes, roots, shifts, batch: int, labels,
                           num_classes: int, threshold: float, stream=None):
    """bgl_order_choose_sequences: (chosen count, errors per tried count, merged order)."""
    train = np.ascontiguousarray(train_nodes, dtype=np.int32)
    roots = np.ascontiguousarray(roots, dtype=np.int64)
    shifts = np.ascontiguousarray(shifts, dtype=np.int64)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    if len(labels) != graph.num_nodes:
        raise ValueError("one label per node")
    chosen = C.c_int32(0)
    errs = np.full(len(roots), np.nan)
    order = np.empty(len(train), dtype=np.int32)
    _check(lib().bgl_order_choose_sequences(graph._h, train.ctypes.data, len(train), len(roots),
                                            roots.ctypes.data, shifts.ctypes.data, int(batch),
                                            labels.ctypes.data, int(num_classes), float(threshold),
                                            C.byref(chosen), errs.ctypes.data, order.ctypes.data,
                                            _stream_handle(stream)))
    return chosen.value, errs[: chosen.value].copy(), order
