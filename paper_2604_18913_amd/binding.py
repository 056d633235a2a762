"""ctypes binding of liblogoskg.so: argument marshalling only.

Every step of the retrieval runs inside the library's HIP kernels.  If the
library is missing this module raises; there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
import weakref
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblogoskg.so")
_lib = None

DIRECTIONS = {"auto": 0, "push": 1, "pull": 2}
NO_COUNTS = 4
WALK_EXACT = 8
STATUS = {0: "OK", 1: "EINVAL", 2: "ENOMEM", 3: "EDEVICE", 4: "ERANGE", 5: "EINTERNAL", 6: "EIO"}


class LogosKGError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"logoskg: {STATUS.get(status, status)}: {text}")
        self.status = status


class _BuildOpts(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("device", ctypes.c_int32),
                ("num_shards", ctypes.c_int32), ("max_resident_shards", ctypes.c_int32),
                ("hbm_shard_budget_bytes", ctypes.c_uint64), ("hub_min_degree", ctypes.c_int32),
                ("host_build", ctypes.c_int32), ("shard_dir", ctypes.c_char_p),
                ("dev_alloc", ctypes.c_void_p), ("dev_free", ctypes.c_void_p), ("alloc_ctx", ctypes.c_void_p)]


_ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
_FREE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)


class _QueryBatch(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("num_queries", ctypes.c_int32),
                ("num_seeds", ctypes.c_int64), ("seed_off", ctypes.c_void_p),
                ("seeds", ctypes.c_void_p), ("k", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("rel_mask", ctypes.c_void_p), ("stream", ctypes.c_void_p)]


class _GraphInfo(ctypes.Structure):
    _fields_ = [("num_triples", ctypes.c_int64), ("num_entities", ctypes.c_int32),
                ("num_relations", ctypes.c_int32), ("num_shards", ctypes.c_int32),
                ("hub_min_degree", ctypes.c_int32), ("num_out_rows", ctypes.c_int64),
                ("num_out_hubs", ctypes.c_int64), ("num_in_rows", ctypes.c_int64),
                ("num_in_hubs", ctypes.c_int64), ("device_bytes", ctypes.c_int64),
                ("pinned_host_bytes", ctypes.c_int64), ("shard_loads", ctypes.c_int64),
                ("shard_evictions", ctypes.c_int64), ("shard_hits", ctypes.c_int64),
                ("shard_bytes_h2d", ctypes.c_int64), ("shard_bytes_disk", ctypes.c_int64),
                ("num_object_ranges", ctypes.c_int32), ("cache_slots", ctypes.c_int32)]


class _ResultInfo(ctypes.Structure):
    _fields_ = [("num_queries", ctypes.c_int32), ("k", ctypes.c_int32),
                ("words_per_entity", ctypes.c_int32), ("num_levels", ctypes.c_int32),
                ("padded_entities", ctypes.c_int64), ("visited", ctypes.c_void_p),
                ("levels", ctypes.c_void_p), ("total_reached", ctypes.c_int64)]


class _HopStats(ctypes.Structure):
    _fields_ = [("direction", ctypes.c_int32), ("shards_touched", ctypes.c_int32),
                ("active_rows", ctypes.c_int64), ("frontier_edges", ctypes.c_int64),
                ("rows_scanned", ctypes.c_int64), ("edges_scanned", ctypes.c_int64),
                ("lines_gathered", ctypes.c_int64), ("entities_reached", ctypes.c_int64)]


class _KernelProfile(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 32), ("launches", ctypes.c_int64),
                ("total_ms", ctypes.c_double), ("max_ms", ctypes.c_double), ("rows", ctypes.c_int64),
                ("edges", ctypes.c_int64), ("lines", ctypes.c_int64), ("items", ctypes.c_int64)]


def library_path() -> str:
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python paper_2604_18913_amd/build_ext.py` "
                          "(there is no CPU fallback)")
    # PyTorch ships its own HIP runtime; import it first so that the library binds to the
    # same runtime instance that owns torch's device buffers and streams.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    P, I32, I64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.logoskg_build.restype = ctypes.c_int
    lib.logoskg_build.argtypes = [P, P, P, I64, I32, I32, ctypes.POINTER(_BuildOpts), ctypes.POINTER(P)]
    lib.logoskg_graph_free.restype = None
    lib.logoskg_graph_free.argtypes = [P]
    lib.logoskg_graph_get_info.restype = ctypes.c_int
    lib.logoskg_graph_get_info.argtypes = [P, ctypes.POINTER(_GraphInfo)]
    lib.logoskg_probe_gather.restype = ctypes.c_int
    lib.logoskg_probe_gather.argtypes = [P, P, P, P]
    lib.logoskg_graph_partition.restype = ctypes.c_int
    lib.logoskg_graph_partition.argtypes = [P, P, P]
    lib.logoskg_khop.restype = ctypes.c_int
    lib.logoskg_khop.argtypes = [P, ctypes.POINTER(_QueryBatch), ctypes.POINTER(P)]
    lib.logoskg_result_get_info.restype = ctypes.c_int
    lib.logoskg_result_get_info.argtypes = [P, ctypes.POINTER(_ResultInfo)]
    lib.logoskg_result_hop_stats.restype = ctypes.c_int
    lib.logoskg_result_hop_stats.argtypes = [P, P]
    lib.logoskg_result_offsets.restype = ctypes.c_int
    lib.logoskg_result_offsets.argtypes = [P, P]
    lib.logoskg_result_fetch.restype = ctypes.c_int
    lib.logoskg_result_fetch.argtypes = [P, I32, I32, I64, P, P, P, P]
    lib.logoskg_result_level_offsets.restype = ctypes.c_int
    lib.logoskg_result_level_offsets.argtypes = [P, I32, P, P]
    lib.logoskg_result_level_fetch.restype = ctypes.c_int
    lib.logoskg_result_level_fetch.argtypes = [P, I32, I32, I32, I64, P, P]
    lib.logoskg_result_triples_offsets.restype = ctypes.c_int
    lib.logoskg_result_triples_offsets.argtypes = [P, I32, I32, I32, P, P]
    lib.logoskg_result_triples_fetch.restype = ctypes.c_int
    lib.logoskg_result_triples_fetch.argtypes = [P, I32, I32, I32, I64, P, P, P, P, P]
    lib.logoskg_result_walks_count.restype = ctypes.c_int
    lib.logoskg_result_walks_count.argtypes = [P, I32, I32, P, P]
    lib.logoskg_result_walks_fetch.restype = ctypes.c_int
    lib.logoskg_result_walks_fetch.argtypes = [P, I32, I32, I64, I64, P, P, P]
    lib.logoskg_result_traversed.restype = ctypes.c_int
    lib.logoskg_result_traversed.argtypes = [P, P, P]
    lib.logoskg_result_free.restype = None
    lib.logoskg_result_free.argtypes = [P]
    lib.logoskg_paths.restype = ctypes.c_int
    lib.logoskg_paths.argtypes = [P, P, P, P, I64, I32, P, P, P]
    lib.logoskg_paths_static.restype = ctypes.c_int
    lib.logoskg_paths_static.argtypes = [P, P, P, P, I64, I32, P, P, P]
    lib.logoskg_prefetch_shards.restype = ctypes.c_int
    lib.logoskg_prefetch_shards.argtypes = [P, P, I32]
    lib.logoskg_schedule_queries.restype = ctypes.c_int
    lib.logoskg_schedule_queries.argtypes = [P, P, P, I64, P]
    lib.logoskg_walks.restype = ctypes.c_int
    lib.logoskg_walks.argtypes = [P, P, P, P, P, I64, I32, P, P, P]
    lib.logoskg_profile_enable.restype = ctypes.c_int
    lib.logoskg_profile_enable.argtypes = [P, I32]
    lib.logoskg_profile_read.restype = ctypes.c_int
    lib.logoskg_profile_read.argtypes = [P, P, I32, ctypes.POINTER(I32)]
    lib.logoskg_last_error.restype = ctypes.c_char_p
    lib.logoskg_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def version() -> str:
    return _load().logoskg_version().decode()


def _check(rc: int):
    if rc != 0:
        raise LogosKGError(rc, _load().logoskg_last_error().decode())


def _torch():
    import torch
    return torch


def _dev_tensor(x, dtype, device):
    torch = _torch()
    if isinstance(x, torch.Tensor):
        return x.to(device=device, dtype=dtype).contiguous()
    return torch.from_numpy(np.ascontiguousarray(x).astype(_NP[dtype], copy=False)).to(device)


_NP = {}


def _init_np():
    torch = _torch()
    _NP.update({torch.int32: np.int32, torch.int64: np.int64, torch.uint8: np.uint8})


def _stream_handle(stream) -> int:
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


class Result:
    """Device-resident state of one k-hop call (level planes, counts)."""

    def __init__(self, graph: "Graph", handle: int):
        self._g = graph
        self._h = ctypes.c_void_p(handle)
        info = _ResultInfo()
        _check(_load().logoskg_result_get_info(self._h, ctypes.byref(info)))
        self.num_queries = info.num_queries
        self.k = info.k
        self.words_per_entity = info.words_per_entity
        self.padded_entities = info.padded_entities
        self.total_reached = info.total_reached
        self._levels_ptr = info.levels
        self._visited_ptr = info.visited

    def offsets(self) -> np.ndarray:
        off = np.zeros(self.num_queries + 1, dtype=np.int64)
        _check(_load().logoskg_result_offsets(self._h, off.ctypes.data_as(ctypes.c_void_p)))
        return off

    def hop_stats(self):
        arr = (_HopStats * max(self.k, 1))()
        _check(_load().logoskg_result_hop_stats(self._h, ctypes.cast(arr, ctypes.c_void_p)))
        names = [f[0] for f in _HopStats._fields_]
        return [{n: int(getattr(arr[i], n)) for n in names} for i in range(self.k)]

    def fetch(self, q_begin: int = 0, q_end: Optional[int] = None, want_hop: bool = True,
              want_pred: bool = True, stream=None, out=None):
        """Query-major lists for queries [q_begin, q_end) as device tensors
        (entity int32, hop uint8 or None, pred int32 or None)."""
        torch = _torch()
        q_end = self.num_queries if q_end is None else q_end
        off = self.offsets()
        n = int(off[q_end] - off[q_begin])
        dev = self._g.device
        if out is None:
            entity = torch.empty(n, dtype=torch.int32, device=dev)
            hop = torch.empty(n, dtype=torch.uint8, device=dev) if want_hop else None
            pred = torch.empty(n, dtype=torch.int32, device=dev) if want_pred else None
        else:
            entity, hop, pred = out
        _check(_load().logoskg_result_fetch(
            self._h, q_begin, q_end, entity.numel(), entity.data_ptr(),
            hop.data_ptr() if hop is not None else None,
            pred.data_ptr() if pred is not None else None, _stream_handle(stream)))
        return entity[:n], (hop[:n] if hop is not None else None), (pred[:n] if pred is not None else None)

    def level(self, h: int, q_begin: int = 0, q_end: Optional[int] = None, stream=None):
        """``logoskg_result_level_offsets`` + ``logoskg_result_level_fetch``: the entities of level
        ``h`` of the queries [q_begin, q_end) as (offsets int64[Q+1] of the whole level, entity
        int32 device tensor)."""
        torch = _torch()
        q_end = self.num_queries if q_end is None else q_end
        off = np.zeros(self.num_queries + 1, dtype=np.int64)
        _check(_load().logoskg_result_level_offsets(self._h, h, off.ctypes.data_as(ctypes.c_void_p),
                                                    _stream_handle(stream)))
        n = int(off[q_end] - off[q_begin])
        entity = torch.empty(n, dtype=torch.int32, device=self._g.device)
        _check(_load().logoskg_result_level_fetch(self._h, h, q_begin, q_end, n, entity.data_ptr(),
                                                  _stream_handle(stream)))
        return off, entity

    def active_triples(self, h: int, q_begin: int = 0, q_end: Optional[int] = None, components: bool = True,
                       out=None, stream=None):
        """``logoskg_result_triples_offsets`` + ``logoskg_result_triples_fetch``: T_h of the queries
        [q_begin, q_end) as (offsets int64[q_end - q_begin + 1], triple, subject, relation, object)
        int32 device tensors (the last three None without ``components``).  ``out`` = four int32
        device tensors (or None entries) to write into instead of new ones."""
        torch = _torch()
        q_end = self.num_queries if q_end is None else q_end
        off = np.zeros(max(q_end - q_begin, 0) + 1, dtype=np.int64)
        _check(_load().logoskg_result_triples_offsets(self._h, h, q_begin, q_end,
                                                      off.ctypes.data_as(ctypes.c_void_p), _stream_handle(stream)))
        n = int(off[-1])
        if out is not None:
            bufs = list(out)
            cap = min(int(b.numel()) for b in bufs if b is not None)
        else:
            bufs = [torch.empty(n, dtype=torch.int32, device=self._g.device) for _ in range(4 if components else 1)]
            bufs += [None] * (4 - len(bufs))
            cap = n
        ptrs = [None if b is None else b.data_ptr() for b in bufs]
        _check(_load().logoskg_result_triples_fetch(self._h, h, q_begin, q_end, cap, *ptrs, _stream_handle(stream)))
        return (off, *[None if b is None else b[:n] for b in bufs])

    def walks_count(self, query: int, length: int, stream=None) -> int:
        """``logoskg_result_walks_count``: number of chains of ``length`` allowed triples of ``query``."""
        total = ctypes.c_int64()
        _check(_load().logoskg_result_walks_count(self._h, query, length, ctypes.byref(total), _stream_handle(stream)))
        return int(total.value)

    def walks_fetch(self, query: int, length: int, first: int, count: int, out=None, stream=None):
        """``logoskg_result_walks_fetch``: chains [first, first + count) of the (query, length) counted
        last as (edges int32[count, length], target int32[count]) device tensors."""
        torch = _torch()
        if out is None:
            edges = torch.empty((count, length), dtype=torch.int32, device=self._g.device)
            target = torch.empty(count, dtype=torch.int32, device=self._g.device)
        else:
            edges, target = out
        _check(_load().logoskg_result_walks_fetch(self._h, query, length, first, count, edges.data_ptr(),
                                                  target.data_ptr(), _stream_handle(stream)))
        return edges[:count], target[:count]

    def traversed(self, stream=None):
        torch = _torch()
        t = torch.empty((self.num_queries, self.k), dtype=torch.int64, device=self._g.device)
        _check(_load().logoskg_result_traversed(self._h, t.data_ptr(), _stream_handle(stream)))
        return t

    def close(self):
        if self._h:
            if self._g._h:  # a result never outlives its graph: Graph.close releases its results first
                _load().logoskg_result_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Graph:
    """A knowledge graph built on one GPU (``logoskg_build``).

    ``num_shards`` > 1 keeps the subject-sorted triples outside HBM, shard by shard (pinned host
    memory, or files under ``shard_dir``), behind a cache of ``max_resident_shards`` /
    ``hbm_shard_budget_bytes``; ``host_build`` sorts the triples on the host.  ``dev_alloc(nbytes) ->
    device address (0 = out of memory)`` and ``dev_free(address)`` become the allocator of the memory
    the calls on this graph take and give back (``logoskg_build_opts.dev_alloc / dev_free``)."""

    def __init__(self, subj, rel, obj, num_entities: int, num_relations: int, device: int = 0,
                 num_shards: int = 0, max_resident_shards: int = 0, hbm_shard_budget_bytes: int = 0,
                 hub_min_degree: int = 0, host_build: bool = False, shard_dir: Optional[str] = None,
                 dev_alloc=None, dev_free=None):
        lib = _load()
        torch = _torch()
        if not _NP:
            _init_np()
        if not torch.cuda.is_available():
            raise RuntimeError("logoskg needs a GPU (no CPU fallback)")
        subj = np.ascontiguousarray(subj, dtype=np.int32)
        rel = np.ascontiguousarray(rel, dtype=np.int32)
        obj = np.ascontiguousarray(obj, dtype=np.int32)
        if not (subj.shape == rel.shape == obj.shape and subj.ndim == 1):
            raise ValueError("subj, rel, obj must be 1-D arrays of equal length")
        # the C callbacks stay referenced by the graph for as long as the library may call them
        self._alloc_cb = None if dev_alloc is None else _ALLOC_FN(lambda nbytes, ctx: dev_alloc(nbytes) or None)
        self._free_cb = None if dev_free is None else _FREE_FN(lambda ptr, ctx: dev_free(ptr))
        opts = _BuildOpts(ctypes.sizeof(_BuildOpts), device, num_shards, max_resident_shards,
                          hbm_shard_budget_bytes, hub_min_degree, 1 if host_build else 0,
                          None if shard_dir is None else os.fsencode(shard_dir),
                          None if self._alloc_cb is None else ctypes.cast(self._alloc_cb, ctypes.c_void_p),
                          None if self._free_cb is None else ctypes.cast(self._free_cb, ctypes.c_void_p), None)
        h = ctypes.c_void_p()
        _check(lib.logoskg_build(subj.ctypes.data_as(ctypes.c_void_p), rel.ctypes.data_as(ctypes.c_void_p),
                                 obj.ctypes.data_as(ctypes.c_void_p), subj.shape[0], num_entities,
                                 num_relations, ctypes.byref(opts), ctypes.byref(h)))
        self._h = h
        self._results = weakref.WeakSet()
        self.device = torch.device("cuda", device)
        self.num_entities = num_entities
        self.num_relations = num_relations
        self.num_triples = int(subj.shape[0])

    def info(self) -> dict:
        gi = _GraphInfo()
        _check(_load().logoskg_graph_get_info(self._h, ctypes.byref(gi)))
        return {f[0]: int(getattr(gi, f[0])) for f in _GraphInfo._fields_}

    def profile_enable(self, level: int):
        """0 = off, 1 = time every kernel launch with HIP events, 2 = also count work units."""
        _check(_load().logoskg_profile_enable(self._h, level))

    def profile_read(self) -> dict:
        """Drain the per-kernel accumulators: name -> dict(launches, total_ms, ...)."""
        n = ctypes.c_int32()
        arr = (_KernelProfile * 64)()
        _check(_load().logoskg_profile_read(self._h, ctypes.cast(arr, ctypes.c_void_p), 64, ctypes.byref(n)))
        out = {}
        for rec in arr[:n.value]:
            out[rec.name.decode()] = dict(launches=int(rec.launches), total_ms=float(rec.total_ms),
                                          max_ms=float(rec.max_ms), rows=int(rec.rows), edges=int(rec.edges),
                                          lines=int(rec.lines), items=int(rec.items))
        return out

    def probe_gather(self, lines, stream=None):
        """Measurement aid: the line gathers of a dense pull hop alone, on `lines` ([num_entities, 16]
        int64 device tensor); returns the OR of the gathered lines (16 words, device)."""
        torch = _torch()
        assert lines.is_cuda and lines.dtype == torch.int64 and lines.is_contiguous()
        assert tuple(lines.shape) == (self.num_entities, 16)
        out = torch.empty(16, dtype=torch.int64, device=lines.device)
        _check(_load().logoskg_probe_gather(self._h, lines.data_ptr(), out.data_ptr(), _stream_handle(stream)))
        return out

    def partition(self):
        n = max(self.info()["num_shards"], 1)
        shard_of = np.zeros(self.num_entities, dtype=np.int32)
        per = np.zeros(n, dtype=np.int64)
        _check(_load().logoskg_graph_partition(self._h, shard_of.ctypes.data_as(ctypes.c_void_p),
                                               per.ctypes.data_as(ctypes.c_void_p)))
        return shard_of, per

    def khop(self, seed_off, seeds, k: int, rel_mask=None, direction: str = "auto", counts: bool = True,
             stream=None, walk_exact: bool = False) -> Result:
        """``logoskg_khop`` for up to 1024 queries; inputs may be numpy arrays
        or device tensors (they are placed in HBM before the call)."""
        torch = _torch()
        seed_off_d = _dev_tensor(seed_off, torch.int64, self.device)
        seeds_d = _dev_tensor(seeds, torch.int32, self.device)
        mask_d = None
        if rel_mask is not None:
            if isinstance(rel_mask, torch.Tensor):
                mask_d = rel_mask.to(self.device).contiguous()
            else:
                mask_d = torch.from_numpy(np.ascontiguousarray(rel_mask, dtype=np.uint64).view(np.int64)).to(self.device)
            if mask_d.numel() != (seed_off_d.numel() - 1) * ((self.num_relations + 63) // 64):
                raise ValueError("rel_mask must be [Q, ceil(R/64)] 64-bit words")
        batch = _QueryBatch(ctypes.sizeof(_QueryBatch), seed_off_d.numel() - 1, seeds_d.numel(),
                            seed_off_d.data_ptr(), seeds_d.data_ptr() if seeds_d.numel() else None, k,
                            DIRECTIONS[direction] | (0 if counts else NO_COUNTS) | (WALK_EXACT if walk_exact else 0),
                            mask_d.data_ptr() if mask_d is not None else None, _stream_handle(stream))
        h = ctypes.c_void_p()
        _check(_load().logoskg_khop(self._h, ctypes.byref(batch), ctypes.byref(h)))
        res = Result(self, h.value)
        self._results.add(res)
        return res

    def paths(self, result: Result, query_idx, target, max_paths: int = 16, stream=None):
        """``logoskg_paths``: (count int32[n], edges int32[n, max_paths, k]) device tensors."""
        torch = _torch()
        q = _dev_tensor(query_idx, torch.int32, self.device)
        t = _dev_tensor(target, torch.int32, self.device)
        n = q.numel()
        count = torch.empty(n, dtype=torch.int32, device=self.device)
        edges = torch.empty((n, max_paths, result.k), dtype=torch.int32, device=self.device)
        _check(_load().logoskg_paths(self._h, result._h, q.data_ptr(), t.data_ptr(), n, max_paths,
                                     count.data_ptr(), edges.data_ptr() if edges.numel() else None,
                                     _stream_handle(stream)))
        return count, edges

    def paths_static(self, result: Result, query_idx, target, count, edges, max_paths: int = 16, stream=None):
        """``logoskg_paths_static``: the listing of ``paths`` written into the caller's device tensors
        ``count`` int32[n] and ``edges`` int32[n, max_paths, k]; ``query_idx`` and ``target`` must
        already be int32 device tensors.  Nothing is allocated on the device."""
        n = query_idx.numel()
        _check(_load().logoskg_paths_static(self._h, result._h, query_idx.data_ptr(), target.data_ptr(), n,
                                            max_paths, count.data_ptr(), edges.data_ptr() if edges.numel() else None,
                                            _stream_handle(stream)))

    def prefetch_shards(self, shards) -> None:
        """``logoskg_prefetch_shards``: ask the shard cache for these shards now (host list)."""
        ids = np.ascontiguousarray(shards, dtype=np.int32)
        _check(_load().logoskg_prefetch_shards(self._h, ids.ctypes.data_as(ctypes.c_void_p), ids.shape[0]))

    def schedule_queries(self, seed_off, seeds) -> np.ndarray:
        """``logoskg_schedule_queries``: the order (int32[Q] of query indices) that groups the
        queries by the sub-graphs their seeds need; host arrays in, host array out."""
        so = np.ascontiguousarray(seed_off, dtype=np.int64)
        sd = np.ascontiguousarray(seeds, dtype=np.int32)
        order = np.zeros(so.shape[0] - 1, dtype=np.int32)
        _check(_load().logoskg_schedule_queries(self._h, so.ctypes.data_as(ctypes.c_void_p),
                                                sd.ctypes.data_as(ctypes.c_void_p), so.shape[0] - 1,
                                                order.ctypes.data_as(ctypes.c_void_p)))
        return order

    def walks(self, result: Result, query_idx, target, length, max_paths: int = 16, stream=None):
        """``logoskg_walks``: (count int32[n], edges int32[n, max_paths, k]) device tensors."""
        torch = _torch()
        q = _dev_tensor(query_idx, torch.int32, self.device)
        t = _dev_tensor(target, torch.int32, self.device)
        d = _dev_tensor(length, torch.int32, self.device)
        n = q.numel()
        count = torch.empty(n, dtype=torch.int32, device=self.device)
        edges = torch.empty((n, max_paths, result.k), dtype=torch.int32, device=self.device)
        _check(_load().logoskg_walks(self._h, result._h, q.data_ptr(), t.data_ptr(), d.data_ptr(), n, max_paths,
                                     count.data_ptr(), edges.data_ptr() if edges.numel() else None,
                                     _stream_handle(stream)))
        return count, edges

    def close(self):
        if self._h:
            for res in list(self._results):  # results borrow the graph's memory pool
                res.close()
            _load().logoskg_graph_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# Same names as the C entry points, for callers that prefer the flat form.
def logoskg_build(subj, rel, obj, num_entities, num_relations, **opts) -> Graph:
    return Graph(subj, rel, obj, num_entities, num_relations, **opts)


def logoskg_khop(graph: Graph, seed_off, seeds, k, rel_mask=None, **kw) -> Result:
    return graph.khop(seed_off, seeds, k, rel_mask, **kw)


def logoskg_paths(graph: Graph, result: Result, query_idx, target, max_paths=16):
    return graph.paths(result, query_idx, target, max_paths)
