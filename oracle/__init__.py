"""CPU oracle for batched k-hop KG retrieval -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP library
and never calls it.  The arithmetic lives in ``khop_oracle.c`` (plain C,
compiled with gcc); this file only builds that library and marshals numpy
arrays into it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "khop_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_khop.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP for one-query-per-thread)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        P = ctypes.c_void_p
        lib.oracle_khop.restype = ctypes.c_int
        lib.oracle_khop.argtypes = [ctypes.c_int64, ctypes.c_int32, P, P, P, ctypes.c_int32,
                                    P, P, ctypes.c_int32, P, ctypes.c_int32, ctypes.c_int32,
                                    ctypes.c_int32, P, ctypes.POINTER(P), ctypes.POINTER(P),
                                    ctypes.POINTER(P), P]
        lib.oracle_paths.restype = ctypes.c_int
        lib.oracle_paths.argtypes = [ctypes.c_int64, ctypes.c_int32, P, P, P, ctypes.c_int32,
                                     P, P, ctypes.c_int32, P, ctypes.c_int32, ctypes.c_int64,
                                     P, P, ctypes.c_int32, P, P]
        lib.oracle_walk_levels.restype = ctypes.c_int
        lib.oracle_walk_levels.argtypes = [ctypes.c_int64, ctypes.c_int32, P, P, P, ctypes.c_int32,
                                           P, P, ctypes.c_int32, P, ctypes.c_int32, ctypes.c_int32,
                                           P, ctypes.POINTER(P)]
        lib.oracle_walk_paths.restype = ctypes.c_int
        lib.oracle_walk_paths.argtypes = [ctypes.c_int64, ctypes.c_int32, P, P, P, ctypes.c_int32,
                                          P, P, ctypes.c_int32, P, ctypes.c_int32, ctypes.c_int64,
                                          P, P, P, ctypes.c_int32, P, P]
        lib.oracle_active_triples.restype = ctypes.c_int64
        lib.oracle_active_triples.argtypes = [ctypes.c_int64, ctypes.c_int32, P, P, ctypes.c_int64, P, P,
                                              ctypes.POINTER(P)]
        lib.oracle_free.argtypes = [P]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def khop(num_entities: int, subj, rel, obj, seed_off, seeds, k: int,
         rel_mask: Optional[np.ndarray] = None, mode: int = 0, nthreads: int = 0):
    """Per-query BFS over the raw triple list.

    Returns ``(reached_off int64[Q+1], entity int32[N], hop uint8[N],
    pred int32[N], traversed int64[Q, k])``; lists are query-major and ascend in
    entity id inside a query.  ``mode=1`` uses no index (full rescan per hop).
    """
    lib = _load()
    subj, p_s = _c(subj, np.int32)
    rel, p_r = _c(rel, np.int32)
    obj, p_o = _c(obj, np.int32)
    seed_off, p_so = _c(seed_off, np.int64)
    seeds, p_sd = _c(seeds, np.int32)
    Q = seed_off.shape[0] - 1
    if rel_mask is not None:
        rel_mask, p_m = _c(rel_mask, np.uint64)
        rw = rel_mask.shape[1]
    else:
        p_m, rw = None, 0
    reached_off = np.zeros(Q + 1, dtype=np.int64)
    trav = np.zeros((Q, max(k, 0)), dtype=np.int64)
    ent, hop, pred = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
    rc = lib.oracle_khop(subj.shape[0], num_entities, p_s, p_r, p_o, Q, p_so, p_sd, k,
                         p_m, rw, mode, nthreads,
                         reached_off.ctypes.data_as(ctypes.c_void_p),
                         ctypes.byref(ent), ctypes.byref(hop), ctypes.byref(pred),
                         trav.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise RuntimeError("oracle_khop failed (bad arguments or out of memory)")
    n = int(reached_off[-1])

    def take(ptr, ctype, dtype):
        if n == 0:
            out = np.zeros(0, dtype=dtype)
        else:
            out = np.ctypeslib.as_array(ctypes.cast(ptr, ctypes.POINTER(ctype)), shape=(n,)).copy()
        lib.oracle_free(ptr)
        return out

    return (reached_off, take(ent, ctypes.c_int32, np.int32), take(hop, ctypes.c_uint8, np.uint8),
            take(pred, ctypes.c_int32, np.int32), trav)


def paths(num_entities: int, subj, rel, obj, seed_off, seeds, k: int, pair_query,
          pair_target, max_paths: int = 16, rel_mask: Optional[np.ndarray] = None):
    """First ``max_paths`` shortest paths per (query, target) pair.

    Returns ``(count int32[n], edges int32[n, max_paths, k])`` with -1 padding;
    every path is written seed -> target.
    """
    lib = _load()
    subj, p_s = _c(subj, np.int32)
    rel, p_r = _c(rel, np.int32)
    obj, p_o = _c(obj, np.int32)
    seed_off, p_so = _c(seed_off, np.int64)
    seeds, p_sd = _c(seeds, np.int32)
    pq, p_pq = _c(pair_query, np.int32)
    pt, p_pt = _c(pair_target, np.int32)
    Q = seed_off.shape[0] - 1
    if rel_mask is not None:
        rel_mask, p_m = _c(rel_mask, np.uint64)
        rw = rel_mask.shape[1]
    else:
        p_m, rw = None, 0
    n = pq.shape[0]
    count = np.zeros(n, dtype=np.int32)
    edges = np.full((n, max_paths, max(k, 0)), -1, dtype=np.int32)
    rc = lib.oracle_paths(subj.shape[0], num_entities, p_s, p_r, p_o, Q, p_so, p_sd, k,
                          p_m, rw, n, p_pq, p_pt, max_paths,
                          count.ctypes.data_as(ctypes.c_void_p),
                          edges.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise RuntimeError("oracle_paths failed")
    return count, edges


def walk_levels(num_entities: int, subj, rel, obj, seed_off, seeds, k: int,
                rel_mask: Optional[np.ndarray] = None, nthreads: int = 0):
    """Walk-exact levels: Eq. 4 iterated without a visited set.

    Returns ``(level_off int64[(k+1)*Q + 1], entity int32[N])``: the entities that
    end a walk of exactly ``h`` allowed triples from a seed of query ``q`` are
    ``entity[level_off[h*Q+q] : level_off[h*Q+q+1]]``, ascending.
    """
    lib = _load()
    subj, p_s = _c(subj, np.int32)
    rel, p_r = _c(rel, np.int32)
    obj, p_o = _c(obj, np.int32)
    seed_off, p_so = _c(seed_off, np.int64)
    seeds, p_sd = _c(seeds, np.int32)
    Q = seed_off.shape[0] - 1
    if rel_mask is not None:
        rel_mask, p_m = _c(rel_mask, np.uint64)
        rw = rel_mask.shape[1]
    else:
        p_m, rw = None, 0
    level_off = np.zeros((k + 1) * Q + 1, dtype=np.int64)
    ent = ctypes.c_void_p()
    rc = lib.oracle_walk_levels(subj.shape[0], num_entities, p_s, p_r, p_o, Q, p_so, p_sd, k,
                                p_m, rw, nthreads, level_off.ctypes.data_as(ctypes.c_void_p),
                                ctypes.byref(ent))
    if rc != 0:
        raise RuntimeError("oracle_walk_levels failed (bad arguments or out of memory)")
    n = int(level_off[-1])
    if n == 0:
        out = np.zeros(0, dtype=np.int32)
    else:
        out = np.ctypeslib.as_array(ctypes.cast(ent, ctypes.POINTER(ctypes.c_int32)), shape=(n,)).copy()
    lib.oracle_free(ent)
    return level_off, out


def active_triples(num_entities: int, subj, rel, frontier, rel_mask_row: Optional[np.ndarray] = None):
    """T_h of one query (Eq. 5-6): indices of the triples whose subject is in
    ``frontier`` (the support of q^(h-1)) and whose relation the query's
    whitelist ``rel_mask_row`` (uint64 words, or None = all) allows, ordered by
    (subject, triple index).  Returns int32[n]."""
    lib = _load()
    subj, p_s = _c(subj, np.int32)
    rel, p_r = _c(rel, np.int32)
    frontier, p_f = _c(frontier, np.int32)
    if rel_mask_row is not None:
        rel_mask_row, p_m = _c(rel_mask_row, np.uint64)
    else:
        p_m = None
    out = ctypes.c_void_p()
    n = lib.oracle_active_triples(subj.shape[0], num_entities, p_s, p_r, frontier.shape[0], p_f, p_m,
                                  ctypes.byref(out))
    if n < 0:
        raise RuntimeError("oracle_active_triples failed (bad arguments or out of memory)")
    if n == 0:
        res = np.zeros(0, dtype=np.int32)
    else:
        res = np.ctypeslib.as_array(ctypes.cast(out, ctypes.POINTER(ctypes.c_int32)), shape=(n,)).copy()
    lib.oracle_free(out)
    return res


def walk_paths(num_entities: int, subj, rel, obj, seed_off, seeds, k: int, pair_query, pair_target,
               pair_len, max_paths: int = 16, rel_mask: Optional[np.ndarray] = None):
    """First ``max_paths`` walks of exactly ``pair_len[i]`` allowed triples from a seed of
    ``pair_query[i]`` to ``pair_target[i]``, ordered by (t_d, .., t_1).

    Returns ``(count int32[n], edges int32[n, max_paths, k])`` with -1 padding;
    every walk is written seed -> target.
    """
    lib = _load()
    subj, p_s = _c(subj, np.int32)
    rel, p_r = _c(rel, np.int32)
    obj, p_o = _c(obj, np.int32)
    seed_off, p_so = _c(seed_off, np.int64)
    seeds, p_sd = _c(seeds, np.int32)
    pq, p_pq = _c(pair_query, np.int32)
    pt, p_pt = _c(pair_target, np.int32)
    pl, p_pl = _c(pair_len, np.int32)
    Q = seed_off.shape[0] - 1
    if rel_mask is not None:
        rel_mask, p_m = _c(rel_mask, np.uint64)
        rw = rel_mask.shape[1]
    else:
        p_m, rw = None, 0
    n = pq.shape[0]
    count = np.zeros(n, dtype=np.int32)
    edges = np.full((n, max_paths, max(k, 0)), -1, dtype=np.int32)
    rc = lib.oracle_walk_paths(subj.shape[0], num_entities, p_s, p_r, p_o, Q, p_so, p_sd, k,
                               p_m, rw, n, p_pq, p_pt, p_pl, max_paths,
                               count.ctypes.data_as(ctypes.c_void_p),
                               edges.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise RuntimeError("oracle_walk_paths failed")
    return count, edges
