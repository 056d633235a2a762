"""Oracle side of the scalable-retrieval pieces (paper Sec. 3.4) -- TEST
INFRASTRUCTURE ONLY, plain Python.

* degree_aware_partition: the partition reading used by this build -- subjects
  sorted by (out-degree descending, id ascending), each given to the shard with
  the fewest triples so far, ties to the lowest shard index.  The paper fixes
  only the properties (disjoint, a subject's triples stay together, high-degree
  subjects spread evenly, balanced), which `check_partition_properties` tests.
* lru_counts: the on-demand cache of capacity n sub-graphs under
  least-recently-used replacement, counting loads, evictions and hits.
* shard_accesses: the sub-graphs Algorithm 1 touches, hop by hop (those that
  hold a subject of the current frontier); the algorithm leaves the order inside
  a hop open, the reading taken is ascending shard index on odd hops and
  descending on even hops.  A hop that the caller says was evaluated by object
  rows (pull) touches every sub-graph of the partition by object range instead,
  numbered after the shards, in the same alternating order.  Pinned by
  hand-worked traces in tests/test_oracle_pins.py.
* fetch_accesses: what a fetch of predecessor edges touches when the cache can hold every unit
  (shards, object ranges, triple indices of the ranges): every object range in ascending order,
  first the range itself, then its triple indices (units numbered behind the ranges).
* schedule_queries: the batch-processing order of Sec. 3.4 -- queries grouped by
  the sub-graphs their seeds need (through P), identical needs adjacent, the
  input order kept among equals.
"""
from __future__ import annotations

import heapq
from collections import OrderedDict

import numpy as np


def degree_aware_partition(num_entities: int, subj: np.ndarray, m: int):
    deg = np.bincount(subj, minlength=num_entities)
    subjects = [int(e) for e in np.nonzero(deg)[0]]
    subjects.sort(key=lambda e: (-int(deg[e]), e))
    heap = [(0, s) for s in range(m)]
    heapq.heapify(heap)
    P = np.full(num_entities, -1, dtype=np.int32)
    loads = np.zeros(m, dtype=np.int64)
    for e in subjects:
        load, s = heapq.heappop(heap)
        P[e] = s
        load += int(deg[e])
        loads[s] = load
        heapq.heappush(heap, (load, s))
    return P, loads


def check_partition_properties(num_entities, subj, P, loads, m):
    deg = np.bincount(subj, minlength=num_entities)
    assert np.all((P >= 0) == (deg > 0)), "exactly the subjects are assigned"
    assert P.max(initial=-1) < m
    # all triples of a subject are in one shard and the shard sizes add up
    assert np.array_equal(np.bincount(P[subj], minlength=m), loads)
    assert loads.sum() == subj.shape[0]
    # balance: greedy longest-first keeps every shard within one largest row of the mean
    assert loads.max() - loads.min() <= max(int(deg.max()), 1)


def lru_counts(accesses, capacity: int):
    cache = OrderedDict()
    loads = evictions = hits = 0
    for a in accesses:
        if a in cache:
            hits += 1
            cache.move_to_end(a)
        else:
            if len(cache) >= capacity:
                cache.popitem(last=False)
                evictions += 1
            cache[a] = True
            loads += 1
    return loads, evictions, hits


def shard_accesses(P, subj, num_entities, k, entity, hop, pull_hops=(), num_shards=0, num_ranges=0):
    """entity / hop: concatenated result lists of all queries of one batch.
    pull_hops: the hops (1-based) evaluated by object rows; they touch the sub-graphs
    num_shards .. num_shards + num_ranges - 1 (the partition by object range)."""
    deg = np.bincount(subj, minlength=num_entities)
    seq = []
    for h in range(1, k + 1):
        front = np.unique(entity[hop == h - 1])
        front = front[deg[front] > 0]
        if front.size == 0:
            break
        if h in pull_hops:
            order = list(range(num_shards, num_shards + num_ranges))
        else:
            order = sorted(set(int(x) for x in P[front]))
        # Alg. 1 does not fix the order in which a hop visits its shards; the reading taken is
        # ascending on odd hops and descending on even ones, so that consecutive hops share the
        # shards at the turning point and a small LRU cache does not thrash
        if h % 2 == 0:
            order.reverse()
        seq.extend(order)
    return seq


def fetch_accesses(num_shards, num_ranges, capacity):
    """Units a list fetch with predecessor edges makes resident (none when the cache cannot hold
    all num_shards + 2 * num_ranges units: the object-sorted triples are then streamed past it)."""
    if capacity < num_shards + 2 * num_ranges:
        return []
    seq = []
    for c in range(num_ranges):
        seq += [num_shards + c, num_shards + num_ranges + c]
    return seq


def query_needs(P, seed_off, seeds):
    """needs[q] = ascending tuple of the distinct sub-graphs that hold a seed of query q."""
    needs = []
    for q in range(len(seed_off) - 1):
        shards = {int(P[e]) for e in seeds[seed_off[q]:seed_off[q + 1]] if P[e] >= 0}
        needs.append(tuple(sorted(shards)))
    return needs


def schedule_queries(P, seed_off, seeds):
    """Order in which to process the queries: sorted by their needs (tuples compared
    lexicographically, the empty need first), input order kept among equal needs."""
    needs = query_needs(P, seed_off, seeds)
    return np.array(sorted(range(len(needs)), key=lambda q: needs[q]), dtype=np.int32)

