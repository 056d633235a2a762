"""Pins for oracle.walk_paths (complete paths of Sec. 3.3 without a visited set: walks of exactly
d allowed triples from a seed to a target): forward enumeration of every walk, walk counts from
integer powers of the adjacency matrix, closed forms, the shortest-path oracle and the
hand-worked example."""
import json
import os

import numpy as np
import pytest

import kggen
import oracle
from helpers import mask_allows, pack_mask

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_example.json")


def all_walks(subj, rel, obj, seeds, d, allowed):
    """Every sequence of d allowed triples that starts at a seed, by plain forward extension."""
    out_edges = {}
    for t in range(len(subj)):
        if allowed is None or int(rel[t]) in allowed:
            out_edges.setdefault(int(subj[t]), []).append(t)
    walks = [((), s) for s in sorted(set(int(x) for x in seeds))]
    for _ in range(d):
        walks = [(w + (t,), int(obj[t])) for w, v in walks for t in out_edges.get(v, [])]
    return walks


def listing(walks, target, max_paths):
    mine = sorted((w for w, v in walks if v == target), key=lambda w: tuple(reversed(w)))
    return mine[:max_paths], len(mine)


def got_rows(count, edges, i, d):
    return [tuple(int(x) for x in edges[i, p, :d]) for p in range(count[i])]


def test_hand_worked_example():
    g = json.load(open(GOLDEN))
    t = np.asarray(g["triples_s_r_o"], dtype=np.int32)
    case = g["cases"][0]
    items = case["walk_paths"]
    cnt, edges = oracle.walk_paths(g["num_entities"], t[:, 0], t[:, 1], t[:, 2], [0, len(case["seeds"])],
                                   case["seeds"], case["k"], [0] * len(items), [x["target"] for x in items],
                                   [x["length"] for x in items], 16)
    for i, x in enumerate(items):
        assert got_rows(cnt, edges, i, x["length"]) == [tuple(r) for r in x["edges"]], x
        assert (edges[i, cnt[i]:] == -1).all() and (edges[i, :, x["length"]:] == -1).all()


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("masked", [False, True])
def test_against_forward_enumeration(seed, masked):
    w = kggen.random_tiny(1200 + seed, E=9 + seed % 3, T=22 + 2 * seed, R=3, Q=3, k=4, masked=masked)
    E = w.num_entities
    for q in range(w.num_queries):
        allowed = None
        if masked:
            allowed = {r for r in range(w.num_relations) if mask_allows(w.rel_mask, q, r)}
        seeds = w.seeds[w.seed_off[q]:w.seed_off[q + 1]]
        for d in range(w.k + 1):
            walks = all_walks(w.subj, w.rel, w.obj, seeds, d, allowed)
            for max_paths in (3, 64):
                cnt, edges = oracle.walk_paths(E, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k, [q] * E,
                                               np.arange(E), [d] * E, max_paths, w.rel_mask if masked else None)
                for v in range(E):
                    want, total = listing(walks, v, max_paths)
                    assert cnt[v] == min(total, max_paths), (q, d, v)
                    assert got_rows(cnt, edges, v, d) == want, (q, d, v)


@pytest.mark.parametrize("seed", range(4))
def test_counts_against_adjacency_powers(seed):
    w = kggen.random_tiny(1250 + seed, E=14, T=40, R=2, Q=4, k=4, masked=bool(seed & 1))
    E = w.num_entities
    for q in range(w.num_queries):
        A = np.zeros((E, E), dtype=np.int64)          # A[i][j] = allowed triples i -> j
        for t in range(w.num_triples):
            if mask_allows(w.rel_mask, q, int(w.rel[t])):
                A[w.subj[t], w.obj[t]] += 1
        x = np.zeros(E, dtype=np.int64)
        x[np.unique(w.seeds[w.seed_off[q]:w.seed_off[q + 1]])] = 1
        for d in range(w.k + 1):
            cnt, _ = oracle.walk_paths(E, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k, [q] * E, np.arange(E),
                                       [d] * E, 4096, w.rel_mask)
            assert np.array_equal(cnt, np.minimum(x, 4096)), (q, d)
            x = x @ A


def test_closed_forms():
    # a directed cycle of 5, seed 0: exactly one walk of every length, ending at d mod 5
    n = 5
    s = np.arange(n, dtype=np.int32)
    o = (s + 1) % n
    r = np.zeros(n, dtype=np.int32)
    for d in range(8):
        cnt, e = oracle.walk_paths(n, s, r, o, [0, 1], [0], 7, [0] * n, np.arange(n), [d] * n, 4)
        assert cnt.tolist() == [int(v == d % n) for v in range(n)]
        assert e[d % n, 0, :d].tolist() == [i % n for i in range(d)]
    # a path with doubled triples: 0 => 1 => 2 => 3, triples 2i and 2i+1 go from i to i+1
    s = np.array([0, 0, 1, 1, 2, 2], dtype=np.int32)
    o = s + 1
    r = np.array([0, 1, 0, 1, 0, 1], dtype=np.int32)
    cnt, e = oracle.walk_paths(4, s, r, o, [0, 1], [0], 3, [0, 0, 0], [3, 3, 2], [3, 2, 2], 16)
    assert cnt.tolist() == [8, 0, 4]
    assert [tuple(x) for x in e[0, :8]] == [(0, 2, 4), (1, 2, 4), (0, 3, 4), (1, 3, 4),
                                            (0, 2, 5), (1, 2, 5), (0, 3, 5), (1, 3, 5)]
    # truncation keeps a prefix of that order; a whitelist leaves one walk
    cnt3, e3 = oracle.walk_paths(4, s, r, o, [0, 1], [0], 3, [0], [3], [3], 3)
    assert cnt3.tolist() == [3] and np.array_equal(e3[0], e[0, :3])
    cnt1, e1 = oracle.walk_paths(4, s, r, o, [0, 1], [0], 3, [0], [3], [3], 16, pack_mask([[1]], 2))
    assert cnt1.tolist() == [1] and e1[0, 0].tolist() == [1, 3, 5]
    # length 0: the empty walk at a seed, nothing elsewhere; bad pairs give 0
    cnt0, _ = oracle.walk_paths(4, s, r, o, [0, 1], [0], 3, [0, 0, 0, 5, 0], [0, 1, 9, 0, 0], [0, 0, 0, 0, 4], 2)
    assert cnt0.tolist() == [1, 0, 0, 0, 0]
    # a self loop lets a walk wait: seed 0 with 0 -> 0 and 0 -> 1
    s = np.array([0, 0], dtype=np.int32)
    o = np.array([0, 1], dtype=np.int32)
    cnt, e = oracle.walk_paths(2, s, np.zeros(2, dtype=np.int32), o, [0, 1], [0], 3, [0], [1], [3], 4)
    assert cnt.tolist() == [1] and e[0, 0].tolist() == [0, 0, 1]


@pytest.mark.parametrize("seed", range(3))
def test_walks_of_minimum_length_are_the_shortest_paths(seed):
    w = kggen.random_tiny(1300 + seed, E=40, T=150, R=3, Q=5, k=4, masked=bool(seed & 1))
    ro, ent, hop, _, _ = oracle.khop(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k, w.rel_mask)
    pq = np.repeat(np.arange(w.num_queries), np.diff(ro)).astype(np.int32)
    c1, e1 = oracle.paths(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k, pq, ent, 8, w.rel_mask)
    c2, e2 = oracle.walk_paths(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k, pq, ent, hop, 8,
                               w.rel_mask)
    assert np.array_equal(c1, c2) and np.array_equal(e1, e2)
