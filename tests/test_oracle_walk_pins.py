"""Pins for oracle.walk_levels (Eq. 4 iterated without a visited set): dense
boolean matrix powers built literally from Eq. 1-3, brute-force enumeration of
all walks, closed forms, and the relation to the min-hop oracle."""
import itertools

import numpy as np
import pytest

import kggen
import oracle
from helpers import mask_allows


def levels_of(w, k=None, masked=True):
    k = w.k if k is None else k
    off, ent = oracle.walk_levels(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k,
                                  w.rel_mask if masked else None)
    Q = w.num_queries
    return [[ent[off[h * Q + q]:off[h * Q + q + 1]].tolist() for q in range(Q)] for h in range(k + 1)]


def one(E, triples, seeds, k, allowed=None, R=None):
    t = np.asarray(triples, dtype=np.int32).reshape(-1, 3)
    mask = None
    if allowed is not None:
        R = R or int(t[:, 1].max()) + 1
        mask = np.zeros((1, (R + 63) // 64), dtype=np.uint64)
        for r in allowed:
            mask[0, r // 64] |= np.uint64(1) << np.uint64(r % 64)
    off, ent = oracle.walk_levels(E, t[:, 0], t[:, 1], t[:, 2], np.array([0, len(seeds)], dtype=np.int64),
                                  np.asarray(seeds, dtype=np.int32), k, mask)
    return [ent[off[h]:off[h + 1]].tolist() for h in range(k + 1)]


# ---------------------------------------------------------------- dense SUB / REL / OBJ powers
@pytest.mark.parametrize("seed", range(10))
@pytest.mark.parametrize("masked", [False, True])
def test_against_boolean_matrix_powers(seed, masked):
    w = kggen.random_tiny(300 + seed, E=20 + seed, T=60 + 6 * seed, R=3, Q=5, k=5, masked=masked)
    E, T, R = w.num_entities, w.num_triples, w.num_relations
    SUB = np.zeros((E, T), dtype=np.int64)
    OBJ = np.zeros((T, E), dtype=np.int64)
    REL = np.zeros((T, R), dtype=np.int64)
    SUB[w.subj, np.arange(T)] = 1      # Eq. 1
    OBJ[np.arange(T), w.obj] = 1       # Eq. 2
    REL[np.arange(T), w.rel] = 1       # Eq. 3
    got = levels_of(w)
    for q in range(w.num_queries):
        m = np.ones(R, dtype=np.int64)
        if masked:
            m = np.array([int(mask_allows(w.rel_mask, q, r)) for r in range(R)], dtype=np.int64)
        qv = np.zeros(E, dtype=np.int64)
        qv[w.seeds[w.seed_off[q]:w.seed_off[q + 1]]] = 1
        for h in range(w.k + 1):
            assert got[h][q] == np.nonzero(qv)[0].tolist(), (q, h)
            active = (qv @ SUB > 0) & (REL @ m > 0)          # Eq. 5 with the whitelist
            qv = (active.astype(np.int64) @ OBJ > 0).astype(np.int64)   # Eq. 4


# ---------------------------------------------------------------- every walk, one by one
@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("masked", [False, True])
def test_against_walk_enumeration(seed, masked):
    w = kggen.random_tiny(400 + seed, E=10 + seed, T=22 + 2 * seed, R=3, Q=4, k=4, masked=masked)
    got = levels_of(w)
    triples = list(zip(w.subj.tolist(), w.rel.tolist(), w.obj.tolist()))
    for q in range(w.num_queries):
        ok = [t for t in triples if not masked or mask_allows(w.rel_mask, q, t[1])]
        seeds = set(w.seeds[w.seed_off[q]:w.seed_off[q + 1]].tolist())
        assert got[0][q] == sorted(seeds)
        for h in range(1, w.k + 1):
            ends = set()
            for walk in itertools.product(ok, repeat=h):      # all sequences of h allowed triples
                if walk[0][0] in seeds and all(walk[i][2] == walk[i + 1][0] for i in range(h - 1)):
                    ends.add(walk[-1][2])
            assert got[h][q] == sorted(ends), (q, h)


# ---------------------------------------------------------------- closed forms
def test_cycle_path_self_loop_and_bipartite():
    n = 7
    cyc = [[i, 0, (i + 1) % n] for i in range(n)]
    lv = one(n, cyc, [2], 16)
    assert all(lv[h] == [(2 + h) % n] for h in range(17))          # the walker goes round
    path = [[i, 0, i + 1] for i in range(5)]
    lv = one(6, path, [0], 8)
    assert [x for x in lv] == [[0], [1], [2], [3], [4], [5], [], [], []]   # falls off the end
    lv = one(3, [[0, 0, 0], [0, 0, 1]], [0], 3)
    assert lv == [[0], [0, 1], [0, 1], [0, 1]]                      # the self loop keeps the seed alive
    a, b = [0, 1, 2], [3, 4]
    bip = [[x, 0, y] for x in a for y in b] + [[y, 1, x] for y in b for x in a]
    lv = one(5, bip, [0], 4)
    assert lv == [[0], b, a, b, a]                                  # sides alternate
    lv = one(5, bip, [0], 4, allowed=[0], R=2)
    assert lv == [[0], b, [], [], []]                               # relation 1 is needed to come back
    lv = one(4, [[0, 0, 1], [0, 0, 2], [1, 0, 3], [2, 0, 3]], [0, 0, 0], 2)
    assert lv == [[0], [1, 2], [3]]                                 # repeated seeds collapse, joins merge
    assert one(3, [[0, 0, 1]], [], 2) == [[], [], []]               # no seed
    assert one(3, [[0, 0, 1]], [2], 0) == [[2]]                     # k = 0


# ---------------------------------------------------------------- relation to the min-hop result
@pytest.mark.parametrize("make", [lambda: kggen.config1(), lambda: kggen.config3(0.002, k=4),
                                  lambda: kggen.config2(0.003, num_queries=70)])
def test_union_is_the_reached_set_and_first_level_is_the_hop(make):
    w = make()
    ro, ent, hop, _, _ = oracle.khop(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k, w.rel_mask)
    lv = levels_of(w)
    for q in range(w.num_queries):
        first = {}
        for h in range(w.k + 1):
            for e in lv[h][q]:
                first.setdefault(e, h)
        a, b = ro[q], ro[q + 1]
        assert sorted(first) == ent[a:b].tolist()
        assert [first[e] for e in ent[a:b].tolist()] == hop[a:b].tolist()
        # one more step of a level is the next level: entities one allowed triple away
    # and a level is never larger than what its predecessor's out-edges can reach
    outdeg = np.bincount(w.subj, minlength=w.num_entities)
    for q in range(min(w.num_queries, 16)):
        for h in range(1, w.k + 1):
            assert len(lv[h][q]) <= int(outdeg[lv[h - 1][q]].sum()) if lv[h - 1][q] else not lv[h][q]
