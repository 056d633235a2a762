"""Pins for oracle.active_triples (the active-triple set T_h of Eq. 5-6): the
dense product q . SUB built literally from Eq. 1-3, the relation t^(h) . OBJ =
q^(h) to the level oracles, the traversed-triple counts of the min-hop oracle,
closed forms and the hand-worked example."""
import json
import os

import numpy as np
import pytest

import kggen
import oracle
from helpers import mask_allows, pack_mask

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_example.json")


def walk_levels_of(w, masked=True):
    off, ent = oracle.walk_levels(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k,
                                  w.rel_mask if masked else None)
    Q = w.num_queries
    return [[ent[off[h * Q + q]:off[h * Q + q + 1]] for q in range(Q)] for h in range(w.k + 1)]


def minhop_levels_of(w, masked=True):
    off, ent, hop, _, trav = oracle.khop(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k,
                                         w.rel_mask if masked else None)
    lv = [[ent[off[q]:off[q + 1]][hop[off[q]:off[q + 1]] == h] for q in range(w.num_queries)]
          for h in range(w.k + 1)]
    return lv, trav


def row_of(w, q, masked):
    return w.rel_mask[q] if (masked and w.rel_mask is not None) else None


# ---------------------------------------------------------------- hand-worked example
def test_hand_worked_example():
    d = json.load(open(GOLDEN))
    t = np.asarray(d["triples_s_r_o"], dtype=np.int32)
    E, R = d["num_entities"], d["num_relations"]
    checked = 0
    for case in d["cases"]:
        if "active_triples" not in case:
            continue
        mask = None if case["allowed_relations"] is None else pack_mask([case["allowed_relations"]], R)
        off, ent, hop, _, _ = oracle.khop(E, t[:, 0], t[:, 1], t[:, 2], np.array([0, len(case["seeds"])]),
                                          case["seeds"], case["k"], mask)
        for h, want in enumerate(case["active_triples"], start=1):
            frontier = ent[hop == h - 1]
            got = oracle.active_triples(E, t[:, 0], t[:, 1], frontier, None if mask is None else mask[0])
            assert got.tolist() == want, (case["note"], h)
            checked += 1
        if "walk_active_triples" in case:
            for h, want in enumerate(case["walk_active_triples"], start=1):
                got = oracle.active_triples(E, t[:, 0], t[:, 1], case["walk_levels"][h - 1],
                                            None if mask is None else mask[0])
                assert got.tolist() == want, (case["note"], "walk", h)
                checked += 1
    assert checked >= 9


# ---------------------------------------------------------------- dense q . SUB
@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("masked", [False, True])
def test_against_dense_incidence_product(seed, masked):
    w = kggen.random_tiny(900 + seed, E=18 + seed, T=50 + 7 * seed, R=3, Q=4, k=4, masked=masked)
    E, T, R = w.num_entities, w.num_triples, w.num_relations
    SUB = np.zeros((E, T), dtype=np.int64)
    OBJ = np.zeros((T, E), dtype=np.int64)
    REL = np.zeros((T, R), dtype=np.int64)
    SUB[w.subj, np.arange(T)] = 1      # Eq. 1
    OBJ[np.arange(T), w.obj] = 1       # Eq. 2
    REL[np.arange(T), w.rel] = 1       # Eq. 3
    levels = walk_levels_of(w, masked)
    for q in range(w.num_queries):
        m = np.array([int(mask_allows(w.rel_mask if masked else None, q, r)) for r in range(R)], dtype=np.int64)
        for h in range(1, w.k + 1):
            qv = np.zeros(E, dtype=np.int64)
            qv[levels[h - 1][q]] = 1
            tv = (qv @ SUB > 0) & (REL @ m > 0)                        # Eq. 5, whitelist applied
            got = oracle.active_triples(E, w.subj, w.rel, levels[h - 1][q], row_of(w, q, masked))
            assert sorted(got.tolist()) == np.nonzero(tv)[0].tolist(), (q, h)      # Eq. 6
            # the order: SUB's rows, triple indices ascending inside a subject
            keys = [(int(w.subj[t]), int(t)) for t in got]
            assert keys == sorted(keys)
            # Eq. 4: the objects of T_h are exactly level h of the walk
            nxt = np.nonzero(tv.astype(np.int64) @ OBJ)[0]
            assert nxt.tolist() == levels[h][q].tolist()
            assert sorted(set(w.obj[got].tolist())) == levels[h][q].tolist()


# ---------------------------------------------------------------- against the min-hop oracle
@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("masked", [False, True])
def test_objects_and_counts_against_minhop(seed, masked):
    w = kggen.random_tiny(950 + seed, E=60, T=260, R=4, Q=6, k=4, masked=masked)
    lv, trav = minhop_levels_of(w, masked)
    for q in range(w.num_queries):
        seen = set()
        for h in range(1, w.k + 1):
            seen |= set(lv[h - 1][q].tolist())
            got = oracle.active_triples(w.num_entities, w.subj, w.rel, lv[h - 1][q], row_of(w, q, masked))
            # new objects of T_h = the entities whose minimum hop is h
            assert sorted(set(w.obj[got].tolist()) - seen) == lv[h][q].tolist(), (q, h)
            # every subject of T_h has hop h - 1, and no triple appears twice
            assert set(w.subj[got].tolist()) <= set(lv[h - 1][q].tolist())
            assert len(set(got.tolist())) == len(got)
            if masked:
                assert all(mask_allows(w.rel_mask, q, int(w.rel[t])) for t in got)
                assert len(got) <= trav[q, h - 1]          # trav counts blocked triples too
            else:
                assert len(got) == trav[q, h - 1]


# ---------------------------------------------------------------- closed forms
def test_closed_forms():
    # a directed path 0 -> 1 -> .. -> 7, triple i = (i, 0, i + 1): T_h from seed 0 is {h - 1}
    n = 8
    s = np.arange(n - 1, dtype=np.int32)
    r = np.zeros(n - 1, dtype=np.int32)
    for h in range(1, n):
        assert oracle.active_triples(n, s, r, [h - 1]).tolist() == [h - 1]
    assert oracle.active_triples(n, s, r, [n - 1]).tolist() == []          # the last entity is no subject
    assert oracle.active_triples(n, s, r, []).tolist() == []
    # a star with the centre given last in the triple list: centre 0 -> leaves, triples reversed
    leaves = np.arange(1, 6, dtype=np.int32)
    s = np.zeros(5, dtype=np.int32)
    assert oracle.active_triples(6, s, np.zeros(5, dtype=np.int32), [0]).tolist() == [0, 1, 2, 3, 4]
    assert oracle.active_triples(6, s, np.zeros(5, dtype=np.int32), leaves).tolist() == []
    # two subjects whose triples interleave in the list: subject order wins over triple order
    s = np.array([3, 1, 3, 1, 2], dtype=np.int32)
    r = np.array([0, 1, 1, 0, 0], dtype=np.int32)
    assert oracle.active_triples(4, s, r, [3, 1]).tolist() == [1, 3, 0, 2]
    assert oracle.active_triples(4, s, r, [1, 3, 3, 1]).tolist() == [1, 3, 0, 2]      # repeats do not matter
    only1 = pack_mask([[1]], 2)[0]
    assert oracle.active_triples(4, s, r, [3, 1], only1).tolist() == [1, 2]
    # relation ids above 63 use the second mask word
    r2 = np.array([64, 1, 70, 0, 0], dtype=np.int32)
    m = pack_mask([[70, 0]], 71)[0]
    assert oracle.active_triples(4, s, r2, [1, 2, 3], m).tolist() == [3, 4, 2]


def test_every_entity_in_the_frontier_gives_every_allowed_triple():
    w = kggen.random_tiny(977, E=40, T=200, R=5, Q=2, k=1, masked=True)
    got = oracle.active_triples(w.num_entities, w.subj, w.rel, np.arange(w.num_entities), w.rel_mask[0])
    want = [t for t in np.lexsort((np.arange(w.num_triples), w.subj))
            if mask_allows(w.rel_mask, 0, int(w.rel[t]))]
    assert got.tolist() == [int(t) for t in want]
