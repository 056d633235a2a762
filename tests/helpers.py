"""Shared test helpers: result unpacking and brute-force definitions used to pin
the oracle.  Nothing here is used by the product path."""
from __future__ import annotations

import sys
import time

import numpy as np

PYTEST_CONFIG = None  # set by conftest.py


def progress(*a):
    """One time-stamped line on the real terminal, past pytest's capture: the full-size cases run
    for minutes, and every finished step of theirs says so."""
    line = time.strftime("%H:%M:%S") + " " + " ".join(str(x) for x in a)
    capman = PYTEST_CONFIG.pluginmanager.getplugin("capturemanager") if PYTEST_CONFIG is not None else None
    if capman is None:
        print(line, flush=True)
        return
    with capman.global_and_fixture_disabled():
        sys.stderr.write("\n" + line)
        sys.stderr.flush()


def pack_mask(allowed_lists, R):
    """allowed_lists[q] = iterable of relation ids or None (= all)."""
    rw = (R + 63) // 64
    m = np.zeros((len(allowed_lists), rw), dtype=np.uint64)
    for q, al in enumerate(allowed_lists):
        ids = range(R) if al is None else al
        for r in ids:
            m[q, r // 64] |= np.uint64(1) << np.uint64(r % 64)
    return m


def mask_allows(mask, q, r):
    if mask is None:
        return True
    return bool((int(mask[q, r // 64]) >> (r % 64)) & 1)


def split_result(reached_off, entity, hop, pred):
    """-> list over queries of dict entity -> (hop, pred)."""
    out = []
    for q in range(len(reached_off) - 1):
        a, b = int(reached_off[q]), int(reached_off[q + 1])
        out.append({int(e): (int(h), int(p)) for e, h, p in zip(entity[a:b], hop[a:b], pred[a:b])})
    return out


def brute_force_query(subj, rel, obj, seeds, k, allowed):
    """Enumerate every walk of length <= k from the seeds through allowed
    triples.  Returns (hop dict, pred dict, walks-by-end dict) where
    walks[v] lists all walks (tuples of edge ids) of length hop[v] ending in v.
    `allowed` is a set of relation ids or None."""
    T = len(subj)
    out_edges = {}
    for t in range(T):
        if allowed is None or int(rel[t]) in allowed:
            out_edges.setdefault(int(subj[t]), []).append(t)
    best = {}
    walks = {}
    frontier = [((), int(s)) for s in sorted(set(int(x) for x in seeds))]
    for _, s in frontier:
        best[s] = 0
        walks[s] = [()]
    for h in range(1, k + 1):
        nxt = []
        for w, v in frontier:
            for t in out_edges.get(v, []):
                nxt.append((w + (t,), int(obj[t])))
        frontier = nxt
        for w, v in frontier:
            if v not in best:
                best[v] = h
                walks[v] = []
            if best[v] == h:
                walks[v].append(w)
    pred = {v: (-1 if best[v] == 0 else min(w[-1] for w in walks[v])) for v in best}
    return best, pred, walks


def brute_force_paths(walks_v, max_paths):
    """Order shortest walks by the edge sequence read from the target backward
    and keep the first max_paths."""
    uniq = sorted(set(walks_v), key=lambda w: tuple(reversed(w)))
    return uniq[:max_paths]


def check_invariants(subj, rel, obj, seed_off, seeds, k, rel_mask, reached_off, entity, hop, pred,
                     queries=None):
    """Properties that any correct (hop, pred) output satisfies, at any size."""
    subj = np.asarray(subj)
    rel = np.asarray(rel)
    obj = np.asarray(obj)
    E = int(max(subj.max(initial=0), obj.max(initial=0))) + 1
    Q = len(reached_off) - 1
    for q in (range(Q) if queries is None else queries):
        a, b = int(reached_off[q]), int(reached_off[q + 1])
        ent, hp, pr = entity[a:b], hop[a:b].astype(np.int64), pred[a:b]
        assert np.all(np.diff(ent) > 0), "entities must ascend strictly"
        h_of = np.full(E, 255, dtype=np.int64)
        h_of[ent] = hp
        sd = np.unique(seeds[int(seed_off[q]):int(seed_off[q + 1])])
        assert np.all(h_of[sd] == 0)
        assert set(ent[hp == 0].tolist()) == set(sd.tolist())
        assert np.all(pr[hp == 0] == -1)
        assert hp.max(initial=0) <= k
        nz = hp > 0
        pe = pr[nz]
        assert np.all(pe >= 0)
        assert np.array_equal(obj[pe], ent[nz]), "pred edge must end in the entity"
        assert np.array_equal(h_of[subj[pe]], hp[nz] - 1), "pred subject one hop closer"
        if rel_mask is None:
            ok = np.ones(subj.shape[0], dtype=bool)
        else:
            words = rel_mask[q][rel >> 6]
            ok = ((words >> (rel & 63).astype(np.uint64)) & np.uint64(1)).astype(bool)
        assert np.all(ok[pe]), "pred edge relation must be allowed"
        hs, ho = h_of[subj], h_of[obj]
        live = ok & (hs < k)
        assert np.all(ho[live] <= hs[live] + 1), "an allowed edge out of a reached subject was missed"
        # minimality of the predecessor edge id
        cand = ok & (hs + 1 == ho) & (ho <= k)
        best = np.full(E, np.iinfo(np.int64).max, dtype=np.int64)
        np.minimum.at(best, obj[cand], np.nonzero(cand)[0])
        assert np.array_equal(best[ent[nz]], pe.astype(np.int64)), "pred must be the smallest valid edge id"
