"""GPU parity of logoskg_walks (walks of exactly d allowed triples from a seed to a target, on a
LOGOSKG_WALK_EXACT result) against oracle.walk_paths, bit-exact: counts and every listed walk."""
import numpy as np
import pytest

import kggen
import oracle

pytestmark = pytest.mark.gpu


def lkg():
    import paper_2604_18913_amd as m
    return m


def check_pairs(w, k, pq, pt, pl, max_paths=16, hub_min_degree=0):
    m = lkg()
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, hub_min_degree=hub_min_degree)
    res = g.khop(w.seed_off, w.seeds, k, w.rel_mask, walk_exact=True)
    cnt, edges = g.walks(res, pq, pt, pl, max_paths)
    want_c, want_e = oracle.walk_paths(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, pq, pt, pl,
                                       max_paths, w.rel_mask)
    assert np.array_equal(cnt.cpu().numpy(), want_c)
    assert np.array_equal(edges.cpu().numpy(), want_e)
    res.close()
    g.close()
    return int(want_c.sum())


def test_every_query_target_and_length_on_tiny_graphs():
    for seed in range(4):
        w = kggen.random_tiny(1400 + seed, E=24, T=90, R=4, Q=70, k=4, masked=bool(seed & 1))
        q, v, d = np.meshgrid(np.arange(w.num_queries), np.arange(w.num_entities), np.arange(w.k + 1), indexing="ij")
        n = check_pairs(w, w.k, q.ravel(), v.ravel(), d.ravel(), max_paths=5)
        assert n > 0
    # pairs that cannot be served: bad query, bad target, bad length
    w = kggen.random_tiny(1410, E=24, T=90, R=4, Q=5, k=3)
    check_pairs(w, 3, [0, 7, -1, 0, 0, 0], [0, 0, 0, 99, -3, 1], [0, 1, 1, 1, 1, 9], max_paths=2)


def level_pairs(w, k, rng, per_level):
    """(query, target, length) samples drawn from the oracle's walk levels, plus misses."""
    Q = w.num_queries
    off, ent = oracle.walk_levels(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, w.rel_mask)
    pq, pt, pl = [], [], []
    for h in range(k + 1):
        a, b = int(off[h * Q]), int(off[(h + 1) * Q])
        if b == a:
            continue
        for pos in rng.integers(a, b, size=per_level):
            q = int(np.searchsorted(off[h * Q:(h + 1) * Q + 1], pos, side="right")) - 1
            pq.append(q); pt.append(int(ent[pos])); pl.append(h)
            pq.append(q); pt.append(int(rng.integers(0, w.num_entities))); pl.append(h)   # mostly a miss
    return np.array(pq), np.array(pt), np.array(pl)


@pytest.mark.parametrize("hub_min", [0, 60])
def test_config2_scaled_sampled_pairs(hub_min):
    w = kggen.config2(0.01)
    rng = np.random.default_rng(5)
    pq, pt, pl = level_pairs(w, 3, rng, 400)
    n = check_pairs(w, 3, pq, pt, pl, max_paths=16, hub_min_degree=hub_min)
    assert n > 1000


def test_whitelists_and_deeper_walks():
    w = kggen.config3(0.01, k=4)
    rng = np.random.default_rng(6)
    pq, pt, pl = level_pairs(w, 4, rng, 300)
    assert check_pairs(w, 4, pq, pt, pl, max_paths=8) > 0


def test_error_paths():
    m = lkg()
    w = kggen.config2(0.003, num_queries=70)
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations)
    res = g.khop(w.seed_off, w.seeds, 2)                    # minimum-hop result: no walk levels
    with pytest.raises(m.LogosKGError):
        g.walks(res, [0], [0], [0])
    res.close()
    res = g.khop(w.seed_off, w.seeds, 2, walk_exact=True)
    with pytest.raises(m.LogosKGError):
        g.walks(res, [0], [0], [0], max_paths=0)
    cnt, edges = g.walks(res, [], [], [])                   # no pairs: nothing to do
    assert cnt.numel() == 0
    res.close()
    g.close()
    # a sharded graph lists walks too (the object rows are read from pinned host memory)
    ws = kggen.config5(0.0003)
    gs = m.Graph(ws.subj, ws.rel, ws.obj, ws.num_entities, ws.num_relations, num_shards=4)
    rs = gs.khop(ws.seed_off, ws.seeds, 2, walk_exact=True)
    lo, lent = oracle.walk_levels(ws.num_entities, ws.subj, ws.rel, ws.obj, ws.seed_off, ws.seeds, 2, None)
    Q = ws.num_queries
    wq, wt = [], []
    for q in range(Q):
        for v in lent[int(lo[2 * Q + q]):int(lo[2 * Q + q + 1])][:4]:
            wq.append(q)
            wt.append(int(v))
    if wq:
        c1, e1 = gs.walks(rs, wq, wt, [2] * len(wq), 16)
        c2, e2 = oracle.walk_paths(ws.num_entities, ws.subj, ws.rel, ws.obj, ws.seed_off, ws.seeds, 2, wq, wt,
                                   [2] * len(wq), 16, None)
        assert np.array_equal(c1.cpu().numpy(), c2) and np.array_equal(e1.cpu().numpy(), e2)
    rs.close()
    gs.close()
