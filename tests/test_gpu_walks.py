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


def bulk_expected(w, k, q, d, walk_exact, cap):
    """Every chain of d triples of query q from the oracle: targets ascending (level d of the walk
    levels, or the entities at hop d), each target's chains in (t_d, .., t_1) order."""
    Q = w.num_queries
    if walk_exact:
        off, ent = oracle.walk_levels(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, w.rel_mask)
        targets = ent[int(off[d * Q + q]):int(off[d * Q + q + 1])]
    else:
        ro, ent, hop, _, _ = oracle.khop(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, w.rel_mask)
        a, b = int(ro[q]), int(ro[q + 1])
        targets = ent[a:b][hop[a:b] == d]
    n = len(targets)
    if n == 0:
        return np.zeros((0, d), np.int32), np.zeros(0, np.int32)
    qs = np.full(n, q, np.int32)
    if walk_exact:
        cnt, edges = oracle.walk_paths(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, qs, targets,
                                       np.full(n, d, np.int32), cap, w.rel_mask)
    else:
        cnt, edges = oracle.paths(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, qs, targets, cap,
                                  w.rel_mask)
    assert cnt.max() < cap, "raise the oracle's bound: a target has more chains than it lists"
    rows = [edges[i, :cnt[i], :d] for i in range(n)]
    return np.concatenate(rows).reshape(int(cnt.sum()), d), np.repeat(targets, cnt).astype(np.int32)


def check_bulk(w, k, queries, walk_exact, cap=4096, page=777, **graph_opts):
    m = lkg()
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, **graph_opts)
    res = g.khop(w.seed_off, w.seeds, k, w.rel_mask, walk_exact=walk_exact)
    listed = 0
    for q in queries:
        for d in range(k + 1):
            want_e, want_t = bulk_expected(w, k, q, d, walk_exact, cap)
            total = res.walks_count(q, d)
            assert total == len(want_t), f"query {q} length {d}: number of chains"
            got_e, got_t = [], []
            for first in range(0, total, page):      # page through the whole list with a fixed buffer
                e, t = res.walks_fetch(q, d, first, min(page, total - first))
                got_e.append(e.cpu().numpy())
                got_t.append(t.cpu().numpy())
            if total:
                assert np.array_equal(np.concatenate(got_t), want_t), f"query {q} length {d}: targets"
                assert np.array_equal(np.concatenate(got_e), want_e), f"query {q} length {d}: chains"
                lo = total // 3                      # any page can be asked for on its own
                e, t = res.walks_fetch(q, d, lo, min(5, total - lo))
                assert np.array_equal(e.cpu().numpy(), want_e[lo:lo + 5]) and np.array_equal(t.cpu().numpy(), want_t[lo:lo + 5])
            listed += total
            with pytest.raises(m.LogosKGError):
                res.walks_fetch(q, d, total, 1)      # past the end
    with pytest.raises(m.LogosKGError):
        res.walks_count(w.num_queries, 0)
    with pytest.raises(m.LogosKGError):
        res.walks_count(0, k + 1)
    with pytest.raises(m.LogosKGError):
        res.walks_fetch(queries[0], k + 5, 0, 0)     # not the (query, length) counted last
    res.close()
    g.close()
    return listed


@pytest.mark.parametrize("walk_exact", [True, False])
def test_bulk_chains_every_query_on_tiny_graphs(walk_exact):
    # every chain of every length of every query: walks of d triples (walk-exact result) and all
    # shortest paths to the entities at hop d (minimum-hop result)
    for seed in range(3):
        w = kggen.random_tiny(1500 + seed, E=30, T=100, R=4, Q=70, k=4, masked=bool(seed & 1))
        n = check_bulk(w, w.k, range(w.num_queries), walk_exact, cap=20000)
        assert n > 0


@pytest.mark.parametrize("walk_exact", [True, False])
def test_bulk_chains_on_scaled_workloads(walk_exact):
    w = kggen.config1()
    assert check_bulk(w, 2, [0, 5, 33, 63], walk_exact) > 0
    w = kggen.config3(0.002, k=3)                       # whitelists, 16-word planes
    live = np.nonzero(np.diff(oracle.khop(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, 3,
                                          w.rel_mask)[0]) > 3)[0]
    assert check_bulk(w, 3, [int(x) for x in live[:4]] + [1023], walk_exact, cap=60000, hub_min_degree=64) > 0
    ws = kggen.config5(0.0003)                          # sharded: rows read from pinned host memory
    live = np.nonzero(np.diff(oracle.khop(ws.num_entities, ws.subj, ws.rel, ws.obj, ws.seed_off, ws.seeds, 2,
                                          None)[0]) > 3)[0]
    assert check_bulk(ws, 2, [int(x) for x in live[:3]], walk_exact, cap=20000, num_shards=4) > 0
