"""Seeded random differential test: small random graphs with random shapes (entities, triples,
relations, queries across the 1 / 4 / 16-word plane sizes, hops, whitelists, direction, hub
threshold, search mode), every public result checked against the oracle bit for bit."""
import numpy as np
import pytest

import kggen
import oracle

pytestmark = pytest.mark.gpu

QUERIES = [1, 5, 64, 65, 200, 256, 257, 700, 1024]


def lkg():
    import paper_2604_18913_amd as m
    return m


def one_case(seed):
    rng = np.random.default_rng(9000 + seed)
    E = int(rng.integers(20, 3000))
    T = int(E * rng.uniform(1.0, 12.0))
    R = int(rng.integers(1, 80))
    Q = int(QUERIES[rng.integers(0, len(QUERIES))])
    k = int(rng.integers(0, 8))
    masked = bool(rng.integers(0, 2))
    direction = ["auto", "push", "pull"][rng.integers(0, 3)]
    hub_min = int([0, 40, 200][rng.integers(0, 3)])
    walk = bool(rng.integers(0, 3) == 0)
    shards = int([0, 0, 0, 2, 5][rng.integers(0, 5)])     # Alg. 1: subject-partitioned graph behind a shard cache
    resident = int(rng.integers(1, shards + 1)) if shards else 0
    if seed % 3 == 0:   # power-law degrees: long and hub object rows, dense frontiers
        scale = float(rng.uniform(0.0005, 0.004))
        k = min(k, 4)
        w = kggen.config3(scale, k=k, num_queries=Q) if masked else kggen.config2(scale, num_queries=Q)
        E, R = w.num_entities, w.num_relations
    else:
        w = kggen.random_tiny(5000 + seed, E=E, T=T, R=R, Q=Q, k=k, masked=masked, max_seeds=4)
    what = dict(seed=seed, E=E, T=w.num_triples, R=R, Q=Q, k=k, masked=masked, direction=direction,
                hub_min=hub_min, walk=walk, shards=shards, resident=resident)
    print(what, flush=True)
    m = lkg()
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, hub_min_degree=hub_min,
                host_build=bool(seed % 5 == 0), num_shards=shards, max_resident_shards=resident)
    res = g.khop(w.seed_off, w.seeds, k, w.rel_mask, direction=direction, walk_exact=walk)
    want = oracle.khop(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, w.rel_mask)
    assert np.array_equal(res.offsets(), want[0]), what          # the reached set is the same in both modes
    q0 = int(rng.integers(0, Q))
    q1 = int(rng.integers(q0, Q + 1))
    if walk:
        loff, lent = oracle.walk_levels(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, w.rel_mask)
        levels = [[lent[loff[h * Q + q]:loff[h * Q + q + 1]] for q in range(Q)] for h in range(k + 1)]
        for h in range(k + 1):
            off, ent = res.level(h, q0, q1)
            a = loff[h * Q:(h + 1) * Q + 1]
            assert np.array_equal(off, a - a[0]), (what, h)
            assert np.array_equal(ent.cpu().numpy(), lent[a[q0]:a[q1]]), (what, h)
        if k > 0:   # walks to sampled members of the last non-empty level
            h = max(hh for hh in range(k + 1) if any(len(x) for x in levels[hh]))
            qs = [q for q in range(Q) if len(levels[h][q])][:40]
            pt = [int(levels[h][q][rng.integers(0, len(levels[h][q]))]) for q in qs]
            cnt, edges = g.walks(res, qs, pt, [h] * len(qs), 8)
            c_o, e_o = oracle.walk_paths(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, qs, pt,
                                         [h] * len(qs), 8, w.rel_mask)
            assert np.array_equal(cnt.cpu().numpy(), c_o) and np.array_equal(edges.cpu().numpy(), e_o), what
    else:
        ent, hop, pred = res.fetch()
        assert np.array_equal(ent.cpu().numpy(), want[1]), what
        assert np.array_equal(hop.cpu().numpy(), want[2]), what
        assert np.array_equal(pred.cpu().numpy(), want[3]), what
        if k > 0:
            assert np.array_equal(res.traversed().cpu().numpy(), want[4]), what
        ent, hop, pred = res.fetch(q0, q1)
        a, b = want[0][q0], want[0][q1]
        assert np.array_equal(ent.cpu().numpy(), want[1][a:b]) and np.array_equal(pred.cpu().numpy(), want[3][a:b]), what
        qe = min(Q, (q0 // 64 + 1) * 64)   # a fetch that stays inside one 64-query word
        if qe > q0:
            ent, hop, pred = res.fetch(q0, qe)
            a, b = want[0][q0], want[0][qe]
            assert np.array_equal(ent.cpu().numpy(), want[1][a:b]) and np.array_equal(hop.cpu().numpy(), want[2][a:b]), what
            assert np.array_equal(pred.cpu().numpy(), want[3][a:b]), what
        levels = [[want[1][want[0][q]:want[0][q + 1]][want[2][want[0][q]:want[0][q + 1]] == h] for q in range(Q)]
                  for h in range(k + 1)]
        if want[0][-1] > 0:
            pq, pt = kggen.sample_reached_pairs(seed, want[0], want[1], 60)
            cnt, edges = g.paths(res, pq, pt, 8)
            c_o, e_o = oracle.paths(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, pq, pt, 8, w.rel_mask)
            assert np.array_equal(cnt.cpu().numpy(), c_o) and np.array_equal(edges.cpu().numpy(), e_o), what
    if k > 0:
        h = int(rng.integers(1, k + 1))
        off, t, s_, r_, o_ = res.active_triples(h, q0, q1)
        want_t = [oracle.active_triples(w.num_entities, w.subj, w.rel, levels[h - 1][q],
                                        None if w.rel_mask is None else w.rel_mask[q]) for q in range(q0, q1)]
        assert np.array_equal(off, np.concatenate([[0], np.cumsum([len(x) for x in want_t])])), (what, h)
        cat = np.concatenate(want_t) if want_t else np.zeros(0, dtype=np.int32)
        assert np.array_equal(t.cpu().numpy(), cat), (what, h)
        assert np.array_equal(o_.cpu().numpy(), w.obj[cat]) and np.array_equal(r_.cpu().numpy(), w.rel[cat])
    # bulk export: every chain of one (query, length), numbered, against the oracle's listing per target
    q = int(rng.integers(0, Q))
    d = int(rng.integers(0, k + 1))
    targets = levels[d][q]
    total = res.walks_count(q, d)
    if len(targets) == 0:
        assert total == 0, what
    else:
        qs = np.full(len(targets), q, np.int32)
        cap = 2000
        if walk:
            c_o, e_o = oracle.walk_paths(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, qs, targets,
                                         np.full(len(targets), d, np.int32), cap, w.rel_mask)
        else:
            c_o, e_o = oracle.paths(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, qs, targets, cap,
                                    w.rel_mask)
        if c_o.max() < cap:   # the oracle listed every chain of every target
            assert total == int(c_o.sum()), (what, q, d)
            e, t = res.walks_fetch(q, d, 0, total)
            assert np.array_equal(t.cpu().numpy(), np.repeat(targets, c_o)), (what, q, d)
            want_e = np.concatenate([e_o[i, :c_o[i], :d] for i in range(len(targets))]).reshape(total, d)
            assert np.array_equal(e.cpu().numpy(), want_e), (what, q, d)
        else:
            assert total >= int(c_o.sum()), (what, q, d)
    res.close()
    g.close()


@pytest.mark.parametrize("block", range(10))
def test_random_cases(block):
    for seed in range(block * 24, block * 24 + 24):
        one_case(seed)
