"""GPU parity of the per-level lists (logoskg_result_level_offsets / _level_fetch): walk-exact
levels against oracle.walk_levels, minimum-hop levels against oracle.khop, bit-exact."""
import numpy as np
import pytest

import kggen
import oracle

pytestmark = pytest.mark.gpu


def lkg():
    import paper_2604_18913_amd as m
    return m


def gpu_levels(w, k, walk_exact, direction="auto", hub_min_degree=0, num_shards=0):
    m = lkg()
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, hub_min_degree=hub_min_degree,
                **({"num_shards": num_shards} if num_shards else {}))
    res = g.khop(w.seed_off, w.seeds, k, w.rel_mask, direction=direction, walk_exact=walk_exact)
    out = []
    for h in range(k + 1):
        off, ent = res.level(h)
        out.append((off, ent.cpu().numpy()))
    reached = res.offsets()
    res.close()
    g.close()
    return out, reached


def check_walk(w, k, **kw):
    Q = w.num_queries
    want_off, want_ent = oracle.walk_levels(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, w.rel_mask)
    got, reached = gpu_levels(w, k, True, **kw)
    for h in range(k + 1):
        off, ent = got[h]
        a = want_off[h * Q:(h + 1) * Q + 1]
        assert np.array_equal(off, a - a[0]), f"level {h} offsets"
        assert np.array_equal(ent, want_ent[a[0]:a[-1]]), f"level {h} entities"
    # the reached set (union of the levels) is the minimum-hop search's
    ro = oracle.khop(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, w.rel_mask)[0]
    assert np.array_equal(reached, ro)


@pytest.mark.parametrize("direction", ["auto", "push", "pull"])
def test_walk_exact_tiny_and_cycles(direction):
    check_walk(kggen.config1(), 4, direction=direction)
    for seed in range(4):
        check_walk(kggen.random_tiny(700 + seed, E=40, T=160, R=4, Q=70, k=6, masked=bool(seed & 1)), 6,
                   direction=direction)


@pytest.mark.parametrize("direction,hub_min", [("auto", 0), ("push", 60), ("pull", 60)])
def test_walk_exact_config2_and_masks(direction, hub_min):
    check_walk(kggen.config2(0.01), 3, direction=direction, hub_min_degree=hub_min)
    check_walk(kggen.config3(0.01, k=4), 4, direction=direction, hub_min_degree=hub_min)


def test_walk_exact_on_a_sharded_graph():
    check_walk(kggen.config5(0.0003), 3, num_shards=4)


def test_min_hop_levels_and_error_paths():
    m = lkg()
    w = kggen.config2(0.005, num_queries=300)
    ro, ent, hop, _, _ = oracle.khop(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k)
    got, _ = gpu_levels(w, w.k, False, hub_min_degree=100)
    for h in range(w.k + 1):
        off, e = got[h]
        want = [ent[ro[q]:ro[q + 1]][hop[ro[q]:ro[q + 1]] == h] for q in range(w.num_queries)]
        assert np.array_equal(off, np.concatenate([[0], np.cumsum([len(x) for x in want])]))
        assert np.array_equal(e, np.concatenate(want))
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations)
    res = g.khop(w.seed_off, w.seeds, 2, walk_exact=True)
    with pytest.raises(m.LogosKGError):
        res.fetch()                      # hop / pred are not defined for walk-exact levels
    with pytest.raises(m.LogosKGError):
        g.paths(res, [0], [0])
    with pytest.raises(m.LogosKGError):
        res.level(3)                     # beyond k
    off, e = res.level(1, 5, 70)         # a sub-range of the queries
    want_off, want_ent = oracle.walk_levels(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, 2)
    Q = w.num_queries
    assert np.array_equal(e.cpu().numpy(), want_ent[want_off[Q + 5]:want_off[Q + 70]])
    res.close()
    g.close()
