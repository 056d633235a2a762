"""GPU parity of the active-triple export (logoskg_result_triples_offsets / _triples_fetch)
against oracle.active_triples fed with the oracle's own levels, bit-exact: the triple indices
in order, and the subject / relation / object columns against the input triples."""
import numpy as np
import pytest

import kggen
import oracle

pytestmark = pytest.mark.gpu


def lkg():
    import paper_2604_18913_amd as m
    return m


def oracle_levels(w, k, walk_exact):
    """levels[h][q] = entity array (ascending) of level h of query q, from the oracle."""
    Q = w.num_queries
    if walk_exact:
        off, ent = oracle.walk_levels(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, w.rel_mask)
        return [[ent[off[h * Q + q]:off[h * Q + q + 1]] for q in range(Q)] for h in range(k + 1)]
    ro, ent, hop, _, _ = oracle.khop(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, k, w.rel_mask)
    return [[ent[ro[q]:ro[q + 1]][hop[ro[q]:ro[q + 1]] == h] for q in range(Q)] for h in range(k + 1)]


def check(w, k, walk_exact, ranges, hops=None, graph_kw=None, host_build=False):
    m = lkg()
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, host_build=host_build, **(graph_kw or {}))
    res = g.khop(w.seed_off, w.seeds, k, w.rel_mask, walk_exact=walk_exact)
    levels = oracle_levels(w, k, walk_exact)
    total = 0
    for h in (hops or range(1, k + 1)):
        for q0, q1 in ranges:
            off, triple, subject, relation, obj = res.active_triples(h, q0, q1)
            triple = triple.cpu().numpy()
            want = [oracle.active_triples(w.num_entities, w.subj, w.rel, levels[h - 1][q],
                                          None if w.rel_mask is None else w.rel_mask[q]) for q in range(q0, q1)]
            want_off = np.concatenate([[0], np.cumsum([len(x) for x in want])]).astype(np.int64)
            assert np.array_equal(off, want_off), (h, q0, q1)
            want_t = np.concatenate(want) if want else np.zeros(0, dtype=np.int32)
            assert np.array_equal(triple, want_t), (h, q0, q1)
            assert np.array_equal(subject.cpu().numpy(), w.subj[want_t])
            assert np.array_equal(relation.cpu().numpy(), w.rel[want_t])
            assert np.array_equal(obj.cpu().numpy(), w.obj[want_t])
            total += len(want_t)
    res.close()
    g.close()
    return total


@pytest.mark.parametrize("walk_exact", [False, True])
def test_tiny_graphs_every_query_and_hop(walk_exact):
    w = kggen.config1()
    n = check(w, 4, walk_exact, [(0, w.num_queries)])
    assert n > 0
    for seed in range(4):
        w = kggen.random_tiny(800 + seed, E=50, T=220, R=5, Q=70, k=5, masked=bool(seed & 1))
        check(w, 5, walk_exact, [(0, 70), (3, 4), (64, 70), (10, 10)])


@pytest.mark.parametrize("host_build", [False, True])
def test_config2_scaled_ranges_and_hub_rows(host_build):
    w = kggen.config2(0.01)        # 1,024 queries on 16-word planes; hub subjects far above 64 triples
    n = check(w, 3, False, [(0, 3), (500, 502), (1023, 1024)], host_build=host_build)
    assert n > 10000
    check(w, 3, True, [(63, 66)], hops=[3], host_build=host_build)


def test_whitelists_on_four_and_sixteen_word_planes():
    w = kggen.config3(0.01, k=4)   # per-query relation whitelists
    assert w.rel_mask is not None
    n = check(w, 4, False, [(0, 4), (w.num_queries - 2, w.num_queries)])
    assert n > 0
    w = kggen.random_tiny(860, E=300, T=3000, R=70, Q=200, k=3, masked=True)   # relation ids above 63
    check(w, 3, True, [(0, 200)])


def test_error_paths_and_repeated_calls(tmp_path):
    m = lkg()
    w = kggen.config2(0.003, num_queries=100)
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations)
    res = g.khop(w.seed_off, w.seeds, 2)
    import ctypes
    from paper_2604_18913_amd import binding
    lib = binding._load()
    off = np.zeros(3, dtype=np.int64)
    p_off = off.ctypes.data_as(ctypes.c_void_p)
    assert lib.logoskg_result_triples_offsets(res._h, 0, 0, 2, p_off, None) != 0      # hop 0 has no triples
    assert lib.logoskg_result_triples_offsets(res._h, 3, 0, 2, p_off, None) != 0      # beyond k
    assert lib.logoskg_result_triples_offsets(res._h, 1, 2, 1, p_off, None) != 0      # bad range
    assert lib.logoskg_result_triples_fetch(res._h, 1, 0, 2, 1 << 30, None, None, None, None, None) != 0  # not prepared
    assert lib.logoskg_result_triples_offsets(res._h, 2, 0, 2, p_off, None) == 0
    n = int(off[2])
    assert n > 0
    import torch
    buf = torch.empty(n, dtype=torch.int32, device="cuda")
    assert lib.logoskg_result_triples_fetch(res._h, 2, 0, 2, n - 1, buf.data_ptr(), None, None, None, None) != 0  # capacity
    assert lib.logoskg_result_triples_fetch(res._h, 2, 0, 3, n, buf.data_ptr(), None, None, None, None) != 0      # other range
    res.level(0)                                                                       # recounts another level
    assert lib.logoskg_result_triples_fetch(res._h, 2, 0, 2, n, buf.data_ptr(), None, None, None, None) != 0
    # prepared again: two fetches in a row give the same list, and only the asked column is written
    a = res.active_triples(2, 0, 2, components=False)
    b = res.active_triples(2, 0, 2)
    assert a[2] is None and torch.equal(a[1], b[1])
    want = np.concatenate([oracle.active_triples(w.num_entities, w.subj, w.rel, lv) for lv in
                           oracle_levels(w, 2, False)[1][:2]])
    assert np.array_equal(b[1].cpu().numpy(), want)
    res.close()
    g.close()
    # shards kept in files have no pinned copy of SUB's rows to copy from: refused
    ws = kggen.config5(0.0003)
    gs = m.Graph(ws.subj, ws.rel, ws.obj, ws.num_entities, ws.num_relations, num_shards=4, shard_dir=str(tmp_path))
    rs = gs.khop(ws.seed_off, ws.seeds, 2)
    with pytest.raises(m.LogosKGError):
        rs.active_triples(1, 0, 1)
    rs.close()
    gs.close()


@pytest.mark.parametrize("walk_exact", [False, True])
def test_sharded_graphs_export_the_same_triples(walk_exact):
    # the rows of SUB are read from the pinned, shard-grouped copy; the triple indices of that order are
    # sorted out on the device at the first export
    w = kggen.config5(0.0005)
    n = check(w, 3, walk_exact, [(0, 40), (1000, 1024)], graph_kw=dict(num_shards=8, max_resident_shards=3))
    assert n > 0
    w = kggen.config3(0.004, k=3)
    n = check(w, 3, walk_exact, [(5, 9), (600, 640)], graph_kw=dict(num_shards=4), host_build=True)
    assert n > 0
