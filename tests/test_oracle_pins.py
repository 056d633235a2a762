"""Pins for the CPU oracle (no GPU): every output integer of oracle.khop and
oracle.paths is checked against something that is not the oracle itself --
dense boolean products of the incidence matrices (paper Eq. 1-4), brute-force
walk enumeration, closed forms, networkx / scipy shortest-path lengths, a
hand-worked example, and invariants."""
import json
import os

import numpy as np
import pytest

import kggen
import oracle
from helpers import (brute_force_paths, brute_force_query, check_invariants, mask_allows,
                     pack_mask, split_result)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run_oracle(w, mode=0, k=None):
    return oracle.khop(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds,
                       w.k if k is None else k, w.rel_mask, mode=mode)


def one_query(E, triples, seeds, k, allowed=None, R=None, mode=0):
    t = np.asarray(triples, dtype=np.int32).reshape(-1, 3)
    R = int(t[:, 1].max(initial=0)) + 1 if R is None else R
    mask = None if allowed is None else pack_mask([allowed], R)
    off = np.array([0, len(seeds)], dtype=np.int64)
    ro, ent, hop, pred, trav = oracle.khop(E, t[:, 0], t[:, 1], t[:, 2], off,
                                           np.asarray(seeds, np.int32), k, mask, mode=mode)
    return ent.tolist(), hop.tolist(), pred.tolist(), trav[0].tolist()


# ---------------------------------------------------------------- pin 0: hand-worked example
@pytest.mark.parametrize("mode", [0, 1])
def test_hand_worked_example(mode):
    g = json.load(open(os.path.join(GOLDEN, "worked_example.json")))
    t = np.asarray(g["triples_s_r_o"], dtype=np.int32)
    for case in g["cases"]:
        ent, hop, pred, trav = one_query(g["num_entities"], t, case["seeds"], case["k"],
                                         case["allowed_relations"], g["num_relations"], mode)
        assert ent == case["entity"], case["note"]
        assert hop == case["hop"], case["note"]
        assert pred == case["pred"], case["note"]
        assert trav == case["traversed"], case["note"]
        mask = (None if case["allowed_relations"] is None
                else pack_mask([case["allowed_relations"]], g["num_relations"]))
        cnt, edges = oracle.paths(g["num_entities"], t[:, 0], t[:, 1], t[:, 2],
                                  np.array([0, len(case["seeds"])], np.int64),
                                  np.asarray(case["seeds"], np.int32), case["k"],
                                  [0], [case["paths"]["target"]], case["paths"]["max_paths"], mask)
        want = case["paths"]["edges"]
        assert cnt[0] == len(want)
        for i, p in enumerate(want):
            row = edges[0, i].tolist()
            assert row[:len(p)] == p and all(x == -1 for x in row[len(p):])


# ---------------------------------------------------------------- pin 1: dense SUB / REL / OBJ products
def dense_matrices(w):
    E, T, R = w.num_entities, w.num_triples, w.num_relations
    SUB = np.zeros((E, T), dtype=bool)
    OBJ = np.zeros((T, E), dtype=bool)
    REL = np.zeros((T, R), dtype=bool)
    SUB[w.subj, np.arange(T)] = True      # Eq. 1
    OBJ[np.arange(T), w.obj] = True       # Eq. 2
    REL[np.arange(T), w.rel] = True       # Eq. 3
    return SUB, OBJ, REL


def bool_mm(a, b):
    return (a.astype(np.int64) @ b.astype(np.int64)) > 0


@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("masked", [False, True])
def test_against_boolean_matrix_powers(seed, masked):
    w = kggen.random_tiny(seed, E=24 + seed, T=70 + 5 * seed, R=3, Q=6, k=4, masked=masked)
    SUB, OBJ, REL = dense_matrices(w)
    ro, ent, hop, pred, trav = run_oracle(w)
    res = split_result(ro, ent, hop, pred)
    for q in range(w.num_queries):
        m = np.ones(w.num_relations, dtype=bool)
        if masked:
            m = np.array([mask_allows(w.rel_mask, q, r) for r in range(w.num_relations)])
        qv = np.zeros((1, w.num_entities), dtype=bool)
        qv[0, w.seeds[w.seed_off[q]:w.seed_off[q + 1]]] = True
        first = {int(e): 0 for e in np.nonzero(qv[0])[0]}
        for h in range(1, w.k + 1):
            t_active = bool_mm(qv, SUB)                     # Eq. 5
            assert int(t_active.sum()) >= 0
            t_allowed = t_active & bool_mm(REL, m[:, None]).T
            qv = bool_mm(t_allowed, OBJ)                    # Eq. 4
            for e in np.nonzero(qv[0])[0]:
                first.setdefault(int(e), h)
        assert {e: hp for e, (hp, _) in res[q].items()} == first


def test_walk_exact_vector_differs_from_min_hop_on_cycles():
    # q^(k) of the plain iteration marks ends of length-k walks; on a 2-cycle the
    # seed reappears at k=2 while its minimum hop stays 0.
    ent, hop, pred, _ = one_query(2, [[0, 0, 1], [1, 0, 0]], [0], 2)
    assert ent == [0, 1] and hop == [0, 1] and pred == [-1, 0]


# ---------------------------------------------------------------- pin 2: brute-force walks (hop, pred, traversed, paths)
@pytest.mark.parametrize("seed", range(10))
@pytest.mark.parametrize("masked", [False, True])
def test_against_walk_enumeration(seed, masked):
    w = kggen.random_tiny(50 + seed, E=14 + seed, T=30 + 3 * seed, R=3, Q=5, k=3, masked=masked)
    ro, ent, hop, pred, trav = run_oracle(w)
    res = split_result(ro, ent, hop, pred)
    outdeg = np.bincount(w.subj, minlength=w.num_entities)
    pq, pt = [], []
    expect_paths = []
    for q in range(w.num_queries):
        allowed = None
        if masked:
            allowed = {r for r in range(w.num_relations) if mask_allows(w.rel_mask, q, r)}
        sd = w.seeds[w.seed_off[q]:w.seed_off[q + 1]]
        best, bpred, walks = brute_force_query(w.subj, w.rel, w.obj, sd, w.k, allowed)
        assert res[q] == {v: (best[v], bpred[v]) for v in best}
        for h in range(1, w.k + 1):
            assert trav[q, h - 1] == sum(int(outdeg[v]) for v in best if best[v] == h - 1)
        for v in range(w.num_entities):
            pq.append(q)
            pt.append(v)
            expect_paths.append(brute_force_paths(walks[v], 4) if v in best else [])
    cnt, edges = oracle.paths(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k,
                              pq, pt, 4, w.rel_mask)
    for i, want in enumerate(expect_paths):
        assert cnt[i] == len(want)
        for j, p in enumerate(want):
            row = edges[i, j].tolist()
            assert tuple(row[:len(p)]) == p and all(x == -1 for x in row[len(p):])
        assert np.all(edges[i, len(want):] == -1)


def test_first_path_is_the_pred_chain():
    w = kggen.config2(0.002, num_queries=16)
    ro, ent, hop, pred, _ = run_oracle(w)
    res = split_result(ro, ent, hop, pred)
    pq, pt = kggen.sample_reached_pairs(0, ro, ent, 300)
    cnt, edges = oracle.paths(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k,
                              pq, pt, 16, None)
    for i in range(len(pq)):
        q, v = int(pq[i]), int(pt[i])
        d = res[q][v][0]
        chain = []
        x = v
        while res[q][x][1] >= 0:
            t = res[q][x][1]
            chain.append(t)
            x = int(w.subj[t])
        assert len(chain) == d and cnt[i] >= 1
        assert edges[i, 0, :d].tolist() == chain[::-1]
        keys = [tuple(edges[i, j, :d][::-1]) for j in range(cnt[i])]
        assert keys == sorted(set(keys))


# ---------------------------------------------------------------- pin 3: closed forms
@pytest.mark.parametrize("mode", [0, 1])
def test_directed_path(mode):
    n = 12
    tri = [[i, 0, i + 1] for i in range(n - 1)]
    ent, hop, pred, trav = one_query(n, tri, [3], 5, mode=mode)
    assert ent == list(range(3, 9))
    assert hop == [v - 3 for v in ent]
    assert pred == [-1] + [v - 1 for v in ent[1:]]
    assert trav == [1] * 5


@pytest.mark.parametrize("mode", [0, 1])
def test_directed_cycle_never_lowers_the_seed(mode):
    n = 5
    tri = [[i, 0, (i + 1) % n] for i in range(n)]
    ent, hop, pred, _ = one_query(n, tri, [2], 9, mode=mode)
    assert ent == [0, 1, 2, 3, 4]
    assert hop == [3, 4, 0, 1, 2]
    assert pred == [4, 0, -1, 2, 3]


def test_out_star_and_in_star():
    n = 9
    out_star = [[0, 0, i] for i in range(1, n)]
    ent, hop, pred, trav = one_query(n, out_star, [0], 3)
    assert ent == list(range(n)) and hop == [0] + [1] * (n - 1) and pred == [-1] + list(range(n - 1))
    assert trav == [n - 1, 0, 0]
    in_star = [[i, 0, 0] for i in range(1, n)]
    ent, hop, pred, _ = one_query(n, in_star, [0], 3)
    assert ent == [0] and hop == [0] and pred == [-1]
    ent, hop, pred, _ = one_query(n, in_star, [4, 6], 3)
    assert ent == [0, 4, 6] and hop == [1, 0, 0] and pred == [3, -1, -1]


@pytest.mark.parametrize("b,k", [(2, 4), (3, 3), (5, 2)])
def test_complete_tree_size(b, k):
    depth = k + 1
    n = (b ** (depth + 1) - 1) // (b - 1)
    tri = [[(c - 1) // b, 0, c] for c in range(1, n)]
    ent, hop, pred, trav = one_query(n, tri, [0], k)
    assert len(ent) == (b ** (k + 1) - 1) // (b - 1)
    assert [hop.count(h) for h in range(k + 1)] == [b ** h for h in range(k + 1)]
    assert trav == [b ** h for h in range(1, k + 1)]


def test_complete_bipartite():
    a, b = 4, 5
    tri = [[i, 0, a + j] for i in range(a) for j in range(b)]
    ent, hop, pred, _ = one_query(a + b, tri, [1, 2], 2)
    assert ent == [1, 2] + list(range(a, a + b))
    assert hop == [0, 0] + [1] * b
    assert pred == [-1, -1] + [b + j for j in range(b)]   # edges of subject 1 come first


def test_tie_break_smallest_edge_id_and_mask_selects_other_edge():
    tri = [[0, 1, 1], [0, 0, 1], [1, 0, 2], [0, 1, 2]]
    ent, hop, pred, _ = one_query(3, tri, [0], 2)
    assert (ent, hop, pred) == ([0, 1, 2], [0, 1, 1], [-1, 0, 3])
    ent, hop, pred, _ = one_query(3, tri, [0], 2, allowed=[0], R=2)
    assert (ent, hop, pred) == ([0, 1, 2], [0, 1, 2], [-1, 1, 2])
    ent, hop, pred, _ = one_query(3, tri, [0], 2, allowed=[], R=2)
    assert (ent, hop, pred) == ([0], [0], [-1])


def test_duplicate_seeds_collapse_and_self_loops():
    tri = [[0, 0, 0], [0, 0, 1], [1, 0, 1]]
    ent, hop, pred, trav = one_query(2, tri, [0, 0, 0], 3)
    assert (ent, hop, pred) == ([0, 1], [0, 1], [-1, 1])
    assert trav == [2, 1, 0]


# ---------------------------------------------------------------- pin 4: library shortest paths
def test_against_networkx_and_scipy_on_config1():
    import networkx as nx
    from scipy.sparse import coo_matrix
    from scipy.sparse.csgraph import shortest_path

    w = kggen.config1()
    ro, ent, hop, pred, _ = run_oracle(w, k=3)
    res = split_result(ro, ent, hop, pred)
    G = nx.DiGraph()
    G.add_nodes_from(range(w.num_entities))
    G.add_edges_from(zip(w.subj.tolist(), w.obj.tolist()))
    A = coo_matrix((np.ones(w.num_triples), (w.subj, w.obj)),
                   shape=(w.num_entities,) * 2).tocsr()
    A.data[:] = 1.0
    for q in range(w.num_queries):
        sd = sorted(set(w.seeds[w.seed_off[q]:w.seed_off[q + 1]].tolist()))
        want = {}
        for s in sd:
            for v, d in nx.single_source_shortest_path_length(G, s, cutoff=3).items():
                want[v] = min(d, want.get(v, 99))
        got = {e: h for e, (h, _) in res[q].items()}
        assert got == want
        if q < 8:
            dist = shortest_path(A, method="D", directed=True, unweighted=True, indices=sd)
            dmin = dist.min(axis=0)
            assert got == {int(v): int(dmin[v]) for v in np.nonzero(dmin <= 3)[0]}


def test_multi_seed_against_networkx_super_source():
    import networkx as nx
    w = kggen.config2(0.001, num_queries=40)
    ro, ent, hop, pred, _ = run_oracle(w)
    res = split_result(ro, ent, hop, pred)
    G = nx.DiGraph()
    G.add_edges_from(zip(w.subj.tolist(), w.obj.tolist()))
    for q in range(w.num_queries):
        H = G.copy()
        sd = set(w.seeds[w.seed_off[q]:w.seed_off[q + 1]].tolist())
        H.add_edges_from(("S", s) for s in sd)
        want = {v: d - 1 for v, d in nx.single_source_shortest_path_length(H, "S", cutoff=w.k + 1).items()
                if v != "S"}
        assert {e: h for e, (h, _) in res[q].items()} == want


# ---------------------------------------------------------------- pin 5: invariants at larger sizes
@pytest.mark.parametrize("make", [lambda: kggen.config1(),
                                  lambda: kggen.config2(0.01, num_queries=24),
                                  lambda: kggen.config3(0.01, k=4, num_queries=24),
                                  lambda: kggen.config4(0.002, num_queries=16),
                                  lambda: kggen.config5(0.0003, num_queries=16)])
def test_invariants(make):
    w = make()
    ro, ent, hop, pred, trav = run_oracle(w)
    check_invariants(w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k, w.rel_mask, ro, ent, hop, pred)
    # results for k restricted to hop <= k-1 equal results for k-1
    ro2, ent2, hop2, pred2, trav2 = run_oracle(w, k=w.k - 1)
    keep = hop <= w.k - 1
    assert np.array_equal(ent[keep], ent2) and np.array_equal(hop[keep], hop2)
    assert np.array_equal(pred[keep], pred2)
    assert np.array_equal(trav[:, : w.k - 1], trav2)


def test_all_ones_mask_equals_no_mask_and_single_relation_equals_subgraph():
    w = kggen.config2(0.003, num_queries=12)
    base = run_oracle(w)
    w.rel_mask = pack_mask([None] * w.num_queries, w.num_relations)
    full = run_oracle(w)
    assert all(np.array_equal(a, b) for a, b in zip(base, full))
    r0 = 0
    w.rel_mask = pack_mask([[r0]] * w.num_queries, w.num_relations)
    ro, ent, hop, pred, _ = run_oracle(w)
    sel = np.nonzero(w.rel == r0)[0]
    sub = oracle.khop(w.num_entities, w.subj[sel], w.rel[sel], w.obj[sel], w.seed_off, w.seeds, w.k)
    assert np.array_equal(ro, sub[0]) and np.array_equal(ent, sub[1]) and np.array_equal(hop, sub[2])
    remapped = np.where(sub[3] >= 0, sel[np.maximum(sub[3], 0)], -1)
    assert np.array_equal(pred, remapped)


def test_query_permutation_only_permutes_results():
    w = kggen.config3(0.003, k=3, num_queries=20)
    base = split_result(*run_oracle(w)[:4])
    perm = np.random.default_rng(5).permutation(w.num_queries)
    lens = np.diff(w.seed_off)
    off2 = np.zeros_like(w.seed_off)
    np.cumsum(lens[perm], out=off2[1:])
    seeds2 = np.concatenate([w.seeds[w.seed_off[p]:w.seed_off[p + 1]] for p in perm])
    r2 = oracle.khop(w.num_entities, w.subj, w.rel, w.obj, off2, seeds2, w.k, w.rel_mask[perm])
    got = split_result(*r2[:4])
    for i, p in enumerate(perm):
        assert got[i] == base[p]


# ---------------------------------------------------------------- pin 6: index-free variant
@pytest.mark.parametrize("make", [lambda: kggen.config1(),
                                  lambda: kggen.config2(0.01, num_queries=48),
                                  lambda: kggen.config3(0.01, k=4, num_queries=48)])
def test_rescan_variant_equals_indexed(make):
    w = make()
    a = run_oracle(w, mode=0)
    b = run_oracle(w, mode=1)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))


def test_oracle_rejects_bad_arguments():
    with pytest.raises(RuntimeError):
        one_query(3, [[0, 0, 1]], [7], 1)
    with pytest.raises(RuntimeError):
        one_query(3, [[0, 0, 1]], [0], 255)


# ---------------------------------------------------------------- Sec. 3.4: partition and cache accounting
def test_partition_properties_and_lru_accounting():
    from oracle import partition as part
    w = kggen.config5(0.0005, num_queries=64)
    for m in (2, 8):
        P, loads = part.degree_aware_partition(w.num_entities, w.subj, m)
        part.check_partition_properties(w.num_entities, w.subj, P, loads, m)
    # the heaviest subjects land in different shards
    deg = np.bincount(w.subj, minlength=w.num_entities)
    top = np.argsort(-deg, kind="stable")[:8]
    P, _ = part.degree_aware_partition(w.num_entities, w.subj, 8)
    assert len(set(P[top].tolist())) == 8
    # LRU: textbook traces
    assert part.lru_counts([0, 1, 2, 0, 1, 2], 3) == (3, 0, 3)
    assert part.lru_counts([0, 1, 2, 0, 1, 2], 2) == (6, 4, 0)
    assert part.lru_counts([0, 1, 0, 2, 0, 3], 2) == (4, 2, 2)
    assert part.lru_counts([], 1) == (0, 0, 0)
    # capacity >= number of shards: loads = distinct shards touched, no eviction (the paper's
    # scalability table shows 16 loads / 0 evictions with 16 sub-graphs cached)
    ro, ent, hop, pred, _ = run_oracle(w)
    seq = part.shard_accesses(P, w.subj, w.num_entities, w.k, ent, hop)
    loads, ev, hits = part.lru_counts(seq, 8)
    assert loads == len(set(seq)) and ev == 0 and loads + hits == len(seq)
    for cap in (1, 2, 4):
        l2, e2, h2 = part.lru_counts(seq, cap)
        assert l2 - e2 <= cap and l2 >= loads and l2 + h2 == len(seq)


def shard_access_trace(part, pull_hops=()):
    """Hand-worked trace of Alg. 1's routing step over 4 sub-graphs and 3 hops.

    Entities 0..9; subjects (with a triple) are 0,1,2,3,4,5,7; entities 6, 8, 9 are no subject.
    Map P:     e: 0  1  2  3  4  5  6  7  8  9
               P: 2  3  1  1  0  0 -1  3 -1 -1
    Batch result (all queries together): level 0 = {0, 5}, level 1 = {1, 2, 7}, level 2 = {3, 4, 8},
    level 3 = {9}.
      hop 1 expands level 0: sub-graphs {P[0], P[5]} = {2, 0}, odd hop -> ascending:   0, 2
      hop 2 expands level 1: {P[1], P[2], P[7]} = {3, 1},       even hop -> descending: 3, 1
      hop 3 expands level 2: {P[3], P[4]} = {1, 0} (8 is no subject), odd -> ascending: 0, 1
    """
    P = np.array([2, 3, 1, 1, 0, 0, -1, 3, -1, -1], dtype=np.int32)
    subj = np.array([0, 1, 2, 3, 4, 5, 7, 0, 5], dtype=np.int32)
    entity = np.array([0, 5, 1, 2, 7, 3, 4, 8, 9, 0, 2], dtype=np.int32)   # two queries' lists, concatenated
    hop = np.array([0, 0, 1, 1, 1, 2, 2, 2, 3, 0, 1], dtype=np.uint8)
    if pull_hops:   # three sub-graphs by object range, numbered 4, 5, 6 behind the four shards
        return part.shard_accesses(P, subj, 10, 3, entity, hop, pull_hops=pull_hops, num_shards=4, num_ranges=3)
    return part.shard_accesses(P, subj, 10, 3, entity, hop)


def test_shard_visit_order_hand_trace():
    from oracle import partition as part
    seq = shard_access_trace(part)
    assert seq == [0, 2, 3, 1, 0, 1]
    # the cache counters that follow from it with two slots: 0 L, 2 L, 3 L (evicts 0), 1 L (evicts 2),
    # 0 L (evicts 3), 1 hit
    assert part.lru_counts(seq, 2) == (5, 3, 1)
    # with one slot nothing is ever hit; with four slots every sub-graph is loaded once
    assert part.lru_counts(seq, 1) == (6, 5, 0)
    assert part.lru_counts(seq, 4) == (4, 0, 2)
    # hop 2 evaluated by object rows: it touches every sub-graph of the partition by object range
    # (three of them here, numbered 4, 5, 6 behind the four shards), an even hop -> descending
    P4 = np.array([2, 3, 1, 1, 0, 0, -1, 3, -1, -1], dtype=np.int32)
    subj = np.array([0, 1, 2, 3, 4, 5, 7, 0, 5], dtype=np.int32)
    entity = np.array([0, 5, 1, 2, 7, 3, 4, 8, 9, 0, 2], dtype=np.int32)
    hop = np.array([0, 0, 1, 1, 1, 2, 2, 2, 3, 0, 1], dtype=np.uint8)
    seq = part.shard_accesses(P4, subj, 10, 3, entity, hop, pull_hops={2}, num_shards=4, num_ranges=3)
    assert seq == [0, 2, 6, 5, 4, 0, 1]
    # hops 2 and 3 by object rows: 6, 5, 4 then (odd hop) 4, 5, 6: the turning point is a hit
    seq = part.shard_accesses(P4, subj, 10, 3, entity, hop, pull_hops={2, 3}, num_shards=4, num_ranges=3)
    assert seq == [0, 2, 6, 5, 4, 4, 5, 6]
    # two slots: 0 L, 2 L, 6 L (evicts 0), 5 L (evicts 2), 4 L (evicts 6), 4 hit, 5 hit, 6 L (evicts 4)
    assert part.lru_counts(seq, 2) == (6, 4, 2)
    # a fetch of predecessor edges: range 0 and its triple indices, range 1 and its triple indices, ..
    assert part.fetch_accesses(4, 3, 10) == [4, 7, 5, 8, 6, 9]
    assert part.fetch_accesses(4, 3, 9) == []      # a cache that cannot hold all 4 + 3 + 3 units is bypassed
    # fewer hops: a prefix of the same trace; an empty frontier ends it
    P = np.array([0, 1], dtype=np.int32)
    assert part.shard_accesses(P, np.array([0], dtype=np.int32), 2, 3, np.array([0, 1], dtype=np.int32),
                               np.array([0, 1], dtype=np.uint8)) == [0]


def test_query_schedule_groups_queries_by_the_subgraphs_of_their_seeds():
    from oracle import partition as part
    # hand example: P maps entities 0..7 to shards; entity 6 is no subject
    P = np.array([2, 0, 1, 0, 2, 1, -1, 0], dtype=np.int32)
    seed_off = np.array([0, 1, 3, 4, 4, 6, 7, 9, 10], dtype=np.int64)
    seeds = np.array([0,  1, 2,  3,  4, 0,  6,  5, 1,  7], dtype=np.int32)
    # needs: q0 (2) q1 (0,1) q2 (0) q3 () q4 (2) q5 () q6 (0,1) q7 (0)
    assert part.query_needs(P, seed_off, seeds) == [(2,), (0, 1), (0,), (), (2,), (), (0, 1), (0,)]
    # () first, then (0), (0,1), (2); equal needs keep their input order
    assert part.schedule_queries(P, seed_off, seeds).tolist() == [3, 5, 2, 7, 1, 6, 0, 4]
    # properties on a generated workload: a permutation; equal needs contiguous and in input order;
    # with one sub-graph per query and one cache slot, the first hop loads each needed sub-graph once
    w = kggen.config5(0.0005, num_queries=512)
    P, _ = part.degree_aware_partition(w.num_entities, w.subj, 8)
    order = part.schedule_queries(P, w.seed_off, w.seeds)
    assert sorted(order.tolist()) == list(range(w.num_queries))
    needs = part.query_needs(P, w.seed_off, w.seeds)
    seen, last = {}, None
    for q in order:
        nd = needs[q]
        if nd != last:
            assert nd not in seen, "a need appears in two separate runs"
            seen[nd] = True
            last = nd
    for nd in seen:
        run = [int(q) for q in order if needs[q] == nd]
        assert run == sorted(run)
    single = [q for q in range(w.num_queries) if len(needs[q]) == 1]
    so = np.concatenate([[0], np.cumsum([w.seed_off[q + 1] - w.seed_off[q] for q in single])])
    sd = np.concatenate([w.seeds[w.seed_off[q]:w.seed_off[q + 1]] for q in single])
    o1 = part.schedule_queries(P, so, sd)
    first_hop = [needs[single[i]][0] for i in o1]
    loads, _, _ = part.lru_counts(first_hop, 1)
    assert loads == len(set(first_hop))
    unsorted_loads, _, _ = part.lru_counts([needs[q][0] for q in single], 1)
    assert unsorted_loads > loads
