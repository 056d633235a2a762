"""GPU parity: the HIP library (through its C ABI) against the CPU oracle,
element by element, on the same seeded inputs.  All work is integer, so the
bar is bit-exact equality."""
import numpy as np
import pytest

import kggen
import oracle
from helpers import check_invariants

pytestmark = pytest.mark.gpu


def lkg():
    import paper_2604_18913_amd as m
    return m


def run_gpu(w, direction="auto", hub_min_degree=0, k=None, want_traversed=True):
    m = lkg()
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, hub_min_degree=hub_min_degree)
    res = g.khop(w.seed_off, w.seeds, w.k if k is None else k, w.rel_mask, direction=direction)
    off = res.offsets()
    ent, hop, pred = res.fetch()
    trav = res.traversed().cpu().numpy() if want_traversed else None
    out = (off, ent.cpu().numpy(), hop.cpu().numpy(), pred.cpu().numpy(), trav)
    stats = res.hop_stats()
    res.close()
    g.close()
    return out, stats


def run_oracle(w, k=None):
    return oracle.khop(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds,
                       w.k if k is None else k, w.rel_mask)


def assert_same(got, want, what=""):
    names = ["reached_off", "entity", "hop", "pred", "traversed"]
    for n, a, b in zip(names, got, want):
        if a is None:
            continue
        assert a.shape == b.shape, f"{what}: {n} shape {a.shape} vs {b.shape}"
        if not np.array_equal(a, b):
            bad = np.nonzero(a.reshape(-1) != b.reshape(-1))[0]
            raise AssertionError(f"{what}: {n} differs at {bad[:8]} ({bad.size} places): "
                                 f"{a.reshape(-1)[bad[:8]]} vs {b.reshape(-1)[bad[:8]]}")


@pytest.mark.parametrize("direction", ["auto", "push", "pull"])
def test_config1_tiny(direction):
    w = kggen.config1()
    print("case config1", direction, flush=True)
    got, stats = run_gpu(w, direction)
    assert_same(got, run_oracle(w), f"config1/{direction}")
    if direction != "auto":
        assert all(s["direction"] in (0, {"push": 1, "pull": 2}[direction]) for s in stats)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("direction", ["push", "pull"])
def test_random_tiny_masked(seed, direction):
    w = kggen.random_tiny(200 + seed, E=40 + 37 * seed, T=200 + 90 * seed, R=5, Q=7 + 20 * seed, k=4,
                          masked=bool(seed % 2))
    print("case tiny", seed, direction, flush=True)
    got, _ = run_gpu(w, direction, hub_min_degree=33 + seed)
    assert_same(got, run_oracle(w), f"tiny{seed}/{direction}")


@pytest.mark.parametrize("Q", [1, 64, 65, 200, 256, 257, 1000, 1024])
def test_query_counts_and_word_widths(Q):
    w = kggen.config2(0.003, num_queries=Q)
    print("case Q", Q, flush=True)
    for direction in ("push", "pull"):
        got, _ = run_gpu(w, direction, hub_min_degree=64)
        assert_same(got, run_oracle(w), f"Q={Q}/{direction}")


@pytest.mark.parametrize("direction,hub_min", [("auto", 0), ("push", 0), ("pull", 0), ("push", 50), ("pull", 50),
                                               ("auto", 300)])
def test_config2_one_percent(direction, hub_min):
    # 30,000 entities / 300,000 triples / 1,024 queries: several tiles, ragged last tile,
    # all three row classes, W = 16.
    w = kggen.config2(0.01)
    print("case config2/100", direction, hub_min, flush=True)
    got, stats = run_gpu(w, direction, hub_min_degree=hub_min)
    want = run_oracle(w)
    assert_same(got, want, f"config2/100 {direction} hub_min={hub_min}")
    check_invariants(w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k, w.rel_mask, *got[:4],
                     queries=range(0, 1024, 97))
    if direction == "pull":
        # the pull kernels have two forms: one tests an edge's frontier bit before it gathers the
        # line, the other (from 60 % of the triples leaving the frontier) gathers every line; this
        # workload must have gone through both
        share = [s["frontier_edges"] / len(w.subj) for s in stats if s["direction"] == 2]
        assert any(x < 0.6 for x in share) and any(x >= 0.6 for x in share), share


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_config3_relation_masks(k):
    w = kggen.config3(0.01, k=k)
    print("case config3/100 k", k, flush=True)
    want = run_oracle(w)
    for direction in ("auto", "push", "pull"):
        got, _ = run_gpu(w, direction, hub_min_degree=200)
        assert_same(got, want, f"config3/100 k={k} {direction}")


def test_config4_and_5_shapes_resident():
    for w in (kggen.config4(0.002, num_queries=1024), kggen.config5(0.0003)):
        print("case", w.name, flush=True)
        want = run_oracle(w)
        for direction in ("auto", "push", "pull"):
            got, _ = run_gpu(w, direction, hub_min_degree=128)
            assert_same(got, want, f"{w.name} {direction}")


def test_k_zero_and_large_k_and_dead_seeds():
    w = kggen.config1()
    got, _ = run_gpu(w, k=0)
    assert_same(got, run_oracle(w, k=0), "k=0")
    got, stats = run_gpu(w, k=40)
    assert_same(got, run_oracle(w, k=40), "k=40")
    # a query whose only seed has no out-edge reaches just the seed
    outdeg = np.bincount(w.subj, minlength=w.num_entities)
    dead = int(np.nonzero(outdeg == 0)[0][0])
    w.seeds = np.full_like(w.seeds, dead)
    got, _ = run_gpu(w, k=3)
    assert_same(got, run_oracle(w, k=3), "dead seeds")
    assert got[0][-1] == w.num_queries


def test_fetch_subranges_and_optional_outputs():
    m = lkg()
    w = kggen.config2(0.004, num_queries=300)
    want = run_oracle(w)
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, hub_min_degree=100)
    res = g.khop(w.seed_off, w.seeds, w.k)
    off = res.offsets()
    assert np.array_equal(off, want[0])
    for q0, q1 in [(0, 1), (5, 70), (64, 128), (100, 300), (299, 300), (17, 17)]:
        ent, hop, pred = res.fetch(q0, q1)
        a, b = off[q0], off[q1]
        assert np.array_equal(ent.cpu().numpy(), want[1][a:b])
        assert np.array_equal(hop.cpu().numpy(), want[2][a:b])
        assert np.array_equal(pred.cpu().numpy(), want[3][a:b])
    ent, hop, pred = res.fetch(want_hop=False, want_pred=False)
    assert hop is None and pred is None and np.array_equal(ent.cpu().numpy(), want[1])
    res.close()
    g.close()


def test_sixteen_word_planes_deep_hops_overlapped_fetch_and_no_hop_output(monkeypatch):
    # more than 256 queries: k <= 6 takes the staged predecessor kernel that also writes the
    # entity / hop lists, deeper searches take the tile kernel with scattered stores plus the
    # list kernel; both must agree with the oracle, also when a fetch spreads its kernels over the
    # helper streams
    m = lkg()
    w = kggen.config2(0.004, num_queries=300)
    for k in (6, 7, 9):
        want = run_oracle(w, k=k)
        got, _ = run_gpu(w, "auto", hub_min_degree=100, k=k)
        assert_same(got, want, f"k={k}")
    monkeypatch.setenv("LOGOSKG_OVERLAP_FETCH", "1")
    want = run_oracle(w)
    got, _ = run_gpu(w, "auto", hub_min_degree=100)
    assert_same(got, want, "overlapped fetch")
    for k in (2, 7):
        assert_same(run_gpu(w, "auto", hub_min_degree=100, k=k)[0], run_oracle(w, k=k), f"overlapped fetch, k={k}")
    monkeypatch.delenv("LOGOSKG_OVERLAP_FETCH")
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, hub_min_degree=100)
    res = g.khop(w.seed_off, w.seeds, w.k)
    ent, hop, pred = res.fetch(want_hop=False)
    assert hop is None
    assert np.array_equal(ent.cpu().numpy(), want[1]) and np.array_equal(pred.cpu().numpy(), want[3])
    res.close()
    g.close()


@pytest.mark.parametrize("caps", ["0,0", "0,96", "10240,0", "700,3"])
@pytest.mark.parametrize("masked", [False, True])
def test_list_writer_without_room_in_its_tables(caps, masked, monkeypatch):
    # the kernel that writes the lists of a 1,024-query batch keeps the edge ids of short object rows
    # and the predecessor lines of mid-size rows in two LDS tables; with the tables shrunk (or gone)
    # it reads the edge ids from memory and moves the lines in a pass of its own: same lists.
    # Fetched whole, as a sub-range of queries that starts inside a word, and without hop numbers.
    w = kggen.config3(0.006, k=3) if masked else kggen.config2(0.006, num_queries=700)
    want = run_oracle(w)
    monkeypatch.setenv("LOGOSKG_EMIT_CAPS", caps)
    got, _ = run_gpu(w, "auto", hub_min_degree=200)
    assert_same(got, want, f"caps {caps}")
    m = lkg()
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, hub_min_degree=200)
    res = g.khop(w.seed_off, w.seeds, w.k, w.rel_mask)
    q0, q1 = 70, min(w.num_queries, 650)
    a, b = int(want[0][q0]), int(want[0][q1])
    ent, hop, pred = res.fetch(q0, q1, want_hop=False)
    assert hop is None
    assert np.array_equal(ent.cpu().numpy(), want[1][a:b]) and np.array_equal(pred.cpu().numpy(), want[3][a:b])
    res.close()
    g.close()


def test_two_runs_are_bit_identical():
    w = kggen.config3(0.01, k=3)
    a, _ = run_gpu(w, "auto", hub_min_degree=100)
    b, _ = run_gpu(w, "auto", hub_min_degree=100)
    assert_same(a, b, "run-to-run")


@pytest.mark.parametrize("masked", [False, True])
def test_paths_against_oracle(masked):
    m = lkg()
    w = kggen.config3(0.004, k=4, num_queries=200) if masked else kggen.config2(0.004, num_queries=200)
    print("case paths", masked, flush=True)
    want = run_oracle(w)
    pq, pt = kggen.sample_reached_pairs(7, want[0], want[1], 3000)
    # add unreachable targets, seeds and out-of-range pairs
    extra_q = np.array([0, 1, 2, 3], np.int32)
    extra_t = np.array([w.num_entities - 1, int(w.seeds[w.seed_off[1]]), 0, 5], np.int32)
    pq = np.concatenate([pq, extra_q])
    pt = np.concatenate([pt, extra_t])
    cnt_o, edges_o = oracle.paths(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k, pq, pt, 16,
                                  w.rel_mask)
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations)
    res = g.khop(w.seed_off, w.seeds, w.k, w.rel_mask)
    cnt, edges = g.paths(res, pq, pt, 16)
    assert np.array_equal(cnt.cpu().numpy(), cnt_o)
    assert np.array_equal(edges.cpu().numpy(), edges_o)
    cnt3, edges3 = g.paths(res, pq, pt, 3)
    assert np.array_equal(cnt3.cpu().numpy(), np.minimum(cnt_o, 3))
    assert np.array_equal(edges3.cpu().numpy(), edges_o[:, :3])
    res.close()
    g.close()


@pytest.mark.parametrize("Q", [3, 300])
def test_degenerate_graphs_and_the_deepest_search(Q):
    # a 300-entity chain searched to the largest k (hop numbers up to 254), a graph without
    # triples, a single entity with a self loop, and relation ids at the top of the 16-bit range
    m = lkg()
    n = 300
    chain = np.arange(n - 1, dtype=np.int32)
    rel = (np.arange(n - 1, dtype=np.int32) * 7919) % 65536
    seed_off = np.arange(Q + 1, dtype=np.int64)
    seeds = (np.arange(Q, dtype=np.int32) * 5) % n
    for k in (254, 6, 1):
        g = m.Graph(chain, rel, chain + 1, n, 65536)
        res = g.khop(seed_off, seeds, k)
        want = oracle.khop(n, chain, rel, chain + 1, seed_off, seeds, k)
        ent, hop, pred = res.fetch()
        got = (res.offsets(), ent.cpu().numpy(), hop.cpu().numpy(), pred.cpu().numpy(),
               res.traversed().cpu().numpy())
        assert_same(got, want, f"chain k={k}")
        res.close()
        g.close()
    empty = np.zeros(0, dtype=np.int32)
    g = m.Graph(empty, empty, empty, 70, 3)
    res = g.khop(seed_off, seeds % 70, 3)
    want = oracle.khop(70, empty, empty, empty, seed_off, seeds % 70, 3)
    ent, hop, pred = res.fetch()
    assert_same((res.offsets(), ent.cpu().numpy(), hop.cpu().numpy(), pred.cpu().numpy(), None), want, "no triples")
    res.close()
    g.close()
    one = np.zeros(1, dtype=np.int32)
    g = m.Graph(one, one, one, 1, 1)
    res = g.khop(seed_off, np.zeros(Q, dtype=np.int32), 4)
    want = oracle.khop(1, one, one, one, seed_off, np.zeros(Q, dtype=np.int32), 4)
    ent, hop, pred = res.fetch()
    assert_same((res.offsets(), ent.cpu().numpy(), hop.cpu().numpy(), pred.cpu().numpy(),
                 res.traversed().cpu().numpy()), want, "self loop")
    res.close()
    g.close()


def test_device_build_equals_host_build():
    # the GPU sort and the host counting sort must give the same CSR: predecessor edges and path
    # listings depend on the order of the entries inside a row
    m = lkg()
    cases = [kggen.config1(), kggen.config2(0.01), kggen.config3(0.005, k=3),
             kggen.random_tiny(900, E=50, T=400, R=3, Q=70, k=4, masked=True)]
    for w in cases:
        outs = []
        for host_build in (False, True):
            g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, host_build=host_build)
            res = g.khop(w.seed_off, w.seeds, w.k, w.rel_mask)
            ent, hop, pred = res.fetch()
            info = {k: v for k, v in g.info().items() if k.startswith("num_")}
            outs.append((res.offsets(), ent.cpu().numpy(), hop.cpu().numpy(), pred.cpu().numpy(),
                         res.traversed().cpu().numpy(), info))
            res.close()
            g.close()
        assert outs[0][5] == outs[1][5], w.name
        assert_same(outs[0][:5], outs[1][:5], w.name)
        assert_same(outs[0][:5], run_oracle(w), w.name)


def test_bad_inputs_are_reported_not_faulted():
    m = lkg()
    w = kggen.config1()
    with pytest.raises(m.LogosKGError):
        bad = w.subj.copy()
        bad[3] = w.num_entities
        m.Graph(bad, w.rel, w.obj, w.num_entities, w.num_relations)
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations)
    seeds = w.seeds.copy()
    seeds[5] = w.num_entities + 3
    with pytest.raises(m.LogosKGError):
        g.khop(w.seed_off, seeds, 2)
    off = w.seed_off.copy()
    off[7] = off[6] - 1
    with pytest.raises(m.LogosKGError):
        g.khop(off, w.seeds, 2)
    with pytest.raises(m.LogosKGError):
        g.khop(w.seed_off, w.seeds, 255)
    res = g.khop(w.seed_off, w.seeds, 2)  # the handle still works afterwards
    assert res.offsets()[-1] == run_oracle(w)[0][-1]
    with pytest.raises(m.LogosKGError):
        import torch
        small = torch.empty(3, dtype=torch.int32, device=g.device)
        res.fetch(out=(small, None, None))
    res.close()
    g.close()


def test_the_callers_allocator_serves_the_memory_of_the_calls():
    # logoskg_build_opts.dev_alloc / dev_free: planes, tables and workspaces of the calls come from
    # the caller (here torch's caching allocator); same results, every block given back
    import torch
    m = lkg()
    w = kggen.config3(0.004, k=3)
    want = oracle.khop(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k, w.rel_mask)
    held, calls = {}, {"alloc": 0, "free": 0, "bytes": 0}

    def dev_alloc(nbytes):
        t = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
        held[t.data_ptr()] = t
        calls["alloc"] += 1
        calls["bytes"] += nbytes
        return t.data_ptr()

    def dev_free(ptr):
        del held[ptr]
        calls["free"] += 1

    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, dev_alloc=dev_alloc, dev_free=dev_free)
    for _ in range(2):
        res = g.khop(w.seed_off, w.seeds, w.k, w.rel_mask)
        ent, hop, pred = res.fetch()
        assert np.array_equal(res.offsets(), want[0]) and np.array_equal(ent.cpu().numpy(), want[1])
        assert np.array_equal(hop.cpu().numpy(), want[2]) and np.array_equal(pred.cpu().numpy(), want[3])
        pq, pt = kggen.sample_reached_pairs(3, want[0], want[1], 200)
        cnt, edges = g.paths(res, pq, pt, 16)
        cnt_o, edges_o = oracle.paths(w.num_entities, w.subj, w.rel, w.obj, w.seed_off, w.seeds, w.k, pq, pt, 16,
                                      w.rel_mask)
        assert np.array_equal(cnt.cpu().numpy(), cnt_o) and np.array_equal(edges.cpu().numpy(), edges_o)
        res.close()
    plane_bytes = (w.num_entities + 63) // 64 * 64 * 16 * 8 * (w.k + 2)
    assert calls["alloc"] >= 3 and calls["bytes"] >= plane_bytes      # the planes alone are that large
    first_round = calls["alloc"]
    res = g.khop(w.seed_off, w.seeds, w.k, w.rel_mask)                # a third call reuses the pool's blocks
    res.close()
    assert calls["alloc"] == first_round
    g.close()
    assert calls["free"] == calls["alloc"] and not held
    with pytest.raises(m.LogosKGError):                               # one callback without the other
        m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, dev_alloc=dev_alloc)
    fail = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, dev_alloc=lambda n: 0,
                   dev_free=lambda p: None)
    with pytest.raises(m.LogosKGError):                               # an allocator that has nothing left
        fail.khop(w.seed_off, w.seeds, w.k, w.rel_mask)
    fail.close()


@pytest.mark.parametrize("masked", [False, True])
def test_fetch_inside_one_word_of_sixteen_word_planes(masked, monkeypatch):
    # A fetch whose queries sit in one 64-query word takes row kernels of its own (an entry per
    # lane, a bit transpose per 64 entries): ranges at word starts, inside a word and at the ragged
    # end, hub rows (block per row and level) and mid rows (wavefront per row), with and without
    # the row buffer, against the oracle's slices.
    m = lkg()
    Q = 700
    w = kggen.config3(0.006, k=3, num_queries=Q) if masked else kggen.config2(0.006, num_queries=Q)
    want = run_oracle(w)
    for hub_min, caps in ((60, None), (0, None), (60, "64,2")):
        if caps:
            monkeypatch.setenv("LOGOSKG_EMIT_CAPS", caps)
        g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, hub_min_degree=hub_min)
        res = g.khop(w.seed_off, w.seeds, w.k, w.rel_mask)
        for q0, q1 in ((0, 64), (64, 128), (70, 100), (127, 128), (640, 700), (699, 700), (5, 6)):
            ent, hop, pred = res.fetch(q0, q1)
            a, b = want[0][q0], want[0][q1]
            what = f"masked={masked} hub_min={hub_min} caps={caps} queries {q0}..{q1}"
            assert np.array_equal(ent.cpu().numpy(), want[1][a:b]), what
            assert np.array_equal(hop.cpu().numpy(), want[2][a:b]), what
            assert np.array_equal(pred.cpu().numpy(), want[3][a:b]), what
        ent, hop, pred = res.fetch(60, 130)  # three words: the line-wide kernels
        a, b = want[0][60], want[0][130]
        assert np.array_equal(pred.cpu().numpy(), want[3][a:b])
        res.close()
        if not caps:  # more than six hops: the row kernels write into the lists themselves
            want7 = run_oracle(w, k=7)
            res = g.khop(w.seed_off, w.seeds, 7, w.rel_mask)
            for q0, q1 in ((64, 128), (650, 700), (3, 4)):
                ent, hop, pred = res.fetch(q0, q1)
                a, b = want7[0][q0], want7[0][q1]
                assert np.array_equal(ent.cpu().numpy(), want7[1][a:b]), (masked, hub_min, q0, q1)
                assert np.array_equal(hop.cpu().numpy(), want7[2][a:b]), (masked, hub_min, q0, q1)
                assert np.array_equal(pred.cpu().numpy(), want7[3][a:b]), (masked, hub_min, q0, q1)
            res.close()
        g.close()
        if caps:
            monkeypatch.delenv("LOGOSKG_EMIT_CAPS")


def test_gather_probe_ors_the_lines_of_all_subjects():
    # the measurement aid reads the line of every entry's subject: its result is the OR over the subjects
    import torch
    m = lkg()
    w = kggen.config2(0.004, num_queries=64)
    g = m.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations)
    rng = np.random.default_rng(5)
    lines = rng.integers(0, 2 ** 62, size=(w.num_entities, 16), dtype=np.int64) & rng.integers(0, 2 ** 62, size=(w.num_entities, 16), dtype=np.int64)
    out = g.probe_gather(torch.from_numpy(lines).cuda())
    want = np.bitwise_or.reduce(lines[np.unique(w.subj)], axis=0)
    assert np.array_equal(out.cpu().numpy(), want)
    g.close()
