"""Seeded synthetic knowledge-graph and query generators.

This module only *draws inputs*: triple lists (subject, relation, object), seed
sets and relation whitelists.  It contains none of the retrieval method's
arithmetic (no traversal, no CSR, no bit planes), so the CPU oracle and the HIP
library can both be fed from it without sharing any logic.

The five workload recipes follow the problem statement of the paper (Sec. 3.1:
a KG is a set of triples over entities and relation types; a query is a set of
entities) and stand in for the biomedical graphs the paper measures on
(UMLS-class and PubMed-KG-class graphs, Sec. 5 "Dataset and Setup"), which are
not redistributable.  Every draw comes from ``numpy.random.Generator(PCG64)``
seeded with ``BASE_SEED + config index``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 2604189130

# Optional callable(str): told when a step of a generator ends (the large workloads take
# minutes to draw; a caller that must show it is alive sets this).
progress = None


def _step(what: str) -> None:
    if progress is not None:
        progress(what)


@dataclass
class Workload:
    """One synthetic KG plus one query batch."""

    name: str
    num_entities: int
    num_relations: int
    subj: np.ndarray  # int32[T]
    rel: np.ndarray  # int32[T]
    obj: np.ndarray  # int32[T]
    seed_off: np.ndarray  # int64[Q+1]
    seeds: np.ndarray  # int32[seed_off[-1]]
    k: int
    rel_mask: Optional[np.ndarray] = None  # uint64[Q, ceil(R/64)] or None (= all allowed)
    manifest: dict = field(default_factory=dict)

    @property
    def num_triples(self) -> int:
        return int(self.subj.shape[0])

    @property
    def num_queries(self) -> int:
        return int(self.seed_off.shape[0] - 1)


# --------------------------------------------------------------------------
# degree sequences
# --------------------------------------------------------------------------

def _powerlaw_cdf(alpha: float, dmin: int, cap: int) -> np.ndarray:
    d = np.arange(dmin, cap + 1, dtype=np.float64)
    pmf = d ** (-alpha)
    pmf /= pmf.sum()
    return np.cumsum(pmf)


def powerlaw_mean(alpha: float, dmin: int, cap: int) -> float:
    d = np.arange(dmin, cap + 1, dtype=np.float64)
    w = d ** (-alpha)
    return float((d * w).sum() / w.sum())


def draw_degrees(rng: np.random.Generator, n: int, total: int, alpha: float,
                 dmin: int, cap: int) -> np.ndarray:
    """Draw up to ``n`` iid degrees from the truncated discrete power law
    P(d) ~ d^-alpha on [dmin, cap] and stop where the running sum reaches
    ``total`` (the last draw is truncated); the rest are 0.  Returns int64[n]
    whose sum is min(total, sum of all n draws)."""
    cdf = _powerlaw_cdf(alpha, dmin, cap)
    u = rng.random(n)
    deg = (np.searchsorted(cdf, u, side="left") + dmin).astype(np.int64)
    np.minimum(deg, cap, out=deg)
    csum = np.cumsum(deg)
    cut = int(np.searchsorted(csum, total, side="left"))
    if cut < n:
        prev = int(csum[cut - 1]) if cut > 0 else 0
        deg[cut] = total - prev
        deg[cut + 1:] = 0
    return deg


def choose_dmin(alpha: float, cap: int, n: int, total: int) -> int:
    """Smallest dmin for which mean(dmin) * n >= total."""
    dmin = 1
    while powerlaw_mean(alpha, dmin, cap) * n < total and dmin < cap:
        dmin += 1
    return dmin


# --------------------------------------------------------------------------
# triple assembly
# --------------------------------------------------------------------------

def _pack_keys(s, r, o, E, R):
    """(s, r, o) -> one uint64 key per triple; needs E*E*R < 2^64."""
    assert float(E) * float(E) * float(R) < 2.0 ** 64 * 0.999, "key does not fit 64 bits"
    E64, R64 = np.uint64(E), np.uint64(R)
    return (s.astype(np.uint64) * R64 + r.astype(np.uint64)) * E64 + o.astype(np.uint64)


def _unpack_keys(key, E, R):
    E64, R64 = np.uint64(E), np.uint64(R)
    o = key % E64
    key = key // E64
    return (key // R64).astype(np.int64), (key % R64).astype(np.int64), o.astype(np.int64)


def _assemble(rng, T, E, R, s_stubs, o_stubs, draw_rel):
    """Pair subject stubs with shuffled object stubs, draw a relation per pair
    and drop exact duplicate (s, r, o) triples.  Duplicates (frequent between
    two hubs) are topped up by re-drawing pairs from the same stub lists, so
    the degree shape is kept, until T distinct triples exist or five rounds
    have passed.  The triples are finally shuffled so that edge ids carry no
    locality.  Ids are whatever the stub lists hold (callers may pass dense
    ranks and map them back)."""
    n = int(min(s_stubs.shape[0], o_stubs.shape[0], T))
    keys = _pack_keys(s_stubs[:n], draw_rel(n), o_stubs[rng.permutation(o_stubs.shape[0])[:n]], E, R)
    _step(f"generator: {n:,} stub pairs drawn")
    keys = np.unique(keys)
    _step(f"generator: {keys.shape[0]:,} distinct triples")
    for _ in range(5):
        missing = T - keys.shape[0]
        if missing <= 0:
            break
        m = int(missing * 1.25) + 16
        new = np.unique(_pack_keys(s_stubs[rng.integers(0, s_stubs.shape[0], size=m)], draw_rel(m),
                                   o_stubs[rng.integers(0, o_stubs.shape[0], size=m)], E, R))
        merged = np.sort(np.concatenate([keys, new]), kind="stable")  # two sorted runs: a linear merge
        keep = np.ones(merged.shape[0], dtype=bool)
        keep[1:] = merged[1:] != merged[:-1]
        keys = merged[keep]
        del merged, keep, new
        _step(f"generator: topped up to {keys.shape[0]:,} distinct triples")
    perm = rng.permutation(keys.shape[0])[:T]
    s, r, o = _unpack_keys(keys[perm], E, R)
    _step("generator: triples shuffled")
    return s, r, o


def _zipf_rank_relations(rng, n, R, alpha):
    w = (np.arange(R, dtype=np.float64) + 1.0) ** (-alpha)
    cdf = np.cumsum(w / w.sum())
    return np.minimum(np.searchsorted(cdf, rng.random(n), side="left"), R - 1)


def _pack_queries(seed_lists):
    lens = np.array([len(x) for x in seed_lists], dtype=np.int64)
    off = np.zeros(len(seed_lists) + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    seeds = (np.concatenate(seed_lists).astype(np.int32)
             if len(seed_lists) and off[-1] > 0 else np.zeros(0, np.int32))
    return off, seeds


def random_seed_sets(rng, Q, E, lo, hi):
    """Q queries; each has a seed count uniform in [lo, hi] and seeds uniform
    over all E entities (repeats inside a query are allowed and collapse)."""
    counts = rng.integers(lo, hi + 1, size=Q)
    flat = rng.integers(0, E, size=int(counts.sum()), dtype=np.int64)
    off = np.zeros(Q + 1, dtype=np.int64)
    np.cumsum(counts, out=off[1:])
    return off, flat.astype(np.int32)


def random_whitelists(rng, Q, R, lo, hi):
    """Per query a whitelist of a uniform number in [lo, hi] of distinct
    relation ids; packed as uint64[Q, ceil(R/64)], bit r%64 of word r//64."""
    rw = (R + 63) // 64
    mask = np.zeros((Q, rw), dtype=np.uint64)
    for q in range(Q):
        n = int(rng.integers(lo, min(hi, R) + 1))
        ids = rng.choice(R, size=n, replace=False)
        for r in ids:
            mask[q, r // 64] |= np.uint64(1) << np.uint64(r % 64)
    return mask


def _correlated_powerlaw_graph(rng, E, T, R, alpha, cap, rel_alpha):
    """Out- and in-degree sequences from the same truncated power law, rank
    matched on one random entity permutation (the entity with the largest
    out-degree also has the largest in-degree), subject and object stubs
    paired at random."""
    cap = max(1, min(cap, E - 1))
    dmin = choose_dmin(alpha, cap, E, T)
    perm = rng.permutation(E)
    dout = np.sort(draw_degrees(rng, E, T, alpha, dmin, cap))[::-1]
    din = np.sort(draw_degrees(rng, E, T, alpha, dmin, cap))[::-1]
    _step("generator: degree sequences drawn")
    if rel_alpha is None:
        draw_rel = lambda n: rng.integers(0, R, size=n)
    else:
        draw_rel = lambda n: _zipf_rank_relations(rng, n, R, rel_alpha)
    # work on ranks (positions in `perm`): only the first `used` ranks carry edges, which keeps
    # the 63-bit triple keys of the duplicate check small enough even for 10^8 entities
    used = int(max((dout > 0).sum(), (din > 0).sum()))
    ranks = np.arange(used, dtype=np.int64)
    s, r, o = _assemble(rng, T, used, R, np.repeat(ranks, dout[:used]), np.repeat(ranks, din[:used]),
                        draw_rel)
    return (perm[s].astype(np.int32), r.astype(np.int32), perm[o].astype(np.int32),
            dict(dmin=dmin, cap=cap, alpha=alpha))


def _finish_manifest(w: Workload, extra: dict) -> Workload:
    outdeg = np.bincount(w.subj, minlength=w.num_entities)
    indeg = np.bincount(w.obj, minlength=w.num_entities)
    live = outdeg[w.seeds] > 0 if w.seeds.size else np.zeros(0, bool)
    w.manifest = dict(
        name=w.name, num_entities=w.num_entities, num_relations=w.num_relations,
        num_triples=w.num_triples, num_queries=w.num_queries, k=w.k,
        max_out_degree=int(outdeg.max()) if outdeg.size else 0,
        max_in_degree=int(indeg.max()) if indeg.size else 0,
        num_subjects=int((outdeg > 0).sum()), num_objects=int((indeg > 0).sum()),
        live_seed_fraction=float(live.mean()) if live.size else 0.0,
        masked=w.rel_mask is not None, **extra)
    _step(f"generator: {w.name} done")
    return w


# --------------------------------------------------------------------------
# the five workloads
# --------------------------------------------------------------------------

def config1(scale: float = 1.0) -> Workload:
    """Tiny KG: 10,000 entities, 50,000 triples, 20 relation types, subject
    out-degrees from P(d) ~ d^-2, objects and relations uniform; 64 queries of
    one uniform seed; k = 2."""
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 1))
    E = max(16, int(10_000 * scale))
    T = max(32, int(50_000 * scale))
    R = 20
    cap = E - 1
    dmin = choose_dmin(2.0, cap, E, T)
    perm = rng.permutation(E)
    dout = draw_degrees(rng, E, T, 2.0, dmin, cap)
    s, r, o = _assemble(rng, T, E, R, np.repeat(perm, dout),
                        np.arange(E, dtype=np.int64).repeat(-(-T // E)),
                        lambda n: rng.integers(0, R, size=n))
    s, r, o = s.astype(np.int32), r.astype(np.int32), o.astype(np.int32)
    off, seeds = random_seed_sets(rng, 64, E, 1, 1)
    w = Workload("config1_tiny", E, R, s, r, o, off, seeds, k=2)
    return _finish_manifest(w, dict(dmin=dmin, cap=cap, alpha=2.0, scale=scale))


def config2(scale: float = 1.0, num_queries: int = 1024) -> Workload:
    """Biomedical-concept-shaped KG: 3,000,000 entities, 30,000,000 triples,
    500 relation types with rank-frequency p(r) ~ (r+1)^-1.1; out- and
    in-degrees from P(d) ~ d^-1.8 capped at 200,000, rank matched; 1,024
    queries of 1-5 uniform seeds; k = 3; all relations allowed."""
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 2))
    E = max(64, int(3_000_000 * scale))
    T = max(128, int(30_000_000 * scale))
    R = 500
    cap = max(8, int(200_000 * min(1.0, scale * 4)))
    s, r, o, info = _correlated_powerlaw_graph(rng, E, T, R, 1.8, cap, 1.1)
    off, seeds = random_seed_sets(rng, num_queries, E, 1, 5)
    w = Workload("config2_biomed", E, R, s, r, o, off, seeds, k=3)
    return _finish_manifest(w, dict(scale=scale, **info))


def config3(scale: float = 1.0, k: int = 3, num_queries: int = 1024) -> Workload:
    """config2's graph and queries with a per-query relation whitelist of
    10-50 of the 500 relation types; k is swept over 1..4 by the caller."""
    w = config2(scale, num_queries)
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 3))
    w.rel_mask = random_whitelists(rng, w.num_queries, w.num_relations, 10, 50)
    w.k = k
    w.name = "config3_relmask"
    w.manifest.update(name=w.name, k=k, masked=True)
    return w


def sample_reached_pairs(seed: int, reached_off: np.ndarray, entity: np.ndarray,
                         n: int):
    """Seeded sample of (query, reached entity) pairs out of a query-major
    result list, used to pick path-reconstruction targets."""
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 1000 + seed))
    total = int(reached_off[-1])
    if total == 0:
        return np.zeros(0, np.int32), np.zeros(0, np.int32)
    idx = np.sort(rng.integers(0, total, size=min(n, total)))
    q = (np.searchsorted(reached_off, idx, side="right") - 1).astype(np.int32)
    return q, entity[idx].astype(np.int32)


def config4(scale: float = 1.0, num_queries: int = 4096) -> Workload:
    """Hub-heavy KG: 20,000,000 entities, 300,000,000 triples, 1,000 uniform
    relation types; 0.01 % of entities are hubs that are the subject of 40 % of
    all triples and the object of 40 % of all triples; the rest have
    P(d) ~ d^-2.2 out-degrees and uniform in-stubs; 4,096 one-seed queries,
    even-indexed ones seeded at hubs; k = 3."""
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 4))
    E = max(1000, int(20_000_000 * scale))
    T = max(4000, int(300_000_000 * scale))
    R = 1000
    n_hub = max(2, int(round(E * 1e-4)))
    hub_edges = int(T * 0.4)
    perm = rng.permutation(E)
    hubs, rest = perm[:n_hub], perm[n_hub:]
    hub_deg = np.full(n_hub, hub_edges // n_hub, dtype=np.int64)
    hub_deg[: hub_edges - int(hub_deg.sum())] += 1
    cap = max(8, min(200_000, rest.shape[0] - 1))
    rest_total = T - hub_edges
    dmin = choose_dmin(2.2, cap, rest.shape[0], rest_total)
    rest_deg = draw_degrees(rng, rest.shape[0], rest_total, 2.2, dmin, cap)
    s_stubs = np.concatenate([np.repeat(hubs, hub_deg), np.repeat(rest, rest_deg)])
    n_edges = s_stubs.shape[0]
    n_obj_hub = int(n_edges * 0.4)
    o_stubs = np.concatenate([
        hubs[rng.integers(0, n_hub, size=n_obj_hub)],
        rest[rng.integers(0, rest.shape[0], size=n_edges - n_obj_hub)]])
    s, r, o = _assemble(rng, T, E, R, s_stubs, o_stubs,
                        lambda n: rng.integers(0, R, size=n))
    s, r, o = s.astype(np.int32), r.astype(np.int32), o.astype(np.int32)
    Q = num_queries
    seeds = np.empty(Q, dtype=np.int32)
    seeds[0::2] = hubs[rng.integers(0, n_hub, size=seeds[0::2].shape[0])]
    seeds[1::2] = rest[rng.integers(0, rest.shape[0], size=seeds[1::2].shape[0])]
    off = np.arange(Q + 1, dtype=np.int64)
    w = Workload("config4_hubheavy", E, R, s, r, o, off, seeds, k=3)
    return _finish_manifest(w, dict(scale=scale, n_hub=n_hub, dmin=dmin, cap=cap,
                                    alpha=2.2))


def config5(scale: float = 1.0, num_queries: int = 1024) -> Workload:
    """Billion-edge KG: 100,000,000 entities, 1,000,000,000 triples, 2,000
    uniform relation types, out- and in-degrees P(d) ~ d^-1.9 capped at
    200,000, rank matched; 1,024 queries of 1-3 uniform seeds; k = 3.  The
    library is asked for 8 shards and a bounded shard cache."""
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 5))
    E = max(64, int(100_000_000 * scale))
    T = max(128, int(1_000_000_000 * scale))
    R = 2000
    cap = max(8, int(200_000 * min(1.0, scale * 100)))
    s, r, o, info = _correlated_powerlaw_graph(rng, E, T, R, 1.9, cap, None)
    off, seeds = random_seed_sets(rng, num_queries, E, 1, 3)
    w = Workload("config5_billion", E, R, s, r, o, off, seeds, k=3)
    return _finish_manifest(w, dict(scale=scale, num_shards=8, **info))


def random_tiny(seed: int, E: int, T: int, R: int, Q: int, k: int,
                masked: bool = False, max_seeds: int = 3) -> Workload:
    """Small uniformly random KG (may contain self loops and parallel edges in
    different relations) for the brute-force checks."""
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 100 + seed))
    s = rng.integers(0, E, size=T)
    o = rng.integers(0, E, size=T)
    r = rng.integers(0, R, size=T)
    s, r, o = _unpack_keys(np.unique(_pack_keys(s, r, o, E, R)), E, R)
    perm = rng.permutation(s.shape[0])
    s, r, o = (s[perm].astype(np.int32), r[perm].astype(np.int32),
               o[perm].astype(np.int32))
    off, seeds = random_seed_sets(rng, Q, E, 1, max_seeds)
    w = Workload(f"tiny_{seed}", E, R, s, r, o, off, seeds, k=k)
    if masked:
        rw = (R + 63) // 64
        m = np.zeros((Q, rw), dtype=np.uint64)
        allow = rng.random((Q, R)) < 0.6
        for q in range(Q):
            for rr in np.nonzero(allow[q])[0]:
                m[q, rr // 64] |= np.uint64(1) << np.uint64(rr % 64)
        w.rel_mask = m
    return _finish_manifest(w, {})


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}
