#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

One step = one pass of logoskg_khop (seed scatter, 3 hops of push/pull
expansion with the visited/level update, per-query counts) followed by
logoskg_result_fetch of every query (query-major entity / hop / predecessor
lists) on the 3,000,000-entity / 30,000,000-triple synthetic KG with 1,024
queries (the second of the five benchmark configurations).  Seeds and the graph
are resident in HBM before the timed region; outputs stay in HBM.

Prints one JSON line: throughput of the whole step, per-kernel times from HIP
events around every launch, the roofline figure of the kernel with the largest
time per step, the expansion kernels taken alone, and the CPU oracle timed on a
sample of the same queries.
"""
from __future__ import annotations

import argparse
import functools
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(kernel: str, p: dict, W: int, k: int, masked: bool, plane_bytes: float,
                      lists_fused: bool = False, level_lists: bool = False) -> float:
    """Bytes the named kernel has to move per step for the work units it reported
    (rows / edges / lines / items); the per-unit figures are stated case by case below."""
    line = 8 * W
    e_bytes = 4 + (2 if masked else 0)
    rows, edges, lines, items = p["rows"], p["edges"], p["lines"], p["items"]
    n = p.get("launches_per_step", 1)
    if kernel.startswith("pull_") and kernel != "pull_finish":
        # per scanned row (or row segment): visited line read + new-level line written + two 4-byte
        # offsets (the visited write-back is not counted); per edge: subject id (+ relation);
        # per DISTINCT frontier line gathered: one line (caches are assumed to absorb repeats)
        return rows * (2 * line + 8) + edges * e_bytes + items * line
    if kernel.startswith("push_"):
        return 0.0  # frontier of hop 1 only: a few hundred KB, not priced
    if kernel == "frontier_census":
        return n * plane_bytes / (64.0 * W)  # the 1-bit-per-entity active bitmap
    if kernel == "lists":
        # visited + levels 1..k streamed once; 4 B entity + 1 B hop written per list entry
        # (the list of one level: that level's plane, 4 B per entry)
        if level_lists:
            return n * plane_bytes + items * 4
        return n * (k + 1) * plane_bytes + items * 5
    if kernel == "pred":
        # list writer of the two-kernel predecessor pass (16-word planes): per (entity, word) of the
        # tiles it covers 64 code bytes + one visited word read (rows = entities x words), per list
        # entry 4 B entity + 1 B hop + 4 B predecessor written
        if lists_fused:
            return rows * 72 + items * 9
        # tile kernel with scattered stores (1 and 4 words, or k > 6): visited + level 0 streamed,
        # 4 B written per list entry, 4 B per object-row entry walked
        return n * 2 * plane_bytes + items * 4 + edges * 4
    if kernel == "pred_walk":
        # first kernel of that pass: per (entity, word) (items) the visited word and the k + 1 level
        # words read, 72 B written; 4 B per object-row entry read; one line per candidate line gathered,
        # but not more than the graph has lines (caches are assumed to absorb repeats)
        return items * 8 * (k + 2) + items * 72 + edges * 4 + min(lines * line, plane_bytes)
    if kernel in ("pred_rows", "pred_mid_rows"):
        return edges * 4
    if kernel == "clear_planes":
        return items * 8
    if kernel == "active_triples":
        # per list entry (one row of SUB): entity id, output position, two row offsets; per triple:
        # triple index + object + relation read (10 B), four int32 columns written
        return rows * 20 + items * 26
    if kernel == "count_tiles":
        return items * 8 * 1.25  # plane read + uint16 per (tile, query) written
    return 0.0


def kernel_sources_sha256(root: str) -> str:
    """Hash of the HIP sources and headers the library is built from."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(root, "paper_2604_18913_amd", "csrc")
    names = sorted(f for f in os.listdir(csrc) if f.endswith((".hip", ".h")))
    for path in [os.path.join(csrc, f) for f in names] + [os.path.join(root, "include", "logoskg.h")]:
        h.update(open(path, "rb").read())
    return h.hexdigest()


def cpu_model() -> str:
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.startswith("model name"):
                return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def note(*a):
    """Progress lines go to stderr: stdout carries the one JSON line."""
    print(time.strftime("%H:%M:%S"), *a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (testing only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-queries", type=int, default=0, help="0 = 512 for configs 1-3, 6 for configs 4 and 5")
    ap.add_argument("--serial-fetch", action="store_true",
                    help="no effect any more (the kernels of a fetch always run in turn unless --overlap-fetch "
                         "is given); kept so that older command lines still run")
    ap.add_argument("--overlap-fetch", action="store_true",
                    help="put the independent kernels of a fetch on helper streams (LOGOSKG_OVERLAP_FETCH=1) in the "
                         "timed region; the per-kernel figures still come from a region without it")
    ap.add_argument("--config", type=int, choices=[1, 2, 3, 4, 5], default=2,
                    help="workload: 2 (default) is the one the metric is quoted on; the others are the "
                         "parity-test shapes, timed the same way "
                         "(4: the first of its four 1,024-query batches; 5: 8 shards, 64 GB shard budget)")
    ap.add_argument("--k", type=int, default=0, help="hops (config 3 sweeps 1..4; 0 = the workload's own)")
    ap.add_argument("--fetch-queries", type=int, default=0,
                    help="fetch the lists of the first N queries only (0 = all; configs 4 and 5 default to 64)")
    ap.add_argument("--resident-shards", type=int, default=0,
                    help="config 5: capacity of the shard cache in shards (the paper's n); 0 = the byte budget only")
    ap.add_argument("--shard-dir", default="",
                    help="config 5: keep the shards in files under this directory (created if missing) "
                         "instead of pinned host memory")
    ap.add_argument("--mode", choices=["minhop", "walk", "triples"], default="minhop",
                    help="minhop (default): the headline path; walk: Eq. 4 iterated without the visited set "
                         "(LOGOSKG_WALK_EXACT), one step = khop + the list of level k of every query; "
                         "triples: one step = khop + the active triples T_k (Eq. 5-7, four columns) of the "
                         "first --fetch-queries queries (default 16)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also launch a plain 1 GiB device copy and a 1 GiB fill, so that rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings can be scaled by a kernel of known size")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding across GPUs, no collectives); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import kggen
    kggen.progress = note  # the large configurations take minutes to generate: say what is going on
    import paper_2604_18913_amd as lkg

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    t0 = time.time()
    cfg = args.config
    graph_opts = {}
    if cfg == 1:
        w = kggen.config1(args.scale)
    elif cfg == 2:
        w = kggen.config2(args.scale)
    elif cfg == 3:
        w = kggen.config3(args.scale, k=args.k or 3)
    elif cfg == 4:
        w = kggen.config4(args.scale)
        w.seed_off = w.seed_off[: min(w.num_queries, 1024) + 1]     # the first of the four batches
        w.seeds = w.seeds[: w.seed_off[-1]]
    else:
        w = kggen.config5(args.scale)
        graph_opts = dict(num_shards=8, hbm_shard_budget_bytes=64 << 30, max_resident_shards=args.resident_shards)
        if args.shard_dir:
            os.makedirs(args.shard_dir, exist_ok=True)
            graph_opts["shard_dir"] = args.shard_dir
    if args.k:
        w.k = args.k
    t_gen = time.time() - t0
    note(f"generated config {cfg} in {t_gen:.0f} s: {w.num_entities:,} entities, {w.num_triples:,} triples")
    t0 = time.time()
    g = lkg.Graph(w.subj, w.rel, w.obj, w.num_entities, w.num_relations, **graph_opts)
    t_build = time.time() - t0
    note(f"built in {t_build:.0f} s")
    dev = g.device
    seed_off = torch.from_numpy(w.seed_off).to(dev)
    seeds = torch.from_numpy(w.seeds).to(dev)
    rel_mask = None if w.rel_mask is None else torch.from_numpy(w.rel_mask.view(np.int64)).to(dev)
    masked = rel_mask is not None
    Q, k = w.num_queries, w.k
    triples = args.mode == "triples"
    nf = args.fetch_queries or (16 if triples else 64 if cfg >= 4 else Q)   # queries whose lists are fetched
    nf = min(nf, Q)

    # practical HBM ceiling of this machine in this run: a plain 1 GiB device copy (reads 1 GiB, writes 1 GiB)
    src = torch.ones(1 << 27, dtype=torch.int64, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    stream_copy_gbps = 10 * 2 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst
    note(f"1 GiB device copy: {stream_copy_gbps:.0f} GB/s (read + write)")

    if args.pmc_calibration:
        src = torch.ones(1 << 27, dtype=torch.int64, device=dev)   # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)        # reads 1 GiB, writes 1 GiB
            dst.fill_(7)          # writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # sizes are deterministic: one untimed call sizes the output buffers
    walk = args.mode == "walk"
    res = g.khop(seed_off, seeds, k, rel_mask, walk_exact=walk)
    off = res.offsets()
    total = int(res.level(k, 0, 0)[0][nf]) if walk else int(off[nf])
    W = res.words_per_entity
    res_epad = res.padded_entities
    n_triples = 0
    if triples:
        first = res.active_triples(k, 0, nf)
        n_triples = int(first[0][-1])
        cols = tuple(first[1:])
        del first
    elif not walk:
        ent = torch.empty(total, dtype=torch.int32, device=dev)
        hop = torch.empty(total, dtype=torch.uint8, device=dev)
        pred = torch.empty(total, dtype=torch.int32, device=dev)
    trav = res.traversed().cpu().numpy()
    hop_stats = res.hop_stats()
    res.close()
    logical_edges = int(trav.sum())

    def step():
        if walk:
            r = g.khop(seed_off, seeds, k, rel_mask, walk_exact=True)
            r.level(k, 0, nf)
        elif triples:
            r = g.khop(seed_off, seeds, k, rel_mask)
            r.active_triples(k, 0, nf, out=cols)
        else:
            r = g.khop(seed_off, seeds, k, rel_mask)
            r.fetch(0, nf, out=(ent, hop, pred))
        return r

    def run_steps(n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            step().close()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    if args.overlap_fetch:
        os.environ["LOGOSKG_OVERLAP_FETCH"] = "1"

    # work units of every kernel (counting mode; not timed)
    g.profile_enable(2)
    r = step()
    torch.cuda.synchronize()
    units = g.profile_read()
    counted_stats = r.hop_stats()
    physical_edges = int(sum(h["edges_scanned"] for h in counted_stats))
    r.close()
    g.profile_enable(0)

    note("work units counted; warm-up")
    run_steps(args.warmup)
    note("timed region")
    # timed region: exactly args.steps steps of the default path, nothing else on the streams:
    # `value` comes from here
    dt = run_steps(args.steps)
    # the same steps with every launch bracketed by HIP events on its own stream (two event records
    # per launch cost a few per cent of a step, which is why they stay out of `value`); the kernels
    # of a fetch run in turn, so each event pair times one kernel alone: these durations feed the
    # per-kernel table and the roofline figures
    os.environ["LOGOSKG_OVERLAP_FETCH"] = "0"
    g.profile_enable(1)
    g.profile_read()
    dt_events = run_steps(args.steps)
    prof = g.profile_read()
    g.profile_enable(0)
    if args.overlap_fetch:
        os.environ["LOGOSKG_OVERLAP_FETCH"] = "1"

    # where a step's time goes: a few more steps with an event after the khop call and after the
    # list call (not part of the timed region)
    phase_ms = [0.0, 0.0]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    for _ in range(5):
        ev[0].record()
        if walk:
            r = g.khop(seed_off, seeds, k, rel_mask, walk_exact=True)
            ev[1].record()
            r.level(k, 0, nf)
        elif triples:
            r = g.khop(seed_off, seeds, k, rel_mask)
            ev[1].record()
            r.active_triples(k, 0, nf, out=cols)
        else:
            r = g.khop(seed_off, seeds, k, rel_mask)
            ev[1].record()
            r.fetch(0, nf, out=(ent, hop, pred))
        ev[2].record()
        torch.cuda.synchronize()
        r.close()
        phase_ms[0] += ev[0].elapsed_time(ev[1]) / 5
        phase_ms[1] += ev[1].elapsed_time(ev[2]) / 5

    # what the line gathers of a dense pull hop cost on their own on this graph (measurement aid of the
    # library: every CSR entry's 128-byte subject line, the pull kernels' access shape, nothing else)
    gather_probe = None
    if W == 16 and cfg != 5:
        plane = torch.zeros((w.num_entities, 16), dtype=torch.int64, device="cuda")
        for _ in range(2):
            g.probe_gather(plane)
        pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        pe[0].record()
        for _ in range(5):
            g.probe_gather(plane)
        pe[1].record()
        torch.cuda.synchronize()
        probe_ms = pe[0].elapsed_time(pe[1]) / 5
        gather_probe = {"lines": int(w.num_triples), "ms": round(probe_ms, 4),
                        "lines_per_s": round(w.num_triples / (probe_ms * 1e-3), 1),
                        "what": "one 128-byte line per entry of the object-sorted CSR, in CSR order"}
        del plane

    ab = functools.partial(algorithmic_bytes, level_lists=walk or triples)
    masked_arg = masked
    ms_per_step = dt / args.steps * 1e3
    qps = Q / (dt / args.steps)
    kernels = {}
    for name, p in prof.items():
        if p["launches"] == 0:
            continue
        u = units.get(name, {})
        per_step = {x: u.get(x, 0) for x in ("rows", "edges", "lines", "items")}
        kernels[name] = dict(launches_per_step=p["launches"] / args.steps,
                             ms_per_step=p["total_ms"] / args.steps,
                             avg_ms=p["total_ms"] / p["launches"],
                             **per_step)
    expansion_names = ("push_", "pull_", "update_", "frontier_", "seed_", "clear_", "live_", "hop_")
    expansion_ms = sum(v["ms_per_step"] for n, v in kernels.items() if n.startswith(expansion_names))
    plane_bytes = float(res_epad * W * 8)
    expansion_bytes = sum(ab(n, v, W, k, masked_arg, plane_bytes) for n, v in kernels.items()
                          if n.startswith(expansion_names))
    # lines the pull kernels gather per second: a dense hop takes the line of every entry it scans
    pull_ms = sum(kernels[n]["ms_per_step"] for n in ("pull_tail", "pull_seg") if n in kernels)
    pull_lines = sum(h["edges_scanned"] if h["frontier_edges"] * 100 >= w.num_triples * 60 else h["lines_gathered"]
                     for h in counted_stats if h["direction"] == 2)
    pull_lines_per_s = round(pull_lines / (pull_ms * 1e-3), 1) if pull_ms > 0 and pull_lines > 0 else None
    lists_fused = "lists" not in kernels  # the predecessor tile kernel wrote the entity / hop lists too
    dom = max(kernels, key=lambda n: kernels[n]["ms_per_step"])
    dk = kernels[dom]
    alg = ab(dom, dk, W, k, masked_arg, plane_bytes, lists_fused) / max(dk["launches_per_step"], 1)
    achieved = alg / (dk["avg_ms"] * 1e-3) / 1e9 if dk["avg_ms"] > 0 else 0.0
    # HBM bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE / WRITE_SIZE,
    # calibrated); counters cannot be read from inside this process
    traffic = None
    traffic_source = None
    valu_view = None
    expansion_measured = None
    here = os.path.dirname(os.path.abspath(__file__))
    tfile = os.path.join(here, "profiles", "pmc_traffic.json")
    if os.path.exists(tfile) and args.scale == 1.0 and cfg == 2 and not walk and nf == Q:
        stored = json.load(open(tfile))
        # the stored counter readings belong to one build of the kernels: they are used only while
        # the kernel sources are the ones they were measured on
        if stored.get("kernel_sources_sha256") == kernel_sources_sha256(here):
            tk = stored.get("kernels", {})
            traffic_source = (f"stored: {stored.get('source')} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of "
                              f"commit {stored.get('commit', '?')}, same kernel sources; not read in this run)")
        else:
            tk = {}
            traffic_source = "none: the kernel sources differ from those profiles/pmc_traffic.json was measured on"
        traffic = tk.get(dom, {}).get("hbm_bytes_per_launch")
        sq = tk.get(dom, {}).get("sq_counters")
        if sq and dk["avg_ms"] > 0:  # how busy the vector ALUs are: the kernel may be bound by instruction issue
            simd_cycles = 1024 * dk["avg_ms"] * 1e-3 * 2.4e9
            valu_view = {"wave_instructions_per_launch": sq["SQ_INSTS_VALU"],
                         "issue_busy_frac": round(sq["SQ_INSTS_VALU"] * 4 / simd_cycles, 3),
                         "lanes_active_per_instruction": round(sq["SQ_THREAD_CYCLES_VALU"] / sq["SQ_ACTIVE_INST_VALU"], 1),
                         "source": "rocprofv3 --pmc SQ_* of the same kernel (profiles/)"}
        expansion_measured = sum(tk[n]["hbm_read_bytes_per_step"] + tk[n]["hbm_write_bytes_per_step"]
                                 for n in kernels if n.startswith(expansion_names) and n in tk)
        expansion_measured += kernels.get("clear_planes", {}).get("items", 0) * 8  # a memset: its own size
    roofline = dict(bound="hbm", kernel=dom, achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBS, 4), traffic=traffic, traffic_source=traffic_source,
                    algorithmic_bytes_per_launch=int(alg), avg_launch_ms=round(dk["avg_ms"], 4),
                    measured="HIP events around every launch, fetch kernels serialized", valu=valu_view)
    # the same figure for every kernel that has a byte model
    exp = {}
    for n, v in kernels.items():
        b = ab(n, v, W, k, masked_arg, plane_bytes, lists_fused)
        if b > 0 and v["ms_per_step"] > 0:
            exp[n] = dict(GBps=round(b / (v["ms_per_step"] * 1e-3) / 1e9, 1),
                          frac=round(b / (v["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                          ms_per_step=round(v["ms_per_step"], 4), bytes_per_step=int(b))

    if triples:
        metric = (f"queries/s, {k}-hop batch-{Q} on configs[{cfg - 1}] (khop + the active triples T_{k} of the first "
                  f"{nf} queries: {n_triples:,} triples with subject, relation and object)")
    elif cfg == 2 and not walk:
        metric = "queries/s, 3-hop batch-1024 on 30M-edge synthetic KG (whole hot path: khop + result lists)"
    elif cfg == 2:
        metric = ("queries/s, walk-exact 3-hop batch-1024 on 30M-edge synthetic KG (khop without the visited set + "
                  "the level-3 list of every query)")
    else:
        metric = (f"queries/s, {k}-hop batch-{Q} on configs[{cfg - 1}] (khop + the lists of the first {nf} queries"
                  + (", walk-exact" if walk else "") + ")")
    workload = f"configs[{cfg - 1}]: {w.num_entities:,} entities, {w.num_triples:,} triples, {w.num_relations:,} " \
               f"relations, {Q:,} queries, k={k}, " + ("per-query relation whitelists" if masked else "no relation mask")
    if cfg == 2:
        workload = ("configs[1]: 3,000,000 entities, 30,000,000 triples, 500 relations, "
                    "1,024 queries x 1-5 seeds, k=3, no relation mask")
    if cfg == 4:
        workload += " (first of four 1,024-query batches)"
    if cfg == 5:
        workload += " (8 shards, 64 GB shard budget, shards cached from pinned host memory" + \
                    (f", at most {args.resident_shards} resident" if args.resident_shards else "") + \
                    (", shards read from files on a cache miss" if args.shard_dir else "") + ")"
    out = {
        "metric": metric,
        "value": round(qps, 1), "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": workload +
                               ("" if args.scale == 1.0 else f" (scaled by {args.scale})"),
                   "num_entities": w.num_entities, "num_triples": w.num_triples, "num_queries": Q, "k": k,
                   "mode": args.mode, "words_per_entity": W, "reached_pairs": total, "queries_fetched": nf,
                   "reached_pairs_all_queries": int(off[-1]), "active_triples": n_triples,
                   "directions": [h["direction"] for h in hop_stats]},
        "gteps_logical": round(logical_edges / (dt / args.steps) / 1e9, 2),
        "gteps_physical": round(physical_edges / (dt / args.steps) / 1e9, 3),
        "logical_edges_per_step": logical_edges, "physical_edges_per_step": physical_edges,
        "ms_per_step_with_events": round(dt_events / args.steps * 1e3, 4),
        "fetch_kernels": "overlapped on helper streams" if args.overlap_fetch else "in turn on one stream",
        "phase_ms": {"khop": round(phase_ms[0], 4), "lists": round(phase_ms[1], 4),
                     "measured": "events after each of the two calls, 5 extra steps"},
        "expansion": {"ms_per_step": round(expansion_ms, 4),
                      "queries_per_s": round(Q / (expansion_ms * 1e-3), 1) if expansion_ms > 0 else None,
                      "algorithmic_GBps": round(expansion_bytes / (expansion_ms * 1e-3) / 1e9, 1) if expansion_ms else None,
                      "hbm_frac": round(expansion_bytes / (expansion_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if expansion_ms else None,
                      "gteps_logical": round(logical_edges / (expansion_ms * 1e-3) / 1e9, 1) if expansion_ms else None,
                      "frac_of_stream_copy": round(expansion_bytes / (expansion_ms * 1e-3) / 1e9 / stream_copy_gbps, 4)
                      if expansion_ms else None,
                      "counter_GBps": round(expansion_measured / (expansion_ms * 1e-3) / 1e9, 1)
                      if expansion_measured and expansion_ms else None,
                      "counter_hbm_frac": round(expansion_measured / (expansion_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
                      if expansion_measured and expansion_ms else None,
                      # the pull kernels' line gathers against the gathers alone (same lines per CSR entry)
                      "gather_probe": gather_probe,
                      "pull_lines_per_s": pull_lines_per_s,
                      "pull_frac_of_gather_probe": round(pull_lines_per_s / gather_probe["lines_per_s"], 4)
                      if gather_probe and pull_lines_per_s else None},
        "stream_copy_GBps": round(stream_copy_gbps, 1),
        "roofline": roofline,
        "kernels": {n: {kk: (round(vv, 4) if isinstance(vv, float) else vv) for kk, vv in v.items()}
                    for n, v in kernels.items()},
        "kernel_hbm": exp,
        "hop_stats": counted_stats,
        "setup_s": {"generate": round(t_gen, 1), "build": round(t_build, 1)},
    }

    if cfg == 5:
        out["shard_cache"] = {kk: vv for kk, vv in g.info().items()
                              if kk.startswith("shard_") or kk in ("num_shards", "pinned_host_bytes", "device_bytes")}
    note(f"{ms_per_step:.3f} ms per step")
    if not args.no_cpu_baseline:
        note("oracle on the host cores")
        import oracle  # the cpu_baseline leg is the only user of the oracle here
        nq = min(args.cpu_queries or (512 if cfg <= 3 else 6), nf)
        so = w.seed_off[: nq + 1]
        sd = w.seeds[: so[-1]]
        mk = None if w.rel_mask is None else w.rel_mask[:nq]
        if triples:
            nq = min(nq, 8)
            so = w.seed_off[: nq + 1]
            sd = w.seeds[: so[-1]]
            mk = None if w.rel_mask is None else w.rel_mask[:nq]
        t0 = time.perf_counter()
        if triples:
            o = oracle.khop(w.num_entities, w.subj, w.rel, w.obj, so, sd, k, mk)
            o_t = []
            for q in range(nq):
                a, b = o[0][q], o[0][q + 1]
                o_t.append(oracle.active_triples(w.num_entities, w.subj, w.rel, o[1][a:b][o[2][a:b] == k - 1],
                                                 None if mk is None else mk[q]))
        elif walk:
            o_off, o_ent = oracle.walk_levels(w.num_entities, w.subj, w.rel, w.obj, so, sd, k, mk)
        else:
            o = oracle.khop(w.num_entities, w.subj, w.rel, w.obj, so, sd, k, mk)
        t_cpu = time.perf_counter() - t0
        cores = oracle.num_threads()  # read here: the single-thread run below leaves the OpenMP setting at 1
        # the oracle's own index build (an empty batch builds it and runs no query), and a
        # single-thread run on the first 64 queries
        t0 = time.perf_counter()
        oracle.khop(w.num_entities, w.subj, w.rel, w.obj, np.zeros(1, dtype=np.int64), np.zeros(0, dtype=np.int32), k, None)
        t_index = time.perf_counter() - t0
        n1 = min(64, nq) if cfg <= 3 else min(2, nq)
        t0 = time.perf_counter()
        oracle.khop(w.num_entities, w.subj, w.rel, w.obj, w.seed_off[: n1 + 1], w.seeds[: w.seed_off[n1]], k,
                    None if w.rel_mask is None else w.rel_mask[:n1], nthreads=1)
        t_one = time.perf_counter() - t0
        got = g.khop(seed_off, seeds, k, rel_mask, walk_exact=walk)
        if triples:
            t_off, t_id, t_s, t_r, t_o = got.active_triples(k, 0, nq)
            want = np.concatenate(o_t) if o_t else np.zeros(0, dtype=np.int32)
            same = (np.array_equal(t_off, np.concatenate([[0], np.cumsum([len(x) for x in o_t])])) and
                    np.array_equal(t_id.cpu().numpy(), want) and np.array_equal(t_s.cpu().numpy(), w.subj[want]) and
                    np.array_equal(t_r.cpu().numpy(), w.rel[want]) and np.array_equal(t_o.cpu().numpy(), w.obj[want]))
        elif walk:
            l_off, l_ent = got.level(k, 0, nq)
            a = o_off[k * nq:(k + 1) * nq + 1]
            same = (np.array_equal(l_off[: nq + 1], a - a[0]) and
                    np.array_equal(l_ent.cpu().numpy(), o_ent[a[0]:a[-1]]))
        else:
            e2, h2, p2 = got.fetch(0, nq)
            same = (np.array_equal(off[: nq + 1], o[0]) and np.array_equal(e2.cpu().numpy(), o[1])
                    and np.array_equal(h2.cpu().numpy(), o[2]) and np.array_equal(p2.cpu().numpy(), o[3]))
        got.close()
        out["cpu_baseline"] = {"value": round(nq / t_cpu, 2), "unit": "queries/s", "cores": cores,
                               "kind": "oracle",
                               "sample": f"first {nq} of the {Q} queries of the same workload, one query per "
                                         f"thread, index build included ({t_cpu:.1f} s)",
                               "matches_gpu": bool(same), "host_cpus": os.cpu_count(), "cpu_model": cpu_model(),
                               "index_build_s": round(t_index, 2),
                               # (None when the index build, timed in a run of its own, is as long as the
                               # whole oracle run: the difference is then noise)
                               "value_without_index_build":
                                   round(nq / (t_cpu - t_index), 2) if t_cpu - t_index > 0.05 * t_cpu else None,
                               "single_thread": {"queries": n1, "seconds": round(t_one, 2),
                                                 "queries_per_s_without_index_build":
                                                     round(n1 / (t_one - t_index), 2)
                                                     if t_one - t_index > 0.05 * t_one else None}}
    g.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
