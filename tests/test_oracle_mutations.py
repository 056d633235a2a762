"""The pins must have teeth: plant one plausible mistake at a time in a scratch
copy of the oracle's C source (on the CPU, never in the product), rebuild it,
and require that at least one pin test fails."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins
import test_oracle_walk_pins as wpins
import test_oracle_triples_pins as tpins
import test_oracle_walk_paths_pins as wppins

MUTATIONS = {
    "tie_break_dropped": ("} else if (st->hop[v] == h && t < st->pred[v]) {",
                          "} else if (0) {"),
    "tie_break_takes_largest": ("st->hop[v] == h && t < st->pred[v]", "st->hop[v] == h && t > st->pred[v]"),
    "mask_ignored": ("    if (!mask) return 1;\n", "    return 1;\n"),
    "mask_bit_index_wrong": ("(mask[r >> 6] >> (r & 63))", "(mask[r >> 6] >> ((r + 1) & 63))"),
    "subject_used_as_target": ("int32_t v = obj[t];\n    if (st->hop[v] == UNREACHED) {",
                               "int32_t v = obj[t > 0 ? t - 1 : t];\n    if (st->hop[v] == UNREACHED) {"),
    # (the traversed[] write is kept inside its k entries so the planted bug cannot corrupt the heap)
    "one_hop_too_many": ("for (int h = 1; h <= k; ++h) {\n        int64_t inspected = 0;",
                         "for (int h = 1; h <= k + 1; ++h) {\n        int64_t inspected = 0; if (h > k) trav = NULL;"),
    "one_hop_too_few": ("for (int h = 1; h <= k; ++h) {", "for (int h = 1; h < k; ++h) {"),
    "traversed_counts_only_allowed": ("                    ++inspected;\n                    if (!relation_allowed(mask, rel[t])) continue;",
                                      "                    if (!relation_allowed(mask, rel[t])) continue;\n                    ++inspected;"),
    "seed_pred_zero": ("st->pred[e] = -1;", "st->pred[e] = 0;"),
    "paths_forward_order": ("row[i] = c->stack[c->d - 1 - i];", "row[i] = c->stack[i];"),
    "paths_wrong_level": ("if (c->hop[c->subj[t]] != level - 1) continue;", "if (c->hop[c->subj[t]] != level) continue;"),
    "paths_ignore_mask": ("        if (!relation_allowed(c->mask, c->rel[t])) continue;\n", ""),
    # walk-exact levels
    "walk_keeps_a_visited_set": ("                int64_t n_nxt = 0;\n                ++mark;", "                int64_t n_nxt = 0;"),
    "walk_mask_dropped": ("                        if (!relation_allowed(mask, rel[t])) continue;\n                        int32_t v = obj[t];",
                          "                        int32_t v = obj[t];"),
    "walk_sets_the_subject": ("                        int32_t v = obj[t];\n                        if (stamp[v] != mark)",
                              "                        int32_t v = subj[t];\n                        if (stamp[v] != mark)"),
    "walk_last_level_missing": ("                if (h == k) break;", "                if (h >= k - 1) break;"),
    # walk listing
    "walk_paths_wrong_level": ("if (!c->member[(size_t)(level - 1) * c->E + c->subj[t]]) continue;",
                               "if (!c->member[(size_t)level * c->E + c->subj[t]]) continue;"),
    "walk_paths_start_anywhere": ("for (int64_t a = seed_off[q]; a < seed_off[q + 1]; ++a) member[seeds[a]] = 1;",
                                  "memset(member, 1, (size_t)E);"),
    "walk_paths_levels_never_advance": ("                        member[(size_t)h * E + obj[t]] = 1;",
                                        "                        member[(size_t)h * E + subj[t]] = 1;"),
    # active-triple sets
    "triples_ignore_whitelist": ("in_q[subj[t]] && relation_allowed(mask, rel[t])", "in_q[subj[t]]"),
    "triples_ordered_by_index_only": ("    if (x->s != y->s) return x->s < y->s ? -1 : 1;\n", ""),
    "triples_subjects_descending": ("return x->s < y->s ? -1 : 1;", "return x->s > y->s ? -1 : 1;"),
    "triples_frontier_shifted": ("        in_q[frontier[i]] = 1;", "        in_q[frontier[i] > 0 ? frontier[i] - 1 : 0] = 1;"),
}

PIN_CALLS = [
    lambda: [pins.test_hand_worked_example(m) for m in (0, 1)],
    lambda: [pins.test_against_boolean_matrix_powers(s, m) for s in range(4) for m in (False, True)],
    lambda: [pins.test_against_walk_enumeration(s, m) for s in range(4) for m in (False, True)],
    lambda: pins.test_tie_break_smallest_edge_id_and_mask_selects_other_edge(),
    lambda: pins.test_directed_cycle_never_lowers_the_seed(0),
    lambda: pins.test_first_path_is_the_pred_chain(),
    lambda: [wpins.test_against_boolean_matrix_powers(s, m) for s in range(3) for m in (False, True)],
    lambda: wpins.test_cycle_path_self_loop_and_bipartite(),
    lambda: wppins.test_hand_worked_example(),
    lambda: [wppins.test_against_forward_enumeration(s, m) for s in range(3) for m in (False, True)],
    lambda: wppins.test_closed_forms(),
    lambda: tpins.test_hand_worked_example(),
    lambda: [tpins.test_against_dense_incidence_product(s, m) for s in range(3) for m in (False, True)],
    lambda: tpins.test_closed_forms(),
]


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path, monkeypatch):
    old, new = MUTATIONS[name]
    src = open(os.path.join(os.path.dirname(oracle.__file__), "khop_oracle.c")).read()
    assert src.count(old) >= 1, "mutation site vanished"
    mutated = tmp_path / "mut.c"
    mutated.write_text(src.replace(old, new))
    lib_path = str(tmp_path / "libmut.so")
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", lib_path,
                           str(mutated)])
    good = oracle._load()
    lib = ctypes.CDLL(lib_path)
    for fn in ("oracle_khop", "oracle_paths", "oracle_walk_levels", "oracle_walk_paths", "oracle_active_triples",
               "oracle_free",
               "oracle_num_threads"):
        getattr(lib, fn).argtypes = getattr(good, fn).argtypes
        getattr(lib, fn).restype = getattr(good, fn).restype
    monkeypatch.setattr(oracle, "_lib", lib)
    caught = False
    for call in PIN_CALLS:
        try:
            call()
        except AssertionError:
            caught = True
            break
    assert caught, f"no pin noticed the planted mistake '{name}'"


# ---------------------------------------------------------------- Sec. 3.4 helpers (plain Python)
PARTITION_MUTATIONS = {
    "shard_order_flipped": ("if h % 2 == 0:", "if h % 2 == 1:"),
    "shard_order_never_reversed": ("if h % 2 == 0:", "if False:"),
    "rows_without_triples_routed": ("front = front[deg[front] > 0]", "front = front[deg[front] >= 0]"),
    "frontier_from_the_wrong_level": ("front = np.unique(entity[hop == h - 1])", "front = np.unique(entity[hop == h])"),
    "lru_evicts_most_recent": ("cache.popitem(last=False)", "cache.popitem(last=True)"),
    "lru_hit_does_not_refresh": ("            cache.move_to_end(a)\n", ""),
    "pulled_hop_routed_by_subject": ("        if h in pull_hops:", "        if False:"),
    "object_ranges_numbered_from_zero": ("order = list(range(num_shards, num_shards + num_ranges))",
                                         "order = list(range(0, num_ranges))"),
    "fetch_takes_the_indices_first": ("seq += [num_shards + c, num_shards + num_ranges + c]",
                                      "seq += [num_shards + num_ranges + c, num_shards + c]"),
    "fetch_through_a_small_cache": ("    if capacity < num_shards + 2 * num_ranges:", "    if capacity < 4:"),
}


@pytest.mark.parametrize("name", sorted(PARTITION_MUTATIONS))
def test_planted_mistake_in_partition_helpers_is_caught(name):
    import types
    old, new = PARTITION_MUTATIONS[name]
    src = open(os.path.join(os.path.dirname(oracle.__file__), "partition.py")).read()
    assert src.count(old) == 1, "mutation site vanished"
    mod = types.ModuleType("partition_mutant")
    exec(compile(src.replace(old, new), "partition_mutant.py", "exec"), mod.__dict__)
    caught = False
    try:
        seq = pins.shard_access_trace(mod)
        assert seq == [0, 2, 3, 1, 0, 1]
        assert mod.lru_counts(seq, 2) == (5, 3, 1)
        assert mod.lru_counts([0, 1, 0, 2, 0, 3], 2) == (4, 2, 2)
        assert pins.shard_access_trace(mod, pull_hops={2}) == [0, 2, 6, 5, 4, 0, 1]
        assert mod.fetch_accesses(4, 3, 10) == [4, 7, 5, 8, 6, 9] and mod.fetch_accesses(4, 3, 9) == []
    except (AssertionError, IndexError):
        caught = True
    assert caught, f"no pin noticed the planted mistake '{name}'"
