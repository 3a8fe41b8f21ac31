"""The pins bite: plausible mistakes planted in the oracle's source (a dropped term, a wrong
sign or index, a swapped operand) must each fail at least one pin.  Every mutant is the
oracle's C file with one edit, compiled into a scratch library and swapped in for the run
of the pin tests (CPU only; nothing here touches the GPU path).  The edits are chosen to
stay inside the arrays, so a mutant computes a wrong answer rather than crashing; the one
that cannot (marked "isolate") runs its checks in a process of its own, where a crash
counts as noticed."""
import ctypes
import os
import subprocess
import sys

import pytest

from oracle import oracle as orc
import test_oracle_pins as pins
import test_oracle_reorder as rpins
import test_oracle_scores as spins

SRC = open(os.path.join(os.path.dirname(orc.__file__), "tier_oracle.c")).read()

# (name, text in the source, replacement, pin tests that must notice)
MUTANTS = [
    ("philox multiplier swapped", "(uint64_t)0xD2511F53u * c0", "(uint64_t)0xCD9E8D57u * c0",
     [pins.test_philox_known_answers]),
    ("philox key schedule dropped", "k1 += 0xBB67AE85u;", "",
     [pins.test_philox_known_answers]),
    ("philox 9 rounds", "round < 10", "round < 9",
     [pins.test_philox_known_answers]),
    ("random64 words swapped", "((uint64_t)w[1] << 32) | (uint64_t)w[0]", "((uint64_t)w[0] << 32) | (uint64_t)w[1]",
     [pins.test_batch_seed_keying, pins.test_draw_follows_floyd_with_documented_keying]),
    ("bounded takes the low half", "* (unsigned __int128)m) >> 64)", "* (unsigned __int128)m) & 0xFFFFFFFFFFFFFFFFull) % m",
     [pins.test_bounded_closed_forms]),
    ("floyd range off by one", "int64_t j = d - k + i;", "int64_t j = d - k + i - 1;",
     [pins.test_draw_follows_floyd_with_documented_keying, pins.test_draw_last_position_reachable_only_through_collision_rule]),
    ("floyd collision rule dropped", "pos[i] = seen ? j : t;", "pos[i] = t;",
     [pins.test_draw_distinct_and_in_range]),
    ("floyd draws from the full range (with replacement fix-up)", "(uint64_t)j + 1u);", "(uint64_t)d);",
     [pins.test_draw_follows_floyd_with_documented_keying, pins.test_draw_uniform_over_subsets_chi_square]),
    ("small degree taken in reverse order", "for (int64_t i = 0; i < d; ++i) pos[i] = i;",
     "for (int64_t i = 0; i < d; ++i) pos[i] = d - 1 - i;",
     [pins.test_draw_small_degree_takes_all_in_order, pins.test_blocks_are_valid_samples]),
    ("layer not in the counter", "(uint32_t)i, layer, TAG_NEIGHBOUR)", "(uint32_t)i, 0u, TAG_NEIGHBOUR)",
     [pins.test_draw_follows_floyd_with_documented_keying]),
    ("new nodes not sorted", "qsort(nodes + n_front, (size_t)n_new, sizeof(int32_t), cmp_i32);", "",
     [pins.test_blocks_are_valid_samples]),
    ("only new nodes draw at a hop", "for (int64_t i = 0; i < n_dst && rc == 0; ++i) {\n            int32_t v = nodes[i];",
     "for (int64_t i = (l ? n_nodes[l - 1] : 0); i < n_dst && rc == 0; ++i) {\n            int32_t v = nodes[i];",
     [pins.test_blocks_are_valid_samples, pins.test_full_fanout_equals_bfs_closure]),
    ("counts every batch twice", "counts[nodes_scratch[i]] += 1u;", "counts[nodes_scratch[i]] += 2u;",
     [pins.test_counts_equal_histogram_of_batch_frontiers]),
    ("counts skip the seeds", "for (int64_t i = 0; i < nn[n_layers]; ++i) counts", "for (int64_t i = nn[0]; i < nn[n_layers]; ++i) counts",
     [pins.test_counts_equal_histogram_of_batch_frontiers]),
    ("draw counts skip the seeds", "for (int64_t i = 0; i < n; ++i) counts[train_ids[lo + i]] += 1u;", "",
     [pins.test_draw_counts_equal_histogram_of_seeds_and_edge_sources]),
    ("draw counts take the edge position for the node", "counts[indices[eid_scratch[i]]] += 1u;",
     "counts[eid_scratch[i] % n_nodes_graph] += 1u;",
     [pins.test_draw_counts_equal_histogram_of_seeds_and_edge_sources, pins.test_draw_counts_full_fanout_closed_form]),
    ("draw counts miss the last hop", "for (int l = 0; l < n_layers; ++l) n_e += ne[l];\n            for (int64_t i = 0; i < n; ++i)",
     "for (int l = 0; l + 1 < n_layers; ++l) n_e += ne[l];\n            for (int64_t i = 0; i < n; ++i)",
     [pins.test_draw_counts_full_fanout_closed_form]),
    ("ranking ascending", "return x->count > y->count ? -1 : 1;   /* descending */", "return x->count > y->count ? 1 : -1;",
     [pins.test_rank_matches_papers_worked_example]),
    ("ties by descending id", "return (x->id > y->id) - (x->id < y->id);                        /* ascending  */",
     "return (x->id < y->id) - (x->id > y->id);",
     [pins.test_rank_equals_stable_library_sort, pins.test_budget_edges]),
    ("budget rounds up", "int64_t n_hot = (int64_t)(budget_bytes / (uint64_t)row_bytes);",
     "int64_t n_hot = (int64_t)((budget_bytes + (uint64_t)row_bytes - 1) / (uint64_t)row_bytes);",
     [pins.test_budget_edges]),
    ("map runs rank -> id", "if (rank) rank[v] = (int32_t)r;", "if (rank) rank[r] = v;",
     [pins.test_rank_matches_papers_worked_example]),
    ("gather ignores the cache", "if (slot[v] >= 0) { row = cache + (size_t)slot[v] * (size_t)row_bytes; ++hit; }",
     "if (slot[v] >= 0) { row = feat + (size_t)v * (size_t)row_bytes; ++hit; }",
     [pins.test_gather_equals_fancy_indexing_for_any_budget]),
    ("gather indexes the cache by id", "row = cache + (size_t)slot[v] * (size_t)row_bytes; ++hit;",
     "row = cache + (size_t)(v % 2) * (size_t)row_bytes; ++hit;",
     [pins.test_gather_equals_fancy_indexing_for_any_budget]),
    ("reorder: lists stay at the old id", "const int64_t i = who[r];", "const int64_t i = r;",
     [rpins.test_reorder_hand_worked_example], "isolate"),      # own process, as for any mutant that moves whole lists
    ("reorder: map applied the wrong way round", "who[rank[i]] = (int32_t)i;", "who[i] = rank[i];",
     [rpins.test_reorder_hand_worked_example, rpins.test_reorder_is_a_relabelling], "isolate"),
    ("reorder: values not renamed", "= rank[indices[indptr[i] + j]];", "= indices[indptr[i] + j];",
     [rpins.test_reorder_hand_worked_example, rpins.test_reorder_is_a_relabelling]),
    ("reorder: lists reversed while moving", "= rank[indices[indptr[i] + j]];", "= rank[indices[indptr[i] + len - 1 - j]];",
     [rpins.test_reorder_hand_worked_example, rpins.test_reorder_is_a_relabelling]),
    ("boundary gather forgets the offset", "row = cold + (size_t)(ids[i] - boundary) * (size_t)row_bytes;",
     "row = cold + (size_t)ids[i] % 3 * (size_t)row_bytes;",
     [rpins.test_rows_follow_their_nodes_and_boundary_gather]),
    ("pagerank shares are not divided", "share[v] = in_degree > 0 ? score[v] / (double)in_degree : score[v];", "share[v] = score[v];",
     [spins.test_wrpr_hand_worked, spins.test_wrpr_equals_sparse_matrix_iteration]),
    ("pagerank pulls the wrong way", "collected[indices[e]] += share[v];", "collected[v] += share[indices[e]];",
     [spins.test_wrpr_hand_worked, spins.test_wrpr_equals_sparse_matrix_iteration]),
    ("pagerank weight inverted", "const double boost = (double)n / (double)n_train;", "const double boost = (double)n_train / (double)n;",
     [spins.test_wrpr_hand_worked]),
    ("pagerank damping swapped", "const double floor_part = (1.0 - damp) / (double)n;\n            const double pulled_part = damp * collected[u];",
     "const double floor_part = damp / (double)n;\n            const double pulled_part = (1.0 - damp) * collected[u];",
     [spins.test_wrpr_equals_sparse_matrix_iteration, spins.test_wrpr_invariants]),
    ("degree counts rows instead of entries", "degree[indices[e]] += 1u;", "degree[indices[e]] = 1u;",
     [spins.test_degree_is_a_bincount]),
]


def _build(tmp_path, text, tag):
    src = tmp_path / f"mutant_{tag}.c"
    lib = tmp_path / f"mutant_{tag}.so"
    src.write_text(text)
    subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-o", str(lib), str(src)],
                   check=True, capture_output=True)
    return str(lib)


@pytest.mark.parametrize("idx", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(idx, tmp_path):
    name, old, new, checks = MUTANTS[idx][:4]
    assert SRC.count(old) == 1, f"mutation site not unique for: {name}"
    lib_path = _build(tmp_path, SRC.replace(old, new), idx)
    if len(MUTANTS[idx]) > 4:
        code = (f"import sys; sys.path[:0] = {[os.path.dirname(__file__), os.path.dirname(os.path.dirname(__file__))]!r}\n"
                f"import test_oracle_mutants as m\n"
                f"sys.exit(0 if m.run_checks({lib_path!r}, {idx}) >= 1 else 3)\n")
        rc = subprocess.run([sys.executable, "-c", code], capture_output=True).returncode
        assert rc != 3, f"no pin noticed: {name}"                   # 0 = caught by a pin, anything else = crashed
        return
    assert run_checks(lib_path, idx) >= 1, f"no pin noticed: {name}"


def run_checks(lib_path, idx):
    """Swap the mutant library in, run the mutant's pin tests, return how many failed."""
    checks = MUTANTS[idx][3]
    lib = ctypes.CDLL(lib_path)
    good = orc._load()
    # give the mutant the same prototypes as the real library
    for sym in ("orc_bounded", "orc_batch_seed", "orc_philox4x32_10", "orc_draw_positions", "orc_sample_minibatch",
                "orc_presample", "orc_presample_draws", "orc_place", "orc_fill_cache", "orc_gather", "orc_reorder_graph", "orc_reorder_rows",
                "orc_gather_boundary", "orc_score_degree", "orc_score_wrpr", "orc_rank_scores"):
        getattr(lib, sym).restype = getattr(good, sym).restype
        getattr(lib, sym).argtypes = getattr(good, sym).argtypes
    caught = 0
    orc._lib = lib
    try:
        for check in checks:
            try:
                check()
            except Exception:                                  # any failure of the pin counts as noticed
                caught += 1
    finally:
        orc._lib = good
    return caught


def test_unmutated_oracle_passes_the_same_checks():
    for m in MUTANTS:
        for check in m[3]:
            check()
