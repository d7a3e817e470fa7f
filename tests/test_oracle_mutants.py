"""The pins bite: each planted mistake in a *copy* of the oracle fails at least one pin.

The mistakes are planted in a temporary copy of ``oracle/surel_oracle.c`` on the CPU
(a dropped term, a wrong index, a transposed operand, a swapped constant); the copy is
compiled with gcc and swapped in for the real library while the pin tests run.  Only
mutants that keep every memory access in bounds are used.
"""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "surel_oracle.c")

MUTANTS = {
    # name: (text to find, replacement)
    "philox_constants_swapped": ("(uint64_t)0xD2511F53u * c0", "(uint64_t)0xCD9E8D57u * c0"),
    "philox_wrong_key_word": ("^ c3 ^ k1", "^ c3 ^ k0"),
    "philox_nine_rounds": ("round < 10", "round < 9"),
    "philox_output_transposed": ("c0 = n0; c1 = n1; c2 = n2; c3 = n3;",
                                 "c0 = n2; c1 = n1; c2 = n0; c3 = n3;"),
    "walk_same_word_every_step": ("return out[(s - 1) & 3];", "return out[0];"),
    "walk_ignores_walk_index": ("{ u, w, (uint32_t)((s - 1) >> 2), 0u }",
                                "{ u, 0u, (uint32_t)((s - 1) >> 2), 0u }"),
    "walk_ignores_start_node": ("{ u, w, (uint32_t)((s - 1) >> 2), 0u }",
                                "{ 0u, w, (uint32_t)((s - 1) >> 2), 0u }"),
    "walk_ignores_seed_high_word": ("(uint32_t)(rng_seed >> 32) };", "0u };"),
    "walk_always_first_neighbour": ("(int64_t)(r % deg)", "(int64_t)0"),
    "walk_biased_choice": ("(int64_t)(r % deg)", "(int64_t)((r % 7u) % deg)"),
    "walk_forgets_to_move": ("walk[s] = cur;", "walk[s] = cur; if (s == 2) cur = u;"),
    "rpe_drops_step_index": ("cnt[(hit - set) * L + s] += 1;", "cnt[(hit - set) * L] += 1;"),
    "rpe_skips_start_position": ("for (int64_t s = 0; s < L; ++s) {\n                const int32_t x = W",
                                 "for (int64_t s = 1; s < L; ++s) {\n                const int32_t x = W"),
    "rpe_keeps_duplicates": ("if (j == 0 || set[j] != set[j - 1])", "if (1)"),
    "rpe_descending": ("return (x > y) - (x < y);", "return (x < y) - (x > y);"),
    "join_takes_largest_head": ("rpe_ids[head[j]] < x", "rpe_ids[head[j]] > x"),
    "join_halves_reversed": ("join_cnt + (total * k + j) * L", "join_cnt + (total * k + (k - 1 - j)) * L"),
    "join_no_zero_fill": ("memset(dst, 0, (size_t)L * sizeof(uint16_t));",
                          "memset(dst, 1, (size_t)L * sizeof(uint16_t));"),
    "ids_looks_in_own_block_only": ("const int32_t b = queries[q * k + j2];\n                    const int32_t *set",
                                    "const int32_t b = queries[q * k + j];\n                    const int32_t *set"),
    "ids_local_instead_of_table_row": ("hit ? rpe_off[b] + (int64_t)(hit - set) : -1;",
                                       "hit ? (int64_t)(hit - set) : -1;"),
    "ids_absent_is_row_zero": ("hit ? rpe_off[b] + (int64_t)(hit - set) : -1;",
                               "hit ? rpe_off[b] + (int64_t)(hit - set) : 0;"),
    "ids_columns_transposed": ("out[(((q * k + j) * M * L) + t) * k + j2] =",
                               "out[(((q * k + j2) * M * L) + t) * k + j] ="),
    "prune_compares_first_entry_only": ("for (int64_t s = 0; s < g_vec_len; ++s)\n        if (x[s] != y[s])",
                                        "for (int64_t s = 0; s < 1; ++s)\n        if (x[s] != y[s])"),
    "prune_descending": ("return x[s] < y[s] ? -1 : 1;", "return x[s] < y[s] ? 1 : -1;"),
    "prune_keeps_duplicates": ("if (r == 0 || cmp_vec(sorted + r * L, sorted + (r - 1) * L) != 0) {",
                               "if (1) {"),
    "prune_code_off_by_one": ("code[r] = (int32_t)((hit - sorted) / L);",
                              "code[r] = (int32_t)((hit - sorted) / L) + (r > 0);"),
    "bfs_queries_of_a_node_descending": ("const int32_t q = held[e];",
                                         "const int32_t q = held[first[u] + first[u + 1] - 1 - e];"),
    "bfs_limit_off_by_one": ("if (n_v + n_new > B1) {", "if (n_v + n_new >= B1) {"),
    "bfs_ignores_full_node_set": ("if (n_b == B2 || n_v == B1)", "if (n_b == B2)"),
    "bfs_forgets_reached_queries": ("in_batch[q] = 1;", ";"),
    "bfs_nodes_in_reverse_tuple_order": (
        "const int32_t x = queries[(int64_t)q * k + j];\n                if (!in_vbar[x]) {",
        "const int32_t x = queries[(int64_t)q * k + (k - 1 - j)];\n                if (!in_vbar[x]) {"),
    "bfs_keeps_repeated_seeds": ("if (!in_vbar[start[i]]) {", "if (1) {"),
    "bfs_counts_a_repeated_node_twice": ("seen |= (queries[(int64_t)q * k + i] == x);", "seen |= 0;"),
    "join_copies_wrong_row": ("memcpy(dst, rpe_cnt + head[j] * L,", "memcpy(dst, rpe_cnt + rpe_off[queries[q * k + j]] * L,"),
}

PIN_TESTS = [
    "test_philox_known_answers",
    "test_walks_two_node_path_alternates",
    "test_walks_star_centre_and_leaf",
    "test_walks_path_end_and_isolated_node",
    "test_walk_stream_is_keyed_on_seed_start_walk_and_step",
    "test_walks_of_one_seed_are_not_copies_of_each_other",
    "test_walks_follow_the_stated_stream_exactly",
    "test_paper_worked_example_fragment",
    "test_rpe_hand_worked_table",
    "test_join_symmetry_and_repeated_node",
    "test_query_rpe_ids_invariants_and_agreement_with_the_union_join",
    "test_query_rpe_ids_on_the_paper_fragment",
    "test_prune_equals_python_set_and_dictionary",
    "test_prune_on_the_paper_fragment",
    "test_prune_orders_by_entries_not_by_bytes",
    "test_bfs_batch_on_a_chain_a_star_and_two_components",
    "test_bfs_batch_limits",
    "test_bfs_batch_with_limits_is_a_prefix_that_stops_for_a_stated_reason",
]
PARAM_PIN_TESTS = [
    ("test_walk_distribution_matches_enumeration", ("lollipop", 4)),
    ("test_walk_distribution_matches_enumeration", ("k4", 3)),
    ("test_rpe_equals_dense_counter_and_keeps_invariants", (50, 4)),
    ("test_join_equals_python_set_union", (2,)),
    ("test_join_equals_python_set_union", (3,)),
    ("test_query_rpe_ids_equal_dictionary_lookups", (2,)),
    ("test_bfs_batch_levels_equal_set_expansion_and_scipy_distances", (3,)),
]


def _run_pins(golden_dir):
    """Names of the pins that fail with whatever library ``oracle`` currently holds."""
    failed = []
    for name in PIN_TESTS:
        fn = getattr(pins, name)
        try:
            if "golden_dir" in fn.__code__.co_varnames[:fn.__code__.co_argcount]:
                fn(golden_dir)
            else:
                fn()
        except (AssertionError, ValueError, IndexError, KeyError):
            failed.append(name)
    for name, args in PARAM_PIN_TESTS:
        try:
            getattr(pins, name)(*args)
        except (AssertionError, ValueError, IndexError, KeyError):
            failed.append(f"{name}{args}")
    return failed


def test_unmutated_oracle_passes_the_runner(golden_dir):
    assert _run_pins(golden_dir) == []


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name, tmp_path, golden_dir, monkeypatch):
    find, repl = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(find) >= 1, f"mutation site for {name} not found"
    mutated = tmp_path / "mutant.c"
    mutated.write_text(text.replace(find, repl))
    lib_path = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-o", str(lib_path),
                    str(mutated)], check=True)
    real = oracle._load()
    mutant = ctypes.CDLL(str(lib_path))
    for fn in ("oracle_philox4x32_10", "oracle_sample_walks", "oracle_build_rpe",
               "oracle_join_queries", "oracle_query_rpe_ids", "oracle_prune_rpe",
               "oracle_bfs_batch"):
        getattr(mutant, fn).argtypes = getattr(real, fn).argtypes
        getattr(mutant, fn).restype = getattr(real, fn).restype
    monkeypatch.setattr(oracle, "_lib", mutant)
    failed = _run_pins(golden_dir)
    assert failed, f"no pin noticed the planted mistake '{name}'"
