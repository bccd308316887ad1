"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C source (a swapped index, a
dropped round, a wrong sign, an off-by-one, a changed tie-break ...), builds it, points the oracle package at the
altered library and runs the pins that are meant to catch that mistake: at least one of them must fail.  Everything
runs on the CPU; the real oracle library is restored afterwards."""
import os
import subprocess

import pytest

import oracle
import test_oracle_2opt as t2
import test_oracle_bcube as tb
import test_oracle_costs as tc
import test_oracle_dbt as td
import test_oracle_local as tl
import test_oracle_probes as tp
import test_oracle_rdswap as ts
import test_oracle_sa as ta

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "cc_oracle.c")

# (name, text in the source, replacement, which occurrence (0-based), pins that must notice)
MUTANTS = [
    ("ring hop direction swapped",
     "int64_t hop = C_(pi[p], pi[pp]);", "int64_t hop = C_(pi[pp], pi[p]);", 0,
     [lambda: tc.test_ring_hop_direction(8)]),
    ("ring max starts from zero hop only",
     "if (objective & 1) acc = (p == 0) ? hop : max64(acc, hop);", "if (objective & 1) acc = hop;", 0,
     [lambda: tc.test_ring_rotation_reversal_transpose(8, oracle.MAX), lambda: tc.test_worked_example_n4(GOLDEN)]),
    ("halving-doubling partner by addition instead of xor",
     "worst = max64(worst, C_(pi[i], pi[i ^ bit]));", "worst = max64(worst, C_(pi[i], pi[(i + bit) % N]));", 0,
     [lambda: tc.test_rd_hypercube_automorphisms(8), lambda: tc.test_rd_clean_hierarchy_closed_form(64, 8),
      lambda: tc.test_worked_example_n4(GOLDEN)]),
    ("halving-doubling last round dropped",
     "for (int32_t bit = 1; bit < N; bit <<= 1) {\n        int64_t worst = 0;\n        for (int32_t i = 0; i < N; ++i)",
     "for (int32_t bit = 1; bit < N / 2; bit <<= 1) {\n        int64_t worst = 0;\n        for (int32_t i = 0; i < N; ++i)", 0,
     [lambda: tc.test_rd_constant(8)]),
    ("SplitMix64 first shift 31 instead of 30",
     "z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;", "z = (z ^ (z >> 31)) * 0xBF58476D1CE4E5B9ULL;", 0,
     [lambda: t2.test_splitmix64_published_vectors(GOLDEN)]),
    ("shuffle range k instead of k + 1",
     "int32_t jdx = (int32_t)((u * (uint64_t)(k + 1)) >> 32);", "int32_t jdx = (int32_t)((u * (uint64_t)k) >> 32);", 0,
     [t2.test_init_tours_uniform_n4]),
    ("2-opt sum delta: removed hop q forgotten",
     "v0 = cur + x0 + y0 - f[i] - f[q];", "v0 = cur + x0 + y0 - f[i] - f[j];", 0,
     [lambda: t2.test_fast_move_values_equal_apply_and_recompute(8, oracle.SUM)]),
    ("2-opt directed: inside hops not reversed",
     "v0 = x0 + y0 + out_f + in_b;", "v0 = x0 + y0 + out_f + in_f;", 0,
     [lambda: t2.test_fast_move_values_equal_apply_and_recompute(8, oracle.SUM_DIRECTED)]),
    ("2-opt new hop uses rank i instead of i - 1",
     "int64_t x0 = C_(t[j], t[i - 1]), y0 = C_(t[q], t[i]);", "int64_t x0 = C_(t[j], t[i]), y0 = C_(t[q], t[i]);", 0,
     [lambda: t2.test_fast_move_values_equal_apply_and_recompute(8, oracle.MAX)]),
    ("2-opt tie-break: last equal value wins",
     "if (!found || v < best->value || (v == best->value && id < best->id)) {", "if (!found || v <= best->value) {", 0,
     [lambda: t2.test_descent_trajectory_definition_vs_fast_and_certificate(9, oracle.MAX)]),
    ("2-opt descent also takes equal-cost moves (bounded by the trace length)",
     "if (!found || best.value >= cur) break;", "if (!found || best.value > cur || applied >= 1000) break;", 0,
     [lambda: t2.test_descent_trajectory_definition_vs_fast_and_certificate(9, oracle.MAX),
      lambda: t2.test_workload_restarts_are_certified_local_optima(3, oracle.MAX_DIRECTED)]),
    ("best restart: last minimum instead of first",
     "if (costs[r] < costs[arg]) arg = r;", "if (costs[r] <= costs[arg]) arg = r;", 0,
     [t2.test_search_is_argmin_over_restarts_lowest_id]),
    ("pair swap: only the two largest links kept",
     "for (int m = 0; m < top[k].n; ++m)\n                    if (top[k].link[m] != lp && top[k].link[m] != lq)",
     "for (int m = 0; m < top[k].n && m < 2; ++m)\n                    if (top[k].link[m] != lp && top[k].link[m] != lq)", 0,
     [lambda: ts.test_fast_swap_values_equal_swap_and_recompute(16, True)]),
    ("pair swap: link of rank p evaluated with its old node",
     "int64_t link_p = max64(C_(t[q], pb), C_(pb, t[q]));", "int64_t link_p = max64(C_(t[p], pb), C_(pb, t[p]));", 0,
     [lambda: ts.test_fast_swap_values_equal_swap_and_recompute(8, True)]),
    ("BCube peer digit without wrap-around",
     "int32_t peer = (int32_t)(j - digit * stride + ((digit + k) % B) * stride);\n                worst = max64(worst, C_(pi[j], pi[peer]));\n            }\n        }\n        total += worst;",
     "int32_t peer = (int32_t)(j - digit * stride + ((digit + k) % B) * stride);\n                if (digit + k >= B) continue;\n                worst = max64(worst, C_(pi[j], pi[peer]));\n            }\n        }\n        total += worst;", 0,
     [lambda: tb.test_base_2_is_halving_doubling(8), lambda: tb.test_digit_automorphisms(16, 4)]),
    ("double binary tree: left child one rank off",
     "int32_t child = pi[((i + m - 1) / 2 + shift) % N];", "int32_t child = pi[((i + m) / 2 + shift) % N];", 0,
     [lambda: td.test_against_explicit_paths(13), td.test_hand_worked_trees]),
    ("double binary tree: second tree ignored",
     "return max64(cco_dbt_tree_cost(c, N, pi, 0), cco_dbt_tree_cost(c, N, pi, 1));",
     "return cco_dbt_tree_cost(c, N, pi, 0);", 0,
     [lambda: td.test_against_explicit_paths(13), td.test_hand_worked_trees]),
    ("annealing: delta with the wrong sign on a removed hop",
     "delta = C_(t[ap], t[bp]) + C_(t[a], t[b]) - C_(t[a], t[ap]) - C_(t[b], t[bp]);",
     "delta = C_(t[ap], t[bp]) + C_(t[a], t[b]) - C_(t[a], t[ap]) + C_(t[b], t[bp]);", 0,
     [lambda: ta.test_chain_bookkeeping_against_recomputation(9, 50)]),
    ("annealing: logarithm's fraction shifted the wrong way",
     "int32_t frac = e >= 12 ? (m >> (e - 12)) : (m << (12 - e));", "int32_t frac = e >= 12 ? (m >> (e - 11)) : (m << (12 - e));", 0,
     [ta.test_log2_fix_exact_at_powers_of_two_and_below_true_log,
      lambda: ta.test_acceptance_probability_tracks_boltzmann_factor(100, 37)]),
    ("annealing: temperature does not cool",
     "int64_t num = (int64_t)t_start * (steps - s) + (int64_t)t_end * s;", "int64_t num = (int64_t)t_start * steps;", 0,
     [ta.test_chain_replayed_move_by_move]),
    ("annealing: uphill moves accepted when they should be rejected",
     "return delta * 4096 * steps <= num * E;", "return delta * 4096 * steps >= num * E;", 0,
     [ta.test_constant_temperature_chain_samples_the_boltzmann_distribution, ta.test_acceptance_special_cases]),
    ("segment insertion: edge behind the segment not removed",
     "int64_t without = cur - C_(A, S1) - C_(S2, B) + C_(A, B);", "int64_t without = cur - C_(A, S1) + C_(A, B);", 0,
     [lambda: tl.test_fast_values_equal_apply_and_recompute(7, 4)]),
    ("segment insertion: reversed segment joined the wrong way round",
     "(o ? C_(P, S2) + C_(S1, Q) : C_(P, S1) + C_(S2, Q));", "(o ? C_(P, S1) + C_(S2, Q) : C_(P, S1) + C_(S2, Q));", 0,
     [lambda: tl.test_fast_values_equal_apply_and_recompute(7, 4),
      lambda: tl.test_circle_metric_displaced_segment_is_repaired_in_one_move(16, 3, True)]),
    ("segment insertion: segment put in front of the gap's first node",
     "if (p == g) at = n;                 /* the segment goes in front of rest[at] */",
     "if (p == g) at = n - 1;", 0,
     [lambda: tl.test_apply_equals_python_list_model(7)]),
    ("segment insertion: gaps next to the segment allowed",
     "if (g >= s - 1 && g <= s + L - 1) return 0;", "if (g >= s && g <= s + L - 2) return 0;", 0,
     [lambda: tl.test_move_set_size_ids_and_validity(6)]),
    ("union of classes: an insertion wins a tie against a 2-opt move",
     "if (f2 && (!found || cand.value < best.value || (cand.value == best.value && cand.id < best.id))) {",
     "if (f2 && (!found || cand.value <= best.value)) {", 0,
     [tl.test_union_tie_goes_to_the_2opt_move]),
    ("orientation flip scored with the hops as walked now",
     "int64_t back = C_(t[(p - 1 + N) % N], t[p]);", "int64_t back = C_(t[p], t[(p - 1 + N) % N]);", 0,
     [lambda: tl.test_flip_on_a_one_way_ring(oracle.SUM_DIRECTED),
      lambda: tl.test_flip_trajectory_definition_vs_fast(9, 2, oracle.MAX_DIRECTED)]),
    ("probes: percentile rank off by one",
     "out[(int64_t)a * N + b] = buf[rank - 1];", "out[(int64_t)a * N + b] = buf[rank < K ? rank : K - 1];", 0,
     [tp.test_hand_worked, lambda: tp.test_against_numpy_nearest_rank_percentile(8, 100, 10)]),
    ("probes: symmetrise with the smaller direction",
     "int32_t m = out[(int64_t)a * N + b] > out[(int64_t)b * N + a] ?", "int32_t m = out[(int64_t)a * N + b] < out[(int64_t)b * N + a] ?", 0,
     [tp.test_hand_worked]),
]


def _nth_replace(text, old, new, which):
    pos = -1
    for _ in range(which + 1):
        pos = text.find(old, pos + 1)
        assert pos >= 0, "mutation target not found in the oracle source"
    return text[:pos] + new + text[pos + len(old):]


@pytest.mark.parametrize("name,old,new,which,pins", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new, which, pins):
    src = _nth_replace(open(SRC).read(), old, new, which)
    c_file, so_file = tmp_path / "mutant.c", tmp_path / "mutant.so"
    c_file.write_text(src)
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", str(c_file), "-o", str(so_file)])
    real = oracle._L()
    failures = 0
    try:
        oracle._lib = oracle._declare(str(so_file))
        for pin in pins:
            try:
                pin()
            except (AssertionError, RuntimeError):
                failures += 1
    finally:
        oracle._lib = real
    assert failures >= 1, f"no pin noticed: {name}"


def test_the_unaltered_source_passes_the_same_pins():
    for _, _, _, _, pins in MUTANTS:
        for pin in pins:
            pin()
