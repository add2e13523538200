"""Do the pins bite?  Plant one plausible mistake at a time in a COPY of the oracle's source
(on the CPU, never in the HIP path), build it, point the oracle wrapper at the mutant and
require that the pin battery fails.  A mutant that survives means a pin is missing."""
import ctypes
import os
import subprocess

import pytest

import oracle
from tests import test_oracle_comm as comm_pins
from tests import test_oracle_compact as compact_pins
from tests import test_oracle_pins as pins
from tests import test_oracle_split as split_pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "rannc_dp_oracle.c")

MUTANTS = {
    "floor_instead_of_ceil": ("return (x + r - 1) / r;", "return x / r;"),
    "sum_instead_of_max": ("prev > cost[e] ? prev : cost[e]", "prev + cost[e]"),
    "min_instead_of_max": ("prev > cost[e] ? prev : cost[e]", "prev < cost[e] ? prev : cost[e]"),
    "fit_exclusive": ("(uint8_t)(m <= M)", "(uint8_t)(m < M)"),
    "keeps_last_minimiser": ("if (v < best) {\n              best = v;\n              bi = i;",
                             "if (v <= best) {\n              best = v;\n              bi = i;"),
    "level0_all_zero": ("V[CELL(0, 0, 0)] = 0;",
                        "for (size_t e0 = 0; e0 < ND; ++e0) V[e0] = 0;"),
    "memory_drops_persistent": ("(P[j] - P[i]) + ceil_div(A[j] - A[i], r)",
                                "ceil_div(A[j] - A[i], r)"),
    "memory_divides_persistent": ("(P[j] - P[i]) + ceil_div(A[j] - A[i], r)",
                                  "ceil_div((P[j] - P[i]) + (A[j] - A[i]), r)"),
    "memory_ignores_replicas": ("(P[j] - P[i]) + ceil_div(A[j] - A[i], r)",
                                "(P[j] - P[i]) + (A[j] - A[i])"),
    "wrong_replica_index": ("* D + (d - dp - 1));", "* D + (dp));"),
    "stage_skips_first_block": ("int64_t h = ceil_div(T[j] - T[i], r);",
                                "int64_t h = ceil_div(T[j] - T[i + 1], r);"),
    "time_ignores_replicas": ("int64_t h = ceil_div(T[j] - T[i], r);",
                              "int64_t h = T[j] - T[i];"),
    "select_prefers_more_stages": ("if (v < best) {\n      best = v;\n      bs = s;",
                                   "if (v <= best) {\n      best = v;\n      bs = s;"),
    "traceback_wrong_replicas": ("replicas[s - 1] = d - dp;", "replicas[s - 1] = dp;"),
    "traceback_wrong_end": ("stage_end[s - 1] = j;", "stage_end[s - 1] = i;"),
    "est_iter_off_by_one": ("(int64_t)MB + n_stages - 1;", "(int64_t)MB + n_stages;"),
    "skips_split_at_s_minus_1": ("for (int32_t i = s - 1; i <= j - 1; ++i)",
                                 "for (int32_t i = s; i <= j - 1; ++i)"),
    "comm_on_last_stage_too": ("if (o && j < N) {", "if (o) {"),
    "comm_ignores_replicas": ("__int128 den = (__int128)r * w,", "__int128 den = (__int128)w,"),
    "comm_takes_cut_before_stage": ("num = (__int128)1000 * o[j - 1];", "num = (__int128)1000 * o[i];"),
    "comm_floor_instead_of_ceil": ("h += (int64_t)((num + den - 1) / den);", "h += (int64_t)(num / den);"),
    "comm_wrong_time_unit": ("num = (__int128)1000 * o[j - 1];", "num = (__int128)1024 * o[j - 1];"),
    "comm_replaces_compute": ("h += (int64_t)((num + den - 1) / den);", "h = (int64_t)((num + den - 1) / den);"),
    "split_max_instead_of_sum": ("V[c] = kept.fwd + kept.bwd;", "V[c] = kept.fwd > kept.bwd ? kept.fwd : kept.bwd;"),
    "split_keeps_last_minimiser": ("if (x->i != y->i) return x->i < y->i;", "if (x->i != y->i) return x->i > y->i;"),
    "split_backward_takes_forward_table": ("cand.bwd = TB[before] > costb[stage] ? TB[before] : costb[stage];",
                                           "cand.bwd = TB[before] > costf[stage] ? TB[before] : costf[stage];"),
    "split_forward_ignores_history": ("cand.fwd = TF[before] > costf[stage] ? TF[before] : costf[stage];",
                                      "cand.fwd = costf[stage];"),
    "split_stores_wrong_half": ("TB[c] = kept.bwd;", "TB[c] = kept.fwd;"),
    "split_history_from_value": ("cand.bwd = TB[before] > costb[stage] ? TB[before] : costb[stage];",
                                 "cand.bwd = V[before] > costb[stage] ? V[before] : costb[stage];"),
    "split_skips_split_at_s_minus_1": ("for (int32_t i = s - 1; i < j; ++i) {", "for (int32_t i = s; i < j; ++i) {"),
    "split_device_loop_stops_early": ("for (int32_t dp = s - 1; dp < d; ++dp) {", "for (int32_t dp = s - 1; dp < d - 1; ++dp) {"),
    "split_wrong_replica_index": ("* D) + (size_t)(d - dp - 1);", "* D) + (size_t)(dp);"),
    "compact_ties_to_the_right": ("else w = ct[r] < ct[l] ? r : l;", "else w = ct[r] <= ct[l] ? r : l;"),
    "compact_takes_the_slower_neighbour": ("else w = ct[r] < ct[l] ? r : l;", "else w = ct[r] > ct[l] ? r : l;"),
    "compact_fit_exclusive": ("if (cm[v] + cm[w] > M) continue;", "if (cm[v] + cm[w] >= M) continue;"),
    "compact_descending_order": ("while (y >= 0 && ct[order[y]] > ct[v])", "while (y >= 0 && ct[order[y]] < ct[v])"),
    "compact_lists_by_the_input_times": ("while (y >= 0 && ct[order[y]] > ct[v])", "while (y >= 0 && t[order[y]] > t[v])"),
    "compact_single_walk_only": ("    if (!merged) break;\n", "    break;\n"),
    "compact_union_keeps_its_turn": ("listed[first] = listed[second] = 0;", "listed[second] = 0;"),
    "compact_count_checked_between_walks_only": ("for (int32_t x = 0; x < n && count > k; ++x) {",
                                                 "for (int32_t x = 0; x < n; ++x) {"),
    "compact_walk_limit_off_by_one": ("(max_passes <= 0 || pass <= max_passes)", "(max_passes <= 0 || pass < max_passes)"),
    "compact_ignores_transient_bytes": ("cm[g] = p[g] + a[g];", "cm[g] = p[g];"),
    "compact_neighbour_times_not_updated": ("ct[first] += ct[second];", "ct[first] += 0;"),
    "device_loop_stops_early": ("for (int32_t dp = s - 1; dp <= d - 1; ++dp)",
                                "for (int32_t dp = s - 1; dp < d - 1; ++dp)"),
}


def battery():
    for row in pins.SMALL[:16]:
        pins.test_brute_force_small(*row)
    for seed in range(4):
        pins.test_ties_everywhere(seed)
    pins.test_prefix_cells_against_enumeration()
    pins.test_tables_against_definition()
    pins.test_fit_boundary_is_inclusive()
    for seed in range(3):
        pins.test_single_stage_closed_form(seed)
        pins.test_memory_not_binding_closed_form(seed)
        pins.test_linear_partition_special_case(seed)
        pins.test_invariants(seed)
    pins.test_zero_activation_fit_independent_of_replicas()
    pins.test_oversized_block_is_infeasible()
    for row in comm_pins.SMALL[:16]:
        comm_pins.test_brute_force_small_with_comm(*row)
    comm_pins.test_worked_example()
    comm_pins.test_tables_against_definition_with_comm()
    comm_pins.test_comm_invariants(0)
    compact_pins.test_worked_example_distinct_times()
    compact_pins.test_worked_example_equal_times_pair_up()
    compact_pins.test_memory_rule_and_no_second_choice()
    compact_pins.test_worked_example_repeated_walks()
    compact_pins.test_worked_example_grown_group_loses_its_turn()
    compact_pins.test_worked_example_second_walk_lists_by_current_times()
    compact_pins.test_worked_example_walks_end_when_nothing_fits()
    for row in split_pins.SMALL[:12]:
        split_pins.test_values_are_plan_values_bounded_by_the_exact_minimum(*row)
    split_pins.test_worked_example_where_one_pair_per_cell_loses()
    for seed in range(3):
        split_pins.test_equal_halves_reduce_to_the_min_max_search(seed)


def test_battery_passes_on_the_real_oracle():
    battery()


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not unique/present"
    cfile = tmp_path / "mutant.c"
    cfile.write_text(src.replace(old, new))
    so = tmp_path / "mutant.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-o", str(so), str(cfile)],
                   check=True)
    real = oracle.lib()
    mutant = ctypes.CDLL(str(so))
    for fn in ("rannc_oracle_prefix", "rannc_oracle_table_entries", "rannc_oracle_tables",
               "rannc_oracle_dp", "rannc_oracle_dp_split", "rannc_oracle_select", "rannc_oracle_traceback",
               "rannc_oracle_est_iter_ns", "rannc_oracle_max_threads", "rannc_oracle_compact"):
        getattr(mutant, fn).argtypes = getattr(real, fn).argtypes
        getattr(mutant, fn).restype = getattr(real, fn).restype
    oracle._lib = mutant
    try:
        with pytest.raises((AssertionError, oracle.OracleError)):
            battery()
    finally:
        oracle._lib = real
