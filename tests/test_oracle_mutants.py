"""Planted mistakes in copies of the oracle's source: every one must be caught by a pin.

This shows the pins are tight enough that a dropped term, a flipped comparison, a wrong
column or a wrong tie order in the oracle would not go unnoticed.  CPU only.
"""
import os

import pytest

import oracle
import pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "select_oracle.c")

# (name, text to find, replacement).  Each 'find' must occur in the source.
MUTANTS = [
    ("accuracy_strict", "if (acc_bp[v] < min_acc_bp)", "if (acc_bp[v] <= min_acc_bp)"),
    ("accuracy_flipped", "if (acc_bp[v] < min_acc_bp)", "if (acc_bp[v] > min_acc_bp)"),
    ("latency_strict", "if (total > (int64_t)slo_us)", "if (total >= (int64_t)slo_us)"),
    ("queue_dropped", "(int64_t)lat_us[v * B + b] + (int64_t)queue_us[v];",
     "(int64_t)lat_us[v * B + b];"),
    ("latency_dropped", "(int64_t)lat_us[v * B + b] + (int64_t)queue_us[v];",
     "(int64_t)queue_us[v];"),
    ("sum_wraps_int32", "(int64_t)lat_us[v * B + b] + (int64_t)queue_us[v];",
     "(int64_t)(int32_t)((uint32_t)lat_us[v * B + b] + (uint32_t)queue_us[v]);"),
    ("cost_order_flipped", "return cv < cw;", "return cv > cw;"),
    ("latency_tie_flipped", "return lv < lw;", "return lv > lw;"),
    ("row_tie_flipped", "return v < w;", "return v > w;"),
    ("latency_tie_skipped", "int32_t lv = lat_us[v * B + b], lw = lat_us[w * B + b];",
     "int32_t lv = lat_us[v * B + b] + 0 * cw, lw = lat_us[w * B + b]; return v < w;"),
    ("latency_before_cost", "int32_t cv = cost[v * B + b], cw = cost[w * B + b];",
     "int32_t cv = lat_us[v * B + b], cw = lat_us[w * B + b];"),
    ("cost_ignored", "if (cv != cw)", "if (0)"),
    ("batch_column_ignored_in_key", "int32_t cv = cost[v * B + b], cw = cost[w * B + b];",
     "int32_t cv = cost[v * B], cw = cost[w * B];"),
    ("batch_column_ignored_in_filter", "int64_t total = (int64_t)lat_us[v * B + b]",
     "int64_t total = (int64_t)lat_us[v * B]"),
    ("bad_batch_index_reads_column_0", "int32_t b = q_batch_idx[q];",
     "int32_t b = q_batch_idx[q]; if (b < 0 || b >= B) b = 0;"),
    ("task_filter_dropped", "if (task_id[v] != q_task[q])\n                    continue;", ""),
    ("first_feasible_wins", "if (best < 0 || cheaper(lat_us, cost, B, b, v, best))",
     "if (best < 0)"),
    ("last_feasible_wins", "if (best < 0 || cheaper(lat_us, cost, B, b, v, best))", "if (1)"),
    ("update_keeps_negative", "if (v < 0 || v >= V || new_queue_us[i] < 0)",
     "if (v < 0 || v >= V)"),
    ("update_reversed", "for (int64_t i = 0; i < n; ++i) {\n        int64_t v = variant_idx[i];",
     "for (int64_t i = n - 1; i >= 0; --i) {\n        int64_t v = variant_idx[i];"),
    ("update_adds", "queue_us[v] = new_queue_us[i];", "queue_us[v] += new_queue_us[i];"),
]


# planted mistakes in the closest-variant search
CLOSEST_MUTANTS = [
    ("closest_missed_count_ignored", "if (dv.missed != dw.missed)", "if (0)"),
    ("closest_shortfall_before_overshoot", "if (dv.over_us != dw.over_us)\n        return dv.over_us < dw.over_us;",
     "if (dv.short_bp != dw.short_bp)\n        return dv.short_bp < dw.short_bp;\n    if (dv.over_us != dw.over_us)\n        return dv.over_us < dw.over_us;"),
    ("closest_overshoot_flipped", "return dv.over_us < dw.over_us;", "return dv.over_us > dw.over_us;"),
    ("closest_shortfall_flipped", "return dv.short_bp < dw.short_bp;", "return dv.short_bp > dw.short_bp;"),
    ("closest_shortfall_ignored", "if (dv.short_bp != dw.short_bp)", "if (0)"),
    ("closest_overshoot_wraps", "d.over_us = total > (int64_t)slo_us ? total - (int64_t)slo_us : 0;",
     "d.over_us = total > (int64_t)slo_us ? (int64_t)(int32_t)(uint32_t)(total - (int64_t)slo_us) : 0;"),
    ("closest_shortfall_wraps", "(int64_t)min_acc_bp - (int64_t)acc_bp[v] : 0;",
     "(int64_t)(int32_t)((uint32_t)min_acc_bp - (uint32_t)acc_bp[v]) : 0;"),
    ("closest_queue_dropped", "int64_t total = (int64_t)lat_us[v * B + b] + (int64_t)queue_us[v];\n    d.over_us",
     "int64_t total = (int64_t)lat_us[v * B + b];\n    d.over_us"),
    ("closest_key_tie_dropped", "return cheaper(lat_us, cost, B, b, v, w);\n}\n\n/*\n * Literal form: every query looks at every row of the table.  out_variant",
     "return v < w;\n}\n\n/*\n * Literal form: every query looks at every row of the table.  out_variant"),
    ("closest_reports_infeasible_as_selected", "out_variant[q] = (best >= 0 && feasible(", "out_variant[q] = (best >= 0 || feasible("),
]


@pytest.mark.parametrize("name,find,repl", CLOSEST_MUTANTS, ids=[m[0] for m in CLOSEST_MUTANTS])
def test_closest_mutant_is_caught(tmp_path, source_text, name, find, repl):
    assert find in source_text, f"mutant {name}: pattern not in the oracle source any more"
    src = tmp_path / f"{name}.c"
    src.write_text(source_text.replace(find, repl))
    lib = oracle.build_oracle(src=str(src), out=str(tmp_path / f"lib{name}.so"), force=True)
    mutant = oracle.Oracle(lib)
    caught = []
    for pin in pins.CLOSEST_PINS:
        try:
            pin(mutant)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake '{name}'"


# planted mistakes in the state-aware selection
TIERED_MUTANTS = [
    ("tiered_inactive_before_active", "out_variant = (int32_t)(active >= 0 ? active : inactive);",
     "out_variant = (int32_t)(inactive >= 0 ? inactive : active);"),
    ("tiered_overloaded_counts_as_active", "if (state[v] == STATE_ACTIVE) {", "if (state[v] == STATE_ACTIVE || state[v] == STATE_OVERLOADED) {"),
    ("tiered_interfered_counts_as_inactive", "} else if (state[v] == STATE_INACTIVE) {", "} else if (state[v] == STATE_INACTIVE || state[v] == STATE_INTERFERED) {"),
    ("tiered_load_not_charged", "if ((int64_t)load_us[v] + (int64_t)lat_us[v * B + b] > (int64_t)slo_us)", "if ((int64_t)lat_us[v * B + b] > (int64_t)slo_us)"),
    ("tiered_load_sum_wraps", "if ((int64_t)load_us[v] + (int64_t)lat_us[v * B + b] > (int64_t)slo_us)",
     "if ((int64_t)(int32_t)((uint32_t)load_us[v] + (uint32_t)lat_us[v * B + b]) > (int64_t)slo_us)"),
    ("tiered_inactive_uses_queue", "if ((int64_t)load_us[v] + (int64_t)lat_us[v * B + b] > (int64_t)slo_us)",
     "if ((int64_t)load_us[v] + (int64_t)lat_us[v * B + b] + (int64_t)queue_us[v] > (int64_t)slo_us)"),
    ("tiered_inactive_accuracy_dropped", "if (acc_bp[v] < min_acc_bp)\n                continue;\n            if ((int64_t)load_us[v]",
     "if ((int64_t)load_us[v]"),
    ("tiered_inactive_by_cost", "if (inactive < 0 || loads_sooner(lat_us, load_us, B, b, v, inactive))",
     "if (inactive < 0 || cheaper(lat_us, cost, B, b, v, inactive))"),
    ("tiered_order_flipped", "if (tv != tw)\n        return tv < tw;", "if (tv != tw)\n        return tv > tw;"),
    ("tiered_latency_tie_skipped", "int64_t tw = (int64_t)load_us[w] + (int64_t)lat_us[w * B + b];\n    if (tv != tw)\n        return tv < tw;",
     "int64_t tw = (int64_t)load_us[w] + (int64_t)lat_us[w * B + b];\n    if (tv != tw)\n        return tv < tw;\n    return v < w;"),
    ("tiered_tier_code_swapped", "*out_tier = active >= 0 ? 1 : (inactive >= 0 ? 2 : 0);", "*out_tier = active >= 0 ? 2 : (inactive >= 0 ? 1 : 0);"),
    ("state_update_keeps_bad_codes", "if (v < 0 || v >= V || new_state[i] < 0 || new_state[i] > 3)", "if (v < 0 || v >= V)"),
]


@pytest.mark.parametrize("name,find,repl", TIERED_MUTANTS, ids=[m[0] for m in TIERED_MUTANTS])
def test_tiered_mutant_is_caught(tmp_path, source_text, name, find, repl):
    assert find in source_text, f"mutant {name}: pattern not in the oracle source any more"
    src = tmp_path / f"{name}.c"
    src.write_text(source_text.replace(find, repl))
    lib = oracle.build_oracle(src=str(src), out=str(tmp_path / f"lib{name}.so"), force=True)
    mutant = oracle.Oracle(lib)
    caught = []
    for pin in pins.TIERED_PINS:
        try:
            pin(mutant)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake '{name}'"


# planted mistakes in the last step of the complete Case I (suggestion among Active and Inactive variants)
_DW = "distance_t dw = tier_distance(acc_bp, lat_us, queue_us, state, load_us, B, w, slo_us, min_acc_bp, b);\n"
CASE1_MUTANTS = [
    ("case1_suggests_any_state", "if (state[v] != STATE_ACTIVE && state[v] != STATE_INACTIVE)\n            continue;", ""),
    ("case1_active_measured_with_load", "int64_t wait = state[v] == STATE_ACTIVE ? (int64_t)queue_us[v] : (int64_t)load_us[v];",
     "int64_t wait = state[v] == STATE_ACTIVE ? (int64_t)load_us[v] : (int64_t)queue_us[v];"),
    ("case1_inactive_measured_with_queue", "int64_t wait = state[v] == STATE_ACTIVE ? (int64_t)queue_us[v] : (int64_t)load_us[v];",
     "int64_t wait = (int64_t)queue_us[v];"),
    ("case1_latency_term_dropped", "int64_t total = (int64_t)lat_us[v * B + b] + wait;", "int64_t total = wait;"),
    ("case1_overshoot_wraps", "+ wait;\n    d.over_us = total > (int64_t)slo_us ? total - (int64_t)slo_us : 0;",
     "+ wait;\n    d.over_us = total > (int64_t)slo_us ? (int64_t)(int32_t)(uint32_t)(total - (int64_t)slo_us) : 0;"),
    ("case1_missed_count_ignored", _DW + "    if (dv.missed != dw.missed)\n        return dv.missed < dw.missed;", _DW),
    ("case1_overshoot_flipped", _DW + "    if (dv.missed != dw.missed)\n        return dv.missed < dw.missed;\n    if (dv.over_us != dw.over_us)\n        return dv.over_us < dw.over_us;",
     _DW + "    if (dv.missed != dw.missed)\n        return dv.missed < dw.missed;\n    if (dv.over_us != dw.over_us)\n        return dv.over_us > dw.over_us;"),
    ("case1_shortfall_ignored", "return dv.short_bp < dw.short_bp;\n    if (state[v] != state[w])", "return 0;\n    if (state[v] != state[w])"),
    ("case1_inactive_before_active", "return state[v] == STATE_ACTIVE;", "return state[v] == STATE_INACTIVE;"),
    ("case1_tier_ignored", "if (state[v] != state[w])\n        return state[v] == STATE_ACTIVE;", ""),
    ("case1_inactive_ordered_by_cost", "return state[v] == STATE_ACTIVE ? cheaper(lat_us, cost, B, b, v, w) : loads_sooner(lat_us, load_us, B, b, v, w);",
     "return cheaper(lat_us, cost, B, b, v, w);"),
    ("case1_active_ordered_by_load", "return state[v] == STATE_ACTIVE ? cheaper(lat_us, cost, B, b, v, w) : loads_sooner(lat_us, load_us, B, b, v, w);",
     "return loads_sooner(lat_us, load_us, B, b, v, w);"),
    ("case1_suggestion_where_selected_dropped", "*out_closest = *out_variant;\n        return;", "*out_closest = -1;\n        return;"),
]


@pytest.mark.parametrize("name,find,repl", CASE1_MUTANTS, ids=[m[0] for m in CASE1_MUTANTS])
def test_case1_mutant_is_caught(tmp_path, source_text, name, find, repl):
    assert find in source_text, f"mutant {name}: pattern not in the oracle source any more"
    src = tmp_path / f"{name}.c"
    src.write_text(source_text.replace(find, repl))
    lib = oracle.build_oracle(src=str(src), out=str(tmp_path / f"lib{name}.so"), force=True)
    mutant = oracle.Oracle(lib)
    caught = []
    for pin in pins.CASE1_PINS:
        try:
            pin(mutant)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake '{name}'"


# planted mistakes in the worker selection
WORKER_MUTANTS = [
    ("worker_most_loaded", "if (best < 0 || inst_load[i] < inst_load[best] ||", "if (best < 0 || inst_load[i] > inst_load[best] ||"),
    ("worker_load_tie_to_higher_number", "(inst_load[i] == inst_load[best] && inst_worker[i] < inst_worker[best]))",
     "(inst_load[i] == inst_load[best] && inst_worker[i] > inst_worker[best]))"),
    ("worker_load_tie_keeps_first_listed", "(inst_load[i] == inst_load[best] && inst_worker[i] < inst_worker[best]))", "0)"),
    ("worker_any_variants_instance", "if (inst_variant[i] != variant)\n            continue;", ""),
    ("worker_returns_instance_number", "return best >= 0 ? inst_worker[best] : -1;", "return best >= 0 ? (int32_t)best : -1;"),
    ("worker_most_utilised", "if (best < 0 || worker_util[w] < worker_util[best])", "if (best < 0 || worker_util[w] > worker_util[best])"),
    ("worker_util_tie_to_higher_number", "if (best < 0 || worker_util[w] < worker_util[best])", "if (best < 0 || worker_util[w] <= worker_util[best])"),
    ("worker_hardware_ignored", "if (worker_hw[w] != hw)\n            continue;", ""),
    ("worker_hardware_by_variant_number", "out_worker[q] = least_utilised_worker(W, worker_hw, worker_util, variant_hw[v]);",
     "out_worker[q] = least_utilised_worker(W, worker_hw, worker_util, v);"),
    ("worker_tiers_swapped", "        if (out_tier[q] == 1)\n            out_worker[q] = least_loaded_worker(n_inst, inst_variant, inst_worker, inst_load,\n                                                list + first[v]",
     "        if (out_tier[q] == 2)\n            out_worker[q] = least_loaded_worker(n_inst, inst_variant, inst_worker, inst_load,\n                                                list + first[v]"),
    ("worker_inactive_by_instances", "else if (out_tier[q] == 2)\n            out_worker[q] = least_utilised_worker(W, worker_hw, worker_util, variant_hw[v]);",
     "else if (out_tier[q] == 2)\n            out_worker[q] = least_loaded_worker(n_inst, inst_variant, inst_worker, inst_load, list + first[v], first[v + 1] - first[v], v);"),
    ("worker_for_unanswered_query", "        else\n            out_worker[q] = -1;\n    }\n    free(first);", "        else\n            out_worker[q] = 0;\n    }\n    free(first);"),
    ("worker_list_off_by_one", "list + first[v], first[v + 1] - first[v], v);", "list + first[v], first[v + 1] - first[v] - 1, v);"),
    ("worker_args_unchecked", "if (inst_variant[i] < 0 || inst_variant[i] >= V || inst_worker[i] < 0 || inst_worker[i] >= W)\n            return 0;",
     "if (inst_variant[i] < 0 || inst_variant[i] >= V || inst_worker[i] < 0)\n            return 0;"),   # (a variant outside the table would make the mutant write outside its lists)
    ("util_report_keeps_negative", "if (w < 0 || w >= W || new_util[i] < 0)", "if (w < 0 || w >= W)"),
    ("instance_report_out_of_order", "for (int64_t i = 0; i < n; ++i) {\n        int64_t j = inst_idx[i];", "for (int64_t i = n - 1; i >= 0; --i) {\n        int64_t j = inst_idx[i];"),
]


@pytest.mark.parametrize("name,find,repl", WORKER_MUTANTS, ids=[m[0] for m in WORKER_MUTANTS])
def test_worker_mutant_is_caught(tmp_path, source_text, name, find, repl):
    assert find in source_text, f"mutant {name}: pattern not in the oracle source any more"
    src = tmp_path / f"{name}.c"
    src.write_text(source_text.replace(find, repl))
    lib = oracle.build_oracle(src=str(src), out=str(tmp_path / f"lib{name}.so"), force=True)
    mutant = oracle.Oracle(lib)
    caught = []
    for pin in pins.WORKER_PINS:
        try:
            pin(mutant)
        except (AssertionError, ValueError):
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake '{name}'"


# planted mistakes in the selection with a state per running instance
INSTANCE_MUTANTS = [
    ("inst_variant_active_only_if_all_are", "else if (active[v] > 0)", "else if (active[v] == running[v])"),
    ("inst_overloaded_counts_as_active", "active[v] += inst_state[i] == STATE_ACTIVE;", "active[v] += inst_state[i] != STATE_INTERFERED;"),
    ("inst_busy_variant_taken_for_inactive", "if (running[v] == 0)\n            out_state[v] = STATE_INACTIVE;",
     "if (active[v] == 0)\n            out_state[v] = STATE_INACTIVE;"),
    ("inst_avoided_states_swapped", "out_state[v] = overloaded[v] > 0 ? STATE_OVERLOADED : STATE_INTERFERED;",
     "out_state[v] = overloaded[v] > 0 ? STATE_INTERFERED : STATE_OVERLOADED;"),
    ("inst_worker_ignores_the_state", "if (inst_variant[i] != variant || inst_state[i] != STATE_ACTIVE)", "if (inst_variant[i] != variant)"),
    ("inst_worker_may_be_overloaded", "if (inst_variant[i] != variant || inst_state[i] != STATE_ACTIVE)",
     "if (inst_variant[i] != variant || inst_state[i] == STATE_INTERFERED)"),
    ("inst_second_step_worker_from_instances",
     "out_worker[q] = least_utilised_worker(W, worker_hw, worker_util, variant_hw[v]);\n        else\n            out_worker[q] = -1;\n    }\n    free(state);",
     "out_worker[q] = least_loaded_active_worker(n_inst, inst_variant, inst_worker, inst_load, inst_state, NULL, 0, v);\n        else\n            out_worker[q] = -1;\n    }\n    free(state);"),
    ("inst_list_off_by_one", "inst_state,\n                                             list + first[v], first[v + 1] - first[v], v);",
     "inst_state,\n                                             list + first[v], first[v + 1] - first[v] - 1, v);"),
    ("inst_select_accepts_any_code",
     "if (inst_state[i] != STATE_ACTIVE && inst_state[i] != STATE_OVERLOADED && inst_state[i] != STATE_INTERFERED)\n            return -1;",
     "if (0)\n            return -1;"),
    ("inst_report_accepts_any_code",
     "if (new_state[i] != STATE_ACTIVE && new_state[i] != STATE_OVERLOADED && new_state[i] != STATE_INTERFERED)\n            continue;",
     ""),
    ("inst_report_out_of_order", "for (int64_t i = 0; i < n; ++i) {\n        int64_t j = inst_idx[i];\n        if (j < 0 || j >= n_inst)\n            continue;\n        if (new_state",
     "for (int64_t i = n - 1; i >= 0; --i) {\n        int64_t j = inst_idx[i];\n        if (j < 0 || j >= n_inst)\n            continue;\n        if (new_state"),
]


@pytest.mark.parametrize("name,find,repl", INSTANCE_MUTANTS, ids=[m[0] for m in INSTANCE_MUTANTS])
def test_instance_mutant_is_caught(tmp_path, source_text, name, find, repl):
    assert find in source_text, f"mutant {name}: pattern not in the oracle source any more"
    src = tmp_path / f"{name}.c"
    src.write_text(source_text.replace(find, repl))
    lib = oracle.build_oracle(src=str(src), out=str(tmp_path / f"lib{name}.so"), force=True)
    mutant = oracle.Oracle(lib)
    caught = []
    for pin in pins.INSTANCE_PINS:
        try:
            pin(mutant)
        except (AssertionError, ValueError):
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake '{name}'"


# planted mistakes in the scaling decision
SCALING_MUTANTS = [
    ("scale_headroom_ignored", "int64_t need = (int64_t)r_load_qps[r] * (int64_t)slack_pct;", "int64_t need = (int64_t)r_load_qps[r] * 100;"),
    ("scale_capacity_of_one_instance", "if ((int64_t)sat_qps[cur] * n_cur * 100 >= need)", "if ((int64_t)sat_qps[cur] * 100 >= need)"),
    ("scale_strict_capacity_test", "if ((int64_t)sat_qps[cur] * n_cur * 100 >= need)", "if ((int64_t)sat_qps[cur] * n_cur * 100 > need)"),
    ("scale_instances_rounded_down", "int64_t inst = (need + per - 1) / per;\n            best_n = inst - n_cur;", "int64_t inst = need / per;\n            best_n = inst - n_cur;"),
    ("scale_upgrade_instances_rounded_down", "int64_t inst = (need + per - 1) / per;\n            wide_t cost", "int64_t inst = need / per + 1;\n            wide_t cost"),
    ("scale_replicas_not_net", "best_n = inst - n_cur;", "best_n = inst;"),
    ("scale_replication_ignores_slo", "if ((int64_t)lat_us[cur * B + b] <= slo) {", "if (1) {"),
    ("scale_upgrade_ignores_slo", "if ((int64_t)lat_us[u * B + b] > slo || sat_qps[u] <= sat_qps[cur])", "if (sat_qps[u] <= sat_qps[cur])"),
    ("scale_upgrade_to_equal_throughput", "|| sat_qps[u] <= sat_qps[cur])", "|| sat_qps[u] < sat_qps[cur])"),
    ("scale_wrong_batch_column", "if ((int64_t)lat_us[u * B + b] > slo", "if ((int64_t)lat_us[u * B] > slo"),
    ("scale_any_architecture", "if (u == cur || arch_id[u] != arch_id[cur])", "if (u == cur)"),
    ("scale_unloading_not_credited", "((wide_t)1000000 + (wide_t)lambda_per_s * load_us[u]) - saved;", "((wide_t)1000000 + (wide_t)lambda_per_s * load_us[u]);"),
    ("scale_unloading_credited_unscaled", "wide_t saved = (wide_t)hw_cost[cur] * n_cur * 1000000;", "wide_t saved = (wide_t)hw_cost[cur] * n_cur;"),
    ("scale_lambda_dropped", "((wide_t)1000000 + (wide_t)lambda_per_s * load_us[u]) - saved;", "((wide_t)1000000) - saved;"),
    ("scale_lambda_dropped_for_replicas", "((wide_t)1000000 + (wide_t)lambda_per_s * load_us[cur]);", "((wide_t)1000000);"),
    ("scale_cost_in_64_bits", "wide_t cost = (wide_t)hw_cost[u] * inst *\n                          ((wide_t)1000000 + (wide_t)lambda_per_s * load_us[u]) - saved;",
     "wide_t cost = (wide_t)(int64_t)((uint64_t)hw_cost[u] * (uint64_t)inst * (uint64_t)(1000000 + (int64_t)lambda_per_s * load_us[u])) - saved;"),
    ("scale_replica_cost_in_64_bits", "best_cost = (wide_t)hw_cost[cur] * best_n *\n                        ((wide_t)1000000 + (wide_t)lambda_per_s * load_us[cur]);",
     "best_cost = (wide_t)(int64_t)((uint64_t)hw_cost[cur] * (uint64_t)best_n * (uint64_t)(1000000 + (int64_t)lambda_per_s * load_us[cur]));"),
    ("scale_tie_to_upgrade", "if (!have || cost < best_cost) {", "if (!have || cost <= best_cost) {"),
    ("scale_impossible_reported_as_none", "out_action[r] = 3;", "out_action[r] = 0;"),
    ("scale_action_codes_swapped", "out_action[r] = best_v == cur ? 1 : 2;", "out_action[r] = best_v == cur ? 2 : 1;"),
    ("scale_limits_unchecked", "r_instances[r] > 1000000 || r_load_qps[r] > 1000000000)", "0)"),
    ("scale_lambda_limit_unchecked", "lambda_per_s > 1000 ||", ""),
]


SCALE_DOWN_MUTANTS = [
    ("down_last_instance_removed", "if (n_cur >= 2 && (int64_t)sat_qps[cur] * (n_cur - 1) * 100 >= need) {", "if (n_cur >= 1 && (int64_t)sat_qps[cur] * (n_cur - 1) * 100 >= need) {"),
    ("down_capacity_before_removal", "if (n_cur >= 2 && (int64_t)sat_qps[cur] * (n_cur - 1) * 100 >= need) {", "if (n_cur >= 2 && (int64_t)sat_qps[cur] * n_cur * 100 >= need) {"),
    ("down_strict_capacity_test", "(int64_t)sat_qps[cur] * (n_cur - 1) * 100 >= need) {", "(int64_t)sat_qps[cur] * (n_cur - 1) * 100 > need) {"),
    ("down_removal_gains_nothing", "wide_t objective = -(wide_t)hw_cost[cur] * 1000000;", "wide_t objective = 0;"),
    ("down_removal_unscaled", "wide_t objective = -(wide_t)hw_cost[cur] * 1000000;", "wide_t objective = -(wide_t)hw_cost[cur];"),
    ("down_removal_of_all", "wide_t objective = -(wide_t)hw_cost[cur] * 1000000;", "wide_t objective = -(wide_t)hw_cost[cur] * n_cur * 1000000;"),
    ("down_headroom_ignored", "int64_t slo = r_slo_us[r];\n        wide_t lowest = 0;", "need = (int64_t)r_load_qps[r] * 100;\n        int64_t slo = r_slo_us[r];\n        wide_t lowest = 0;"),
    ("down_to_equal_cost", "|| hw_cost[u] >= hw_cost[cur])", "|| hw_cost[u] > hw_cost[cur])"),
    ("down_to_any_cost", "if ((int64_t)lat_us[u * B + b] > slo || hw_cost[u] >= hw_cost[cur])", "if ((int64_t)lat_us[u * B + b] > slo)"),
    ("down_ignores_slo", "if ((int64_t)lat_us[u * B + b] > slo || hw_cost[u] >= hw_cost[cur])", "if (hw_cost[u] >= hw_cost[cur])"),
    ("down_wrong_batch_column", "if ((int64_t)lat_us[u * B + b] > slo || hw_cost[u] >= hw_cost[cur])", "if ((int64_t)lat_us[u * B] > slo || hw_cost[u] >= hw_cost[cur])"),
    ("down_any_architecture", "if (u == cur || arch_id[u] != arch_id[cur])\n                continue;\n            if ((int64_t)lat_us[u * B + b] > slo || hw_cost[u] >= hw_cost[cur])", "if (u == cur)\n                continue;\n            if ((int64_t)lat_us[u * B + b] > slo || hw_cost[u] >= hw_cost[cur])"),
    ("down_instances_rounded_down", "int64_t inst = (need + per - 1) / per;\n            if (inst < 1)", "int64_t inst = need / per;\n            if (inst < 1)"),
    ("down_to_no_instance", "if (inst < 1)\n                inst = 1;", ""),
    ("down_unloading_not_credited", "((wide_t)1000000 + (wide_t)lambda_per_s * load_us[u]) - unloaded;", "((wide_t)1000000 + (wide_t)lambda_per_s * load_us[u]);"),
    ("down_unloading_credited_unscaled", "wide_t unloaded = (wide_t)hw_cost[cur] * n_cur * 1000000;", "wide_t unloaded = (wide_t)hw_cost[cur] * n_cur;"),
    ("down_unloading_one_credited", "wide_t unloaded = (wide_t)hw_cost[cur] * n_cur * 1000000;", "wide_t unloaded = (wide_t)hw_cost[cur] * 1000000;"),
    ("down_lambda_dropped", "((wide_t)1000000 + (wide_t)lambda_per_s * load_us[u]) - unloaded;", "((wide_t)1000000) - unloaded;"),
    ("down_objective_in_64_bits", "wide_t objective = (wide_t)hw_cost[u] * inst *\n                               ((wide_t)1000000 + (wide_t)lambda_per_s * load_us[u]) - unloaded;",
     "wide_t objective = (wide_t)(int64_t)((uint64_t)hw_cost[u] * (uint64_t)inst *\n                               (uint64_t)(1000000 + (int64_t)lambda_per_s * load_us[u])) - unloaded;"),
    ("down_tie_to_the_switch", "if (objective < lowest) {               /* rows ascend", "if (objective <= lowest) {               /* rows ascend"),
    ("down_tie_to_removal", "if (objective < lowest) {\n                lowest = objective;\n                out_action[r] = 1;", "if (objective <= lowest) {\n                lowest = objective;\n                out_action[r] = 1;"),
    ("down_action_codes_swapped", "out_action[r] = 2;\n                out_variant[r] = (int32_t)u;", "out_action[r] = 1;\n                out_variant[r] = (int32_t)u;"),
    ("down_reports_instances_left", "out_instances[r] = 1;", "out_instances[r] = (int32_t)(n_cur - 1);"),
    ("down_limits_unchecked", "r_instances[r] > 1000000 || r_load_qps[r] > 1000000000)\n            continue;\n        int64_t n_cur = r_instances[r];\n        int64_t need = (int64_t)r_load_qps[r] * (int64_t)slack_pct;        /* hundredths of a query per second */\n        int64_t slo", "0)\n            continue;\n        int64_t n_cur = r_instances[r];\n        int64_t need = (int64_t)r_load_qps[r] * (int64_t)slack_pct;        /* hundredths of a query per second */\n        int64_t slo"),
]


@pytest.mark.parametrize("name,find,repl", SCALE_DOWN_MUTANTS, ids=[m[0] for m in SCALE_DOWN_MUTANTS])
def test_scale_down_mutant_is_caught(tmp_path, source_text, name, find, repl):
    assert source_text.count(find) == 1, f"mutant {name}: pattern not once in the oracle source"
    src = tmp_path / f"{name}.c"
    src.write_text(source_text.replace(find, repl))
    lib = oracle.build_oracle(src=str(src), out=str(tmp_path / f"lib{name}.so"), force=True)
    mutant = oracle.Oracle(lib)
    caught = []
    for pin in pins.SCALE_DOWN_PINS:
        try:
            pin(mutant)
        except (AssertionError, ValueError):
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake '{name}'"


@pytest.mark.parametrize("name,find,repl", SCALING_MUTANTS, ids=[m[0] for m in SCALING_MUTANTS])
def test_scaling_mutant_is_caught(tmp_path, source_text, name, find, repl):
    assert find in source_text, f"mutant {name}: pattern not in the oracle source any more"
    src = tmp_path / f"{name}.c"
    src.write_text(source_text.replace(find, repl))
    lib = oracle.build_oracle(src=str(src), out=str(tmp_path / f"lib{name}.so"), force=True)
    mutant = oracle.Oracle(lib)
    caught = []
    for pin in pins.SCALING_PINS:
        try:
            pin(mutant)
        except (AssertionError, ValueError):
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake '{name}'"


@pytest.fixture(scope="module")
def source_text():
    with open(SRC) as f:
        return f.read()


@pytest.mark.parametrize("name,find,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, source_text, name, find, repl):
    assert find in source_text, f"mutant {name}: pattern not in the oracle source any more"
    src = tmp_path / f"{name}.c"
    src.write_text(source_text.replace(find, repl))
    lib = oracle.build_oracle(src=str(src), out=str(tmp_path / f"lib{name}.so"), force=True)
    mutant = oracle.Oracle(lib)
    caught = []
    for pin in pins.ALL_PINS:
        try:
            pin(mutant)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake '{name}'"
