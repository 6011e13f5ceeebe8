"""The pins have teeth: a plausible mistake planted in a COPY of the oracle fails one of them.

Each case copies the oracle's sources to a temporary directory, rewrites one expression of
the dynamic program, of the strategy enumerator, of a table builder or of the pipeline
reduction (a transposed operand, a dropped term, a tie broken the other way, an off-by-one
in the fit test, ...), compiles the copy with gcc and runs the pin functions of
`test_oracle_pins`, `test_oracle_tables` and `test_oracle_pipeline` against it.  At least one pin must fail for every mutant, and none for the
unmodified copy.  Everything here runs on the CPU; the real oracle is never touched.
"""
import importlib.util
import os
import shutil

import pytest

import test_oracle_pins as pins
import test_oracle_pipeline as pipeline_pins
import test_oracle_tables as table_pins

ORACLE_DIR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")

# (name, source file, text in it, replacement); every text occurs exactly once, and every
# mutant still indexes within its arrays (it computes something wrong, it does not crash)
DP, PIPE = "gsearch_oracle.c", "pipeline_oracle.c"
MUTANTS = [(n, DP, a, b) for n, a, b in [
    ("inner_tie_takes_the_last_index",
     "if (v < best) { best = v; arg = i; }", "if (v <= best) { best = v; arg = i; }"),
    ("transition_table_transposed",
     "src[i] + Rl[(size_t)i * S + j]", "src[i] + Rl[(size_t)j * S + i]"),
    ("layer_time_dropped",
     "Cl[(size_t)e * S + j] = best + T[(size_t)l * S + j];", "Cl[(size_t)e * S + j] = best;"),
    ("transition_index_ignored",
     "bp + plane * (size_t)l;\n        const float *Rl = R + (size_t)r_index[l] * S * S;",
     "bp + plane * (size_t)l;\n        const float *Rl = R;"),
    ("fit_test_off_by_one",
     "if (e < o) {", "if (e <= o) {"),
    ("first_layer_fit_test_off_by_one",
     "(e >= O[s]) ? T[s] : INFINITY", "(e > O[s]) ? T[s] : INFINITY"),
    ("first_layer_time_of_the_wrong_strategy",
     "(e >= O[s]) ? T[s] : INFINITY", "(e >= O[s]) ? T[S - 1 - s] : INFINITY"),
    ("memory_of_the_layer_not_deducted",
     "Cp + (size_t)(e - o) * S;", "Cp + (size_t)e * S;"),
    ("final_tie_takes_the_last_index",
     "if (v < bc) { bc = v; bs = s; }", "if (v <= bc && v < INFINITY) { bc = v; bs = s; }"),
    ("backtrace_keeps_the_budget",
     "                e -= o;\n", ""),
    ("backtrace_forgets_the_first_layer_memory",
     "            used += O[s];\n", ""),
    ("batch_tie_takes_the_last_instance",
     "if (best_cost[b] < gbest) { gbest = best_cost[b]; garg = b; }",
     "if (best_cost[b] <= gbest && best_cost[b] < INFINITY) { gbest = best_cost[b]; garg = b; }"),
    ("batch_winner_is_the_costliest_instance",
     "if (best_cost[b] < gbest) { gbest = best_cost[b]; garg = b; }",
     "if (garg < 0 || (best_cost[b] > gbest && best_cost[b] < INFINITY)) { gbest = best_cost[b]; garg = b; }"),
    ("batch_reads_the_first_instance_tables",
     "T + off, O + off, R, r_index + (size_t)b * L,", "T, O, R, r_index,"),
    ("curve_is_a_maximum",
     "if (v < m) m = v;", "if (!(v < m) && v < INFINITY) m = v;"),
    # strategy enumerator and the two table builders
    ("sharding_over_a_single_replica_kept",
     "if (sdp == 1 && dp == 1) continue;", ""),
    ("tensor_and_sequence_degrees_swapped",
     "d[0] = tp; d[1] = sp;", "d[0] = sp; d[1] = tp;"),
    ("combined_degree_cap_ignored",
     "if (tpsp_max > 0 && tp * sp > tpsp_max) continue;", ""),
    ("recomputation_costs_no_time",
     "if (ckpt) { flops = flops * 4.0; flops = flops / 3.0; }", ""),
    ("tensor_parallel_volume_not_scaled",
     "x = x * h;\n                    x = x * (tp - 1.0);", "x = x * h;\n                    x = x * tp;"),
    ("sharded_gradients_cost_the_same",
     "if (sdp) x = x * 1.5;", ""),
    ("sequence_parallel_term_dropped",
     "x = x / sp;\n                    comm = comm + x;", "x = x / sp;"),
    ("recomputation_keeps_every_activation",
     "if (ckpt) act = act * keep;", ""),
    ("states_sharded_without_being_asked",
     "const double shard = sdp ? dp : 1.0;", "const double shard = dp;"),
    ("bins_rounded_down",
     "const double bins = ceil((state + act) / bin);", "const double bins = floor((state + act) / bin);"),
    ("transition_volume_of_the_source_layout",
     "x = x * (n / gj);", "x = x * (n / gi);"),
    ("transition_weights_swapped",
     "(a[0] == c[0]) ? 1.0 : 0.5;", "(a[0] == c[0]) ? 0.5 : 1.0;"),
    ("transition_keeps_the_larger_share",
     "keepfrac = keepfrac / hi;", "keepfrac = keepfrac / lo;"),
    ("profiled_bins_rounded_down",
     "const double bins = ceil((state + a) / bin);", "const double bins = floor((state + a) / bin);"),
    ("profiled_overlap_hides_nothing",
     "ms = ms + (1.0 - overlap) * dpc;", "ms = ms + dpc;"),
    ("profiled_bandwidth_of_the_wrong_group",
     "dpc = v / bw[gd];", "dpc = v / bw[gt];"),
    ("profiled_state_factor_dropped",
     "double state = sf * param;", "double state = param;"),
]] + [(n, PIPE, a, b) for n, a, b in [
    ("bubble_counts_every_micro_batch",
     "(float)(group_micro[g] - 1) * mx;", "(float)group_micro[g] * mx;"),
    ("bubble_of_the_last_stage",
     "if (t > mx) mx = t;", "mx = t;"),
    ("infeasible_member_ignored",
     "|| isinf(stage_cost[b])) { ok = 0; break; }", ") { ok = 0; break; }"),
    ("candidate_tie_takes_the_last",
     "if (cost < best) { best = cost; arg = g; }", "if (cost <= best && cost < INFINITY) { best = cost; arg = g; }"),
]]


def pin_calls(mod):
    calls = [(pins.test_hand_worked_example, (mod, n))
             for n in ("worked_example_a.txt", "worked_example_b.txt")]
    calls += [(pins.test_exhaustive_enumeration, (mod, i)) for i in (False, True)]
    calls += [(f, (mod,)) for f in (
        pins.test_budget_monotonicity_and_infeasibility,
        pins.test_zero_transition_is_multiple_choice_knapsack,
        pins.test_state_graph_shortest_path_scipy,
        pins.test_unconstrained_budget_is_viterbi_chain,
        pins.test_single_strategy_is_running_sum_and_single_layer_is_min,
        pins.test_tie_break_is_lowest_index_everywhere,
        pins.test_batch_wrapper_global_min,
        table_pins.test_enumerator_caps_give_the_benchmark_shapes,
        table_pins.test_table_builder_exact_on_power_of_two_inputs,
        table_pins.test_table_builder_scales_and_clamps,
        table_pins.test_profiled_table_builder_exact_on_power_of_two_inputs,
        pipeline_pins.test_hand_values_and_rules,
        pipeline_pins.test_against_independent_evaluation)]
    calls += [(table_pins.test_enumerator_closed_form_uncapped, (mod, k)) for k in range(8)]
    return calls


def build_copy(tmp_path, name, source, old, new):
    dst = tmp_path / f"oracle_copy_{name}"
    dst.mkdir()
    for f in os.listdir(ORACLE_DIR):
        if f.endswith(".c") or f == "__init__.py":
            shutil.copy(os.path.join(ORACLE_DIR, f), dst / f)
    if old is not None:
        src = dst / source
        text = src.read_text()
        assert text.count(old) == 1, f"mutation site of {name} not found exactly once"
        src.write_text(text.replace(old, new))
    spec = importlib.util.spec_from_file_location(f"oracle_copy_{name}", dst / "__init__.py")
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod.build(force=True)
    return mod


def failing_pins(mod):
    failed = []
    for f, args in pin_calls(mod):
        try:
            f(*args)
        except AssertionError:
            failed.append(f.__name__)
    return failed


def test_the_unmodified_copy_passes_every_pin(tmp_path):
    assert failing_pins(build_copy(tmp_path, "plain", None, None, None)) == []


@pytest.mark.parametrize("name,source,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(tmp_path, name, source, old, new):
    failed = failing_pins(build_copy(tmp_path, name, source, old, new))
    assert failed, f"no pin notices the mutant {name}"
