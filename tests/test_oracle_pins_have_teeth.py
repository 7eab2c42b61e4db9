"""Each plausible slip planted in a copy of the oracle (on the CPU, never in the library) must be caught by
at least one of the pins in test_oracle_plan.py / test_oracle_pipeline.py / test_oracle_model.py."""
import contextlib
import inspect
import textwrap

import pytest

import test_oracle_model as TM
import test_oracle_pipeline as TD
import test_oracle_plan as TP
from oracle import model as OM
from oracle import pipeline as OD
from oracle import plan as OP

PLAN_PINS = [TP.test_small_message_example_from_introduction, TP.test_hand_timeline_three_layers,
             TP.test_tau_b_and_tau_c_of_hand_example, TP.test_two_layer_cases_by_hand, TP.test_single_layer_closed_form,
             TP.test_wfbp_closed_forms, TP.test_iteration_time_equals_group_level_timeline,
             TP.test_algorithm1_on_hand_example_and_theorem_gap, TP.test_algorithm1_followed_by_hand_on_four_layers,
             TP.test_each_decision_matches_the_layer_type_rule,
             TP.test_limit_large_startup_gives_one_group, TP.test_groups_worked_example,
             TP.test_group_and_layout_invariants, TP.test_group_ready_times_by_hand_and_against_a_running_sum,
             TP.test_plan_optimal_equals_exhaustive_minimum,
             TP.test_plan_optimal_on_hand_example_and_wide_ranges]
DATA_PINS = [TD.test_widen_bf16_known_patterns_and_against_torch, TD.test_reduce_bf16_inputs_accumulate_in_binary32,
             TD.test_widen_f16_against_the_definition_of_binary16_for_every_pattern,
             TD.test_reduce_f16_inputs_accumulate_in_binary32,
             TD.test_pack_worked_example, TD.test_pack_round_trip_and_buffer_size, TD.test_reduce_order_is_left_to_right,
             TD.test_reduce_small_integers_are_exact, TD.test_reduce_identical_copies_returns_input,
             TD.test_reduce_replayed_in_binary64_with_explicit_rounding, TD.test_reduce_non_power_of_two_uses_reciprocal_multiply,
             TD.test_update_replayed_in_binary64_with_explicit_rounding, TD.test_update_differs_from_a_fused_multiply_add,
             TD.test_momentum_zero_reduces_to_plain_sgd, TD.test_merged_step_tiny_case_by_hand,
             TD.test_arrival_driven_pack_equals_whole_group_pack]
MODEL_PINS = [TM.test_table2_two_workers_by_hand, TM.test_table2_entries_for_eight_and_large_N,
              TM.test_fit_recovers_lines_and_the_papers_example,
              TM.test_simulation_reproduces_the_qualitative_claims_of_section_6_4]


@contextlib.contextmanager
def planted(module, func, old, new):
    """Re-define module.func with `old` replaced by `new` in its source, for the duration of the block."""
    original = getattr(module, func)
    src = textwrap.dedent(inspect.getsource(original))
    assert src.count(old) >= 1, f"{func}: pattern {old!r} not found"
    scope = module.__dict__
    exec(compile(src.replace(old, new), f"<mutant of {func}>", "exec"), scope)
    try:
        yield
    finally:
        setattr(module, func, original)


def caught_by(pins):
    hits = []
    for pin in pins:
        try:
            pin()
        except AssertionError:
            hits.append(pin.__name__)
        except Exception as exc:          # a crash also exposes the slip
            hits.append(f"{pin.__name__} ({type(exc).__name__})")
    return hits


PLAN_MUTANTS = [
    ("allreduce_time", "a + b * float(message_bytes)", "a - b * float(message_bytes)"),
    ("allreduce_time", "a + b * float(message_bytes)", "b * float(message_bytes)"),
    ("backward_start_times", "tau_b[l + 1] + t_b1[l + 1]", "tau_b[l + 1] + t_b1[l]"),
    ("comm_start_times", "max(tau_c[l + 1] + t_c1[l + 1], tau_b1[l] + t_b1[l])", "max(tau_c[l + 1], tau_b1[l] + t_b1[l])"),
    ("comm_start_times", "max(tau_c[l + 1] + t_c1[l + 1], tau_b1[l] + t_b1[l])", "min(tau_c[l + 1] + t_c1[l + 1], tau_b1[l] + t_b1[l])"),
    ("comm_start_times", "tau_c[L] = tau_b1[L] + t_b1[L]", "tau_c[L] = tau_b1[L]"),
    ("timeline", "p[l - 1] = p[l - 1] + p[l]", "p[l - 1] = p[l - 1]"),
    ("timeline", "p[l - 1] = p[l - 1] + p[l]", "p[l - 1] = p[l]"),
    ("iteration_time", "return tau_c[1] + t_c[1]", "return tau_c[1]"),
    ("timeline", "0.0 if m[l] == MERGED else", "allreduce_time(a, b, 0) if m[l] == MERGED else"),
    ("timeline", "for l in range(L, 1, -1):", "for l in range(2, L + 1):"),
    ("plan_algorithm1", "- tau_c[l] < a", "- tau_c[l] <= a"),
    ("plan_algorithm1", "- tau_c[l] < a", "- tau_c[l] > a"),
    ("plan_algorithm1", "tau_b[l - 1] + t_b[l - 1] - tau_c[l] < a", "tau_b[l] + t_b[l] - tau_c[l] < a"),
    ("plan_algorithm1", "tau_b[l - 1] + t_b[l - 1] - tau_c[l] < a", "tau_b[l - 1] + t_b[l - 1] - tau_c[l - 1] < a"),
    ("plan_algorithm1", "timeline(m, size_bytes", "timeline([NORMAL] * L, size_bytes"),
    ("plan_algorithm1", "m[l - 1] = MERGED", "m[l - 2] = MERGED"),
    ("plan_algorithm1", "for l in range(L, 1, -1):", "for l in range(2, L + 1):"),
    ("plan_optimal", "start = F[i] if F[i] > ready[k] else ready[k]", "start = ready[k]"),
    ("plan_optimal", "prefix[k] - prefix[i]", "prefix[k] - prefix[i - 1]"),
    ("groups_in_arrival_order", "for l in range(L, 0, -1):", "for l in range(1, L + 1):"),
    ("groups_in_arrival_order", "if merged[l - 1] == NORMAL:", "if merged[l - 1] == MERGED:"),
    ("merge_layout", "tensor_off[i] = fill", "tensor_off[i] = fill + int(n_elems[i])"),
    ("group_ready_times", "l = members[-1] + 1", "l = members[0] + 1"),
    ("group_ready_times", "ready.append(tau_b[l] + t_b1[l])", "ready.append(tau_b[l])"),
]

DATA_MUTANTS = [
    ("pack", "buf[fill:fill + n] = grads[i]", "buf[total - fill - n:total - fill] = grads[i]"),
    ("reduce_average", "for g in range(1, P):", "for g in range(P - 1, 0, -1):"),
    ("reduce_average", "np.float32(1.0) / np.float32(P)", "np.float32(1.0) / np.float32(P + 1)"),
    ("reduce_average", "return np.multiply(acc, inv, dtype=np.float32)", "return np.divide(acc, np.float32(P), dtype=np.float32) if P == 3 else np.multiply(acc, inv, dtype=np.float32)"),
    ("reduce_average", "acc = np.add(acc, as_f32(worker_buffers[g]), dtype=np.float32)",
     "acc = np.add(acc.astype(np.float64), as_f32(worker_buffers[g]).astype(np.float64))"),
    ("sgd_momentum", "w[...] = np.subtract(w, t2, dtype=np.float32)", "w[...] = np.add(w, t2, dtype=np.float32)"),
    ("sgd_momentum", "t1 = np.multiply(v, mu, dtype=np.float32)\n    v[...] = np.add(t1, g, dtype=np.float32)",
     "v[...] = (v.astype(np.float64) * np.float64(mu) + g.astype(np.float64)).astype(np.float32)"),
    ("sgd_momentum", "v[...] = np.add(t1, g, dtype=np.float32)", "v[...] = np.add(t1, np.multiply(g, eta), dtype=np.float32)"),
    ("sgd_momentum", "t2 = np.multiply(v, eta, dtype=np.float32)", "t2 = np.multiply(g, eta, dtype=np.float32)"),
    ("widen_bf16", "<< np.uint32(16)", "<< np.uint32(15)"),
    ("widen_f16", "x.astype(np.float32)", "x.view(np.uint16).astype(np.float32)"),
    ("as_f32", "return widen_f16(x)", "return widen_bf16(x.view(np.uint16))"),
    ("pack_as_gradients_arrive", "if merged[l - 1] == 0:", "if merged[l - 1] == 1 or l == 1:"),
]

MODEL_MUTANTS = [
    ("allreduce_ab", "return 2.0 * (N - 1) * alpha, (2.0 * (N - 1) / N) * beta + ((N - 1) / N) * gamma",
     "return 2.0 * N * alpha, (2.0 * (N - 1) / N) * beta + ((N - 1) / N) * gamma"),
    ("allreduce_ab", "2.0 * beta - (1.0 / N) * (2.0 * beta + gamma) + gamma", "2.0 * beta + (1.0 / N) * (2.0 * beta + gamma) + gamma"),
    ("allreduce_ab", "return alpha * lg, (beta + gamma) * lg", "return alpha * lg, (beta + gamma)"),
    ("fit_ab", "return float(a), float(b)", "return float(b), float(a)"),
    ("simulate", "t_s = t_forward + OP.single_layer_time", "t_s = OP.single_layer_time"),
]


@pytest.mark.parametrize("func,old,new", PLAN_MUTANTS)
def test_planted_slip_in_plan_oracle_is_caught(func, old, new):
    with planted(OP, func, old, new):
        assert caught_by(PLAN_PINS), f"no pin notices {func}: {old!r} -> {new!r}"
    assert not caught_by(PLAN_PINS[:4])          # and the untouched oracle is clean again


@pytest.mark.parametrize("func,old,new", DATA_MUTANTS)
def test_planted_slip_in_pipeline_oracle_is_caught(func, old, new):
    with planted(OD, func, old, new):
        assert caught_by(DATA_PINS), f"no pin notices {func}: {old!r} -> {new!r}"


@pytest.mark.parametrize("func,old,new", MODEL_MUTANTS)
def test_planted_slip_in_model_oracle_is_caught(func, old, new):
    with planted(OM, func, old, new):
        assert caught_by(MODEL_PINS), f"no pin notices {func}: {old!r} -> {new!r}"
