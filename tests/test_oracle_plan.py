"""Pins for oracle/plan.py: every check here is against something the paper or plain arithmetic
fixes, never against the oracle's own formulas re-typed."""
import os

import numpy as np
import pytest

import workloads as W
from oracle import plan as OP

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(fname):
    out = []
    with open(os.path.join(GOLDEN, fname)) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                out.append(line.split())
    return out


# ----------------------------------------------------------------------------------------
# Eq. 10 / Eq. 11: cost model against the paper's printed example and fitted constants
# ----------------------------------------------------------------------------------------

def test_small_message_example_from_introduction():
    rows = _rows("allreduce_small_message_example.txt")
    (m1, t1), (m2, t2), (sep, mer) = [(float(x), float(y)) for x, y in rows]
    # the two printed points determine the line
    b = (t2 - t1) / (m2 - m1)
    a = t1 - b * m1
    assert a == pytest.approx(1.2e-3, rel=1e-9)
    assert b == pytest.approx(1.5e-9, rel=1e-9)
    assert OP.allreduce_time(a, b, int(m1)) == pytest.approx(t1, rel=1e-12)
    assert OP.allreduce_time(a, b, int(m2)) == pytest.approx(t2, rel=1e-12)
    # two separate 200 KB messages cost 3 ms, one merged 400 KB message 1.8 ms
    assert 2 * OP.allreduce_time(a, b, int(m1)) == pytest.approx(sep, rel=1e-12)
    assert OP.allreduce_time(a, b, int(m1) + int(m1)) == pytest.approx(mer, rel=1e-12)
    # Eq. 11: merging saves exactly one startup time
    assert sep - mer == pytest.approx(a, rel=1e-9)


def test_fitted_constants_are_linear_with_positive_intercept():
    for _, a, b, startup_us in _rows("fitted_allreduce_ab.txt"):
        a, b = float(a), float(b)
        assert OP.allreduce_time(a, b, 0) == a
        assert a * 1e6 == pytest.approx(float(startup_us), rel=1e-3)
        for m1, m2 in ((1024, 768), (4 * 25_500_000, 1024)):
            lhs = OP.allreduce_time(a, b, m1) + OP.allreduce_time(a, b, m2)
            rhs = OP.allreduce_time(a, b, m1 + m2)
            assert lhs > rhs                      # Eq. 11
            assert lhs - rhs == pytest.approx(a, rel=1e-6)


# ----------------------------------------------------------------------------------------
# Eq. 6-8 + Eq. 12-14: timeline evaluated by hand
# ----------------------------------------------------------------------------------------

HAND_BYTES = [0, 0, 100]
HAND_TB = [49.1, 0.9, 0.0]


def test_hand_timeline_three_layers():
    for *flags, t in _rows("hand_timeline_L3.txt"):
        m = [int(f) for f in flags]
        assert OP.iteration_time(m, HAND_BYTES, HAND_TB, 1.0, 1.0) == pytest.approx(float(t), abs=1e-12)


def test_tau_b_and_tau_c_of_hand_example():
    t_b = [None] + HAND_TB
    tau_b = OP.backward_start_times(t_b)
    assert tau_b[1:] == pytest.approx([0.9, 0.0, 0.0])
    tau_c = OP.comm_start_times([None, 1.0, 1.0, 101.0], t_b, tau_b)
    assert tau_c[1:] == pytest.approx([102.0, 101.0, 0.0])


def test_layer_one_cannot_be_merged():
    with pytest.raises(ValueError):
        OP.iteration_time([1, 0], [4, 4], [1.0, 1.0], 1.0, 1.0)


def test_two_layer_cases_by_hand():
    # L = 2, a = 10, b = 1/byte.  layer 2 ready at t_b2; layer 1 ready at t_b2 + t_b1.
    a, b = 10.0, 1.0
    # Case 1 (hidden): t_c2 = 10 + 5 = 15 <= t_b1 = 100.  normal: 3+100 + (10+7) = 120 ; merged: 103 + 10 + 12 = 125
    assert OP.iteration_time([0, 0], [7, 5], [100.0, 3.0], a, b) == pytest.approx(120.0)
    assert OP.iteration_time([0, 1], [7, 5], [100.0, 3.0], a, b) == pytest.approx(125.0)
    # Case 2 (partial overlap, wait 4 < a): normal: 3 + 15 + 17 = 35 ; merged: 3 + 4 + 22 = 29
    assert OP.iteration_time([0, 0], [7, 5], [4.0, 3.0], a, b) == pytest.approx(35.0)
    assert OP.iteration_time([0, 1], [7, 5], [4.0, 3.0], a, b) == pytest.approx(29.0)
    # Case 3 (partial overlap, wait 12 >= a): normal: 3 + 15 + 17 = 35 ; merged: 3 + 12 + 22 = 37
    assert OP.iteration_time([0, 0], [7, 5], [12.0, 3.0], a, b) == pytest.approx(35.0)
    assert OP.iteration_time([0, 1], [7, 5], [12.0, 3.0], a, b) == pytest.approx(37.0)
    # and Algorithm 1 takes the cheaper one each time
    assert OP.plan_algorithm1([7, 5], [100.0, 3.0], a, b) == [0, 0]
    assert OP.plan_algorithm1([7, 5], [4.0, 3.0], a, b) == [0, 1]
    assert OP.plan_algorithm1([7, 5], [12.0, 3.0], a, b) == [0, 0]
    # equality of the wait with a keeps the layer normal (Case 3 is ">=")
    assert OP.plan_algorithm1([7, 5], [10.0, 3.0], a, b) == [0, 0]


# ----------------------------------------------------------------------------------------
# closed forms for the two classical schedules
# ----------------------------------------------------------------------------------------

def _rand_instance(rng, L, **kw):
    p = W.make_random_profile(rng, L, **kw)
    return [int(x) for x in p.size_bytes], [float(x) for x in p.t_backward], p.a, p.b


def test_single_layer_closed_form():
    rng = np.random.default_rng(1)
    for _ in range(50):
        L = int(rng.integers(1, 30))
        by, tb, a, b = _rand_instance(rng, L)
        expect = sum(tb) + a + b * sum(by)                    # Eq. 9 with t_f = 0
        assert OP.single_layer_time(by, tb, a, b) == pytest.approx(expect, rel=1e-12)


def test_wfbp_closed_forms():
    rng = np.random.default_rng(2)
    for _ in range(50):
        L = int(rng.integers(2, 30))
        by = [int(x) for x in rng.integers(1, 1000, size=L)]
        # fully hidden: every backward step is longer than the message it has to hide
        a, b = 1e-6, 1e-9
        tb = [1.0] * L
        assert OP.wfbp_time(by, tb, a, b) == pytest.approx(sum(tb) + (a + b * by[0]), rel=1e-12)
        # communication bound: messages queue back to back after the first gradient
        a = 100.0
        expect = tb[-1] + sum(a + b * x for x in by)
        assert OP.wfbp_time(by, tb, a, b) == pytest.approx(expect, rel=1e-12)


def _group_timeline(groups, by, tb, a, b):
    """Written from the prose definition of a normal layer, not from Eq. 7: a group's single message
    starts once its last member's gradient exists and the previous message has ended."""
    L = len(by)
    ready = {}
    clock = 0.0
    for i in range(L - 1, -1, -1):
        clock += tb[i]
        ready[i] = clock
    end_prev = 0.0
    for members in groups:
        start = max(ready[min(members)], end_prev)
        end_prev = start + (a + b * sum(by[i] for i in members))
    return end_prev


def test_iteration_time_equals_group_level_timeline():
    rng = np.random.default_rng(3)
    for _ in range(300):
        L = int(rng.integers(1, 14))
        by, tb, a, b = _rand_instance(rng, L)
        m = [0] + [int(x) for x in rng.integers(0, 2, size=L - 1)]
        groups = OP.groups_in_arrival_order(m)
        assert OP.iteration_time(m, by, tb, a, b) == pytest.approx(_group_timeline(groups, by, tb, a, b),
                                                                   rel=1e-12)


# ----------------------------------------------------------------------------------------
# Algorithm 1: rule, limits, exhaustive search
# ----------------------------------------------------------------------------------------

def test_algorithm1_on_hand_example_and_theorem_gap():
    m = OP.plan_algorithm1(HAND_BYTES, HAND_TB, 1.0, 1.0)
    assert m == [0, 0, 1]
    t_greedy = OP.iteration_time(m, HAND_BYTES, HAND_TB, 1.0, 1.0)
    t_best, m_best = OP.bruteforce_best(HAND_BYTES, HAND_TB, 1.0, 1.0)
    assert t_greedy == pytest.approx(102.9)
    assert t_best == pytest.approx(102.0) and m_best == [0, 1, 0]
    # the plan is a single-flip local optimum only: Theorem 1's optimality claim does not hold here
    assert t_best < t_greedy < OP.wfbp_time(HAND_BYTES, HAND_TB, 1.0, 1.0)


def test_algorithm1_followed_by_hand_on_four_layers():
    """The message time of a layer that received merged bytes must be re-derived: two levels further down
    the decision depends on it."""
    *flags, t = _rows("hand_plan_L4.txt")[0]
    by, tb = [1, 1, 1, 100], [3.0, 5.0, 0.5, 0.0]
    m = OP.plan_algorithm1(by, tb, 1.0, 1.0)
    assert m == [int(f) for f in flags]
    assert OP.iteration_time(m, by, tb, 1.0, 1.0) == pytest.approx(float(t))


def test_each_decision_matches_the_layer_type_rule():
    """Layer l is merged iff tau_b^(l-1) + t_b^(l-1) < tau_c^(l) + a, with tau_c^(l) taken from the
    timeline in which the decisions for layers above l are already applied and layers <= l normal."""
    rng = np.random.default_rng(4)
    for _ in range(200):
        L = int(rng.integers(2, 25))
        by, tb, a, b = _rand_instance(rng, L)
        m = OP.plan_algorithm1(by, tb, a, b)
        t_b1 = [None] + tb
        tau_b = OP.backward_start_times(t_b1)
        for l in range(L, 1, -1):
            partial = [0] * L
            for j in range(l + 1, L + 1):
                partial[j - 1] = m[j - 1]
            p = [None] + list(by)
            for j in range(L, 1, -1):
                if partial[j - 1]:
                    p[j - 1] += p[j]
            t_c = [None] + [0.0 if partial[j - 1] else OP.allreduce_time(a, b, p[j]) for j in range(1, L + 1)]
            tau_c = OP.comm_start_times(t_c, t_b1, tau_b)
            assert bool(m[l - 1]) == OP.merge_rule_holds(l, tau_b, t_b1, tau_c, a)


def test_limit_large_startup_gives_one_group():
    rng = np.random.default_rng(5)
    for _ in range(30):
        L = int(rng.integers(1, 40))
        by, tb, _, b = _rand_instance(rng, L)
        a = 1.001 * sum(tb) + 1e-9
        assert OP.plan_algorithm1(by, tb, a, b) == [0] + [1] * (L - 1)


def test_limit_hidden_messages_with_long_gaps_gives_wfbp():
    rng = np.random.default_rng(6)
    for _ in range(30):
        L = int(rng.integers(1, 40))
        by = [int(x) for x in rng.integers(1, 10_000, size=L)]
        a, b = 1e-4, 1e-9
        # every backward step is at least twice the longest possible single message, and > a
        tb = [float(x) for x in rng.uniform(2.0, 3.0, size=L) * (a + b * 10_000)]
        assert OP.plan_algorithm1(by, tb, a, b) == [0] * L


def test_zero_cost_model_keeps_every_layer_normal():
    rng = np.random.default_rng(7)
    by, tb, _, _ = _rand_instance(rng, 20)
    assert OP.plan_algorithm1(by, tb, 0.0, 0.0) == [0] * 20
    assert OP.plan_algorithm1([5], [1.0], 1.0, 1.0) == [0]
    assert OP.plan_algorithm1([], [], 1.0, 1.0) == []


def test_all_plans_enumerates_two_to_the_L_minus_one():
    for L in range(1, 9):
        plans = [tuple(m) for m in OP.all_plans(L)]
        assert len(plans) == len(set(plans)) == 2 ** (L - 1)
        assert all(m[0] == 0 for m in plans)


def test_bruteforce_invariants_and_suboptimality_rate(capsys):
    rng = np.random.default_rng(8)
    trials, subopt, worst = 250, 0, 0.0
    for _ in range(trials):
        L = int(rng.integers(2, 11))
        by, tb, a, b = _rand_instance(rng, L)
        m = OP.plan_algorithm1(by, tb, a, b)
        t_g = OP.iteration_time(m, by, tb, a, b)
        t_best, _ = OP.bruteforce_best(by, tb, a, b)
        t_w = OP.wfbp_time(by, tb, a, b)
        t_s = OP.single_layer_time(by, tb, a, b)
        tol = 1e-12 * max(t_w, t_s)
        assert t_best <= t_g + tol                    # nothing beats the exhaustive optimum
        assert t_best <= min(t_w, t_s) + tol          # WFBP and single-buffer are never better than it
        assert t_g <= t_w + tol                       # an accepted merge never delays the last message
        if t_g > t_best * (1 + 1e-9):
            subopt += 1
            worst = max(worst, t_g / t_best - 1)
    with capsys.disabled():
        print(f"\n[oracle] Algorithm 1 sub-optimal on {subopt}/{trials} random instances (L<=10), "
              f"worst gap {100 * worst:.2f}%")


def test_accepted_merge_lowers_end_of_lower_layers_message():
    """Lemma 1's content: when the rule fires for l (layers below still normal) the message of layer
    l-1 ends earlier with l merged than with l normal."""
    rng = np.random.default_rng(9)
    for _ in range(200):
        by, tb, a, b = _rand_instance(rng, 2)
        t_n = OP.iteration_time([0, 0], by, tb, a, b)
        t_m = OP.iteration_time([0, 1], by, tb, a, b)
        m = OP.plan_algorithm1(by, tb, a, b)
        assert (m == [0, 1]) == (t_m < t_n)


def test_toy_profile_plan_is_the_exhaustive_optimum():
    p = W.make_profile("toy_mlp")
    by = [int(x) for x in p.size_bytes]
    tb = [float(x) for x in p.t_backward]
    m = OP.plan_algorithm1(by, tb, p.a, p.b)
    t_best, _ = OP.bruteforce_best(by, tb, p.a, p.b)
    assert sum(1 for _ in OP.all_plans(p.L)) == 128
    assert OP.iteration_time(m, by, tb, p.a, p.b) == pytest.approx(t_best, rel=1e-12)


def test_plan_is_deterministic():
    p = W.make_profile("tiny_layers")
    by = [int(x) for x in p.size_bytes][:200]
    tb = [float(x) for x in p.t_backward][:200]
    assert OP.plan_algorithm1(by, tb, p.a, p.b) == OP.plan_algorithm1(list(by), list(tb), p.a, p.b)


# ----------------------------------------------------------------------------------------
# grouping (Algorithm 2) and buffer layout (Sec. 5.3)
# ----------------------------------------------------------------------------------------

def test_groups_worked_example():
    # layers 1..6; layers 6 and 5 merged down into 4, layer 3 alone, layer 2 merged into 1
    m = [0, 1, 0, 0, 1, 1]
    assert OP.groups_in_arrival_order(m) == [[5, 4, 3], [2], [1, 0]]
    tg, off, ge = OP.merge_layout([10, 20, 30, 40, 50, 60], m)
    assert tg == [2, 2, 1, 0, 0, 0]
    assert off == [20, 0, 0, 110, 60, 0]
    assert ge == [150, 30, 30]


def test_group_ready_times_by_hand_and_against_a_running_sum():
    """Pins: (1) the hand timeline of tests/golden/hand_timeline_L3.txt (Eq. 6: gradients of layers 3, 2, 1 exist
    at 0, 0.9 and 50); (2) with every layer normal the ready times are the running sum of the backward times in
    arrival order, which numpy.cumsum forms with the same sequence of binary64 additions; (3) any plan's ready
    times are that sequence picked at the normal layers, and the last one is the whole backward pass."""
    t_b = [49.1, 0.9, 0.0]
    assert OP.group_ready_times([0, 0, 0], t_b) == [0.0, 0.9, 50.0]
    assert OP.group_ready_times([0, 0, 1], t_b) == [0.9, 50.0]          # layers {3,2} then {1}
    assert OP.group_ready_times([0, 1, 0], t_b) == [0.0, 50.0]          # {3} then {2,1}
    assert OP.group_ready_times([0, 1, 1], t_b) == [50.0]
    # the six-layer worked example: groups {6,5,4}, {3}, {2,1} close at layers 4, 3, 1
    t6 = [1.0, 2.0, 4.0, 8.0, 16.0, 32.0]
    assert OP.group_ready_times([0, 1, 0, 0, 1, 1], t6) == [32.0 + 16.0 + 8.0, 60.0, 63.0]
    rng = np.random.default_rng(77)
    for _ in range(100):
        L = int(rng.integers(1, 80))
        t = rng.uniform(0.0, 1e-3, size=L)
        running = np.cumsum(t[::-1])                                       # arrival order: layer L first
        assert OP.group_ready_times([0] * L, t) == running.tolist()
        m = [0] + [int(x) for x in rng.integers(0, 2, size=L - 1)]
        ready = OP.group_ready_times(m, t)
        normal_layers_in_arrival_order = [i for i in range(L - 1, -1, -1) if m[i] == 0]
        assert ready == [running[L - 1 - i] for i in normal_layers_in_arrival_order]
        assert ready[-1] == running[-1]
        assert all(x <= y for x, y in zip(ready, ready[1:]))
    assert OP.group_ready_times([], []) == []


def test_group_and_layout_invariants():
    rng = np.random.default_rng(10)
    for _ in range(100):
        L = int(rng.integers(1, 60))
        n = [int(x) for x in rng.integers(0, 500, size=L)]
        m = [0] + [int(x) for x in rng.integers(0, 2, size=L - 1)]
        groups = OP.groups_in_arrival_order(m)
        flat = [i for g in groups for i in g]
        assert flat == list(range(L - 1, -1, -1))             # contiguous, each layer exactly once
        assert len(groups) == L - sum(m)
        for g in groups:
            assert m[g[-1]] == 0 and all(m[i] == 1 for i in g[:-1])
        tg, off, ge = OP.merge_layout(n, m)
        assert sum(ge) == sum(n)                              # buffers total the model size (Sec. 5.3)
        for k, g in enumerate(groups):
            assert ge[k] == sum(n[i] for i in g)
            pos = 0
            for i in g:
                assert tg[i] == k and off[i] == pos
                pos += n[i]


def test_profiles_match_table_4_and_config_sizes():
    table = {r[0]: (int(r[1]), float(r[2])) for r in _rows("dnn_table.txt")}
    p = W.make_profile("resnet50")
    assert p.L == table["ResNet-50"][0]
    assert p.total_elems / 1e6 == pytest.approx(table["ResNet-50"][1], abs=0.1)
    assert p.total_elems == 25_557_032
    assert p.total_elems * 4 / 1e6 == pytest.approx(102, abs=0.5)     # "all-reduce 102 MB" (Sec. 1)
    assert W.make_profile("vgg16").total_elems == 138_357_544
    assert W.make_profile("vgg16").L == 32
    t = W.make_profile("transformer")
    assert (t.L, t.total_elems) == (391, 335_141_888)
    assert W.make_profile("toy_mlp").total_elems == 300_938
    c3 = W.make_profile("tiny_layers")
    assert c3.L == 1000 and 16 <= int(c3.n_elems.min()) and int(c3.n_elems.max()) <= 262144


@pytest.mark.parametrize("name", W.PROFILE_NAMES)
def test_plans_of_the_five_profiles_are_valid_and_no_worse_than_wfbp(name):
    p = W.make_profile(name)
    by = [int(x) for x in p.size_bytes]
    tb = [float(x) for x in p.t_backward]
    m = OP.plan_algorithm1(by, tb, p.a, p.b)
    assert m[0] == 0 and len(m) == p.L
    t = OP.iteration_time(m, by, tb, p.a, p.b)
    assert t <= OP.wfbp_time(by, tb, p.a, p.b) * (1 + 1e-12)
    assert t >= sum(tb)                                       # cannot end before backpropagation does


# ----------------------------------------------------------------------------------------
# exact optimum (dynamic programme) against its definition: the exhaustive minimum
# ----------------------------------------------------------------------------------------

def test_plan_optimal_equals_exhaustive_minimum():
    rng = np.random.default_rng(20)
    for trial in range(400):
        L = int(rng.integers(1, 13))
        by, tb, a, b = _rand_instance(rng, L, size_hi=10 ** 6 if trial % 2 else 5000, allow_empty=True)
        t_dp, m_dp = OP.plan_optimal(by, tb, a, b)
        t_bf, _ = OP.bruteforce_best(by, tb, a, b)
        assert t_dp == t_bf                                         # same operations, same bits
        assert m_dp[0] == 0
        assert OP.iteration_time(m_dp, by, tb, a, b) == t_dp        # the returned plan attains it


@pytest.mark.parametrize("L", [14, 15, 16])
def test_exhaustive_search_up_to_sixteen_layers(L):
    """All 2^(L-1) plans at the largest sizes the exhaustive check is asked for: the dynamic programme attains
    the minimum bit for bit, Algorithm 1 is never better than it and never worse than wait-free
    backpropagation, and neither baseline beats the minimum."""
    rng = np.random.default_rng(300 + L)
    for trial in range(2):
        by, tb, a, b = _rand_instance(rng, L, size_hi=10 ** 6 if trial else 5000)
        t_bf, m_bf = OP.bruteforce_best(by, tb, a, b)
        assert sum(1 for _ in OP.all_plans(L)) == 2 ** (L - 1)
        t_dp, m_dp = OP.plan_optimal(by, tb, a, b)
        assert t_dp == t_bf and OP.iteration_time(m_dp, by, tb, a, b) == t_bf
        t_g = OP.iteration_time(OP.plan_algorithm1(by, tb, a, b), by, tb, a, b)
        t_w, t_s = OP.wfbp_time(by, tb, a, b), OP.single_layer_time(by, tb, a, b)
        tol = 1e-12 * max(t_w, t_s)
        assert t_bf <= t_g + tol and t_g <= t_w + tol and t_bf <= min(t_w, t_s) + tol
        groups = OP.groups_in_arrival_order(m_bf)                     # contiguous, cover every layer once
        assert [i for g in groups for i in g] == list(range(L - 1, -1, -1))


def test_plan_optimal_on_hand_example_and_wide_ranges():
    t, m = OP.plan_optimal(HAND_BYTES, HAND_TB, 1.0, 1.0)
    assert m == [0, 1, 0] and t == pytest.approx(102.0)
    # tie: zero startup and zero slope make every plan end with the backward pass; longest groups win
    t, m = OP.plan_optimal([4, 4, 4], [1.0, 2.0, 3.0], 0.0, 0.0)
    assert t == 6.0 and m == [0, 1, 1]
    rng = np.random.default_rng(21)
    worse = 0
    for _ in range(200):
        L = int(rng.integers(2, 40))
        by, tb, a, b = _rand_instance(rng, L)
        t_opt, m_opt = OP.plan_optimal(by, tb, a, b)
        t_g = OP.iteration_time(OP.plan_algorithm1(by, tb, a, b), by, tb, a, b)
        assert t_opt <= t_g and t_opt <= OP.wfbp_time(by, tb, a, b) and t_opt <= OP.single_layer_time(by, tb, a, b)
        assert t_opt >= sum(tb)
        worse += t_g > t_opt
    assert worse > 0          # Algorithm 1 really is beaten on some instances
