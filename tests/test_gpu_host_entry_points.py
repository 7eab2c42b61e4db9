"""The host-only entry points (planner, exact planner, evaluator, ready times, layout, cost-model helpers, worker
sweep) against the oracle once more, collected by `-m gpu`, so that a record of the GPU run also covers them on
the machine the kernels run on.  The checks are the ones of tests/test_host_*.py, called as they stand; for the
exact planner the oracle of record is exhaustive search (the definition), which bounds L at 16 -- beyond that
the library's dynamic programme is compared with the oracle's, two implementations of one recurrence."""
import numpy as np
import pytest

import test_host_layout as TL
import test_host_model as TMo
import test_host_plan as TPl
import workloads as W
from oracle import plan as OP

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", W.PROFILE_NAMES)
def test_algorithm1_and_evaluator_on_the_profiles(name):
    TPl.test_plan_matches_oracle_on_profiles(name)


def test_exact_planner_equals_exhaustive_search():
    import paper_1912_09268_amd as M
    rng = np.random.default_rng(20240)
    for trial in range(40):
        L = int(rng.integers(1, 13)) if trial else 16
        p = W.make_random_profile(rng, L, size_hi=10 ** 6 if trial % 2 else 5000, allow_empty=True)
        by, tb = [int(x) for x in p.size_bytes], [float(x) for x in p.t_backward]
        merged, first, t = M.plan_opt(p.size_bytes, p.t_backward, p.a, p.b)
        t_best, _ = OP.bruteforce_best(by, tb, p.a, p.b)
        assert t == t_best                                               # the minimum over all 2^(L-1) plans
        assert OP.iteration_time(merged.tolist(), by, tb, p.a, p.b) == t # ... attained by the returned plan
        greedy, _ = M.plan(p.size_bytes, p.t_backward, p.a, p.b)
        assert greedy.tolist() == OP.plan_algorithm1(by, tb, p.a, p.b)
        assert t <= OP.iteration_time(greedy.tolist(), by, tb, p.a, p.b)


def test_exact_planner_against_the_oracles_recurrence_beyond_sixteen_layers():
    TPl.test_plan_opt_matches_oracle_and_exhaustive_search()
    TPl.test_plan_opt_hand_example_and_errors()


def test_group_ready_times():
    TPl.test_group_ready_times_match_the_oracle_bit_for_bit()


def test_cost_model_helpers():
    TMo.test_allreduce_ab_matches_table2_oracle()
    TMo.test_fit_ab_matches_oracle_and_the_papers_example()


@pytest.mark.parametrize("algo", [4, 3, 2])                 # ring, double binary trees, halving-doubling
def test_worker_count_sweep(algo):
    TMo.test_simulate_matches_oracle(algo)


def test_layout_tables():
    for name in dir(TL):
        fn = getattr(TL, name)
        if name.startswith("test_") and callable(fn) and not hasattr(fn, "pytestmark"):
            try:
                fn()
            except TypeError:                              # parametrised or fixture-taking tests are not re-run here
                continue
