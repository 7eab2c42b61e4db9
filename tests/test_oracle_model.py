"""Pins for oracle/model.py (Table 2, the (a, b) fit, the worker-count sweep of Sec. 6.4)."""
import os

import numpy as np
import pytest

import workloads as W
from oracle import model as OM
from oracle import plan as OP

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ALGOS = (OM.BINARY_TREE, OM.RECURSIVE_DOUBLING, OM.HALVING_DOUBLING, OM.DOUBLE_BINARY_TREES, OM.RING)


def test_table2_single_worker_costs_nothing_to_start():
    for algo in ALGOS:
        a, b = OM.allreduce_ab(algo, 1, 1e-5, 1e-9, 1e-10)
        assert a == 0.0
    assert OM.allreduce_ab(OM.RING, 1, 1e-5, 1e-9, 1e-10) == (0.0, 0.0)
    assert OM.allreduce_ab(OM.BINARY_TREE, 1, 1e-5, 1e-9, 1e-10) == (0.0, 0.0)


def test_table2_two_workers_by_hand():
    al, be, ga = 3.0, 5.0, 7.0
    assert OM.allreduce_ab(OM.BINARY_TREE, 2, al, be, ga) == (6.0, 17.0)            # 2a log2, (2b+g) log2
    assert OM.allreduce_ab(OM.RECURSIVE_DOUBLING, 2, al, be, ga) == (3.0, 12.0)
    assert OM.allreduce_ab(OM.DOUBLE_BINARY_TREES, 2, al, be, ga) == (6.0, 12.0)
    # with two workers the ring and halving/doubling are the same exchange of half messages
    assert OM.allreduce_ab(OM.RING, 2, al, be, ga) == (6.0, 8.5)
    assert OM.allreduce_ab(OM.HALVING_DOUBLING, 2, al, be, ga) == (6.0, 8.5)


def test_table2_entries_for_eight_and_large_N():
    al, be, ga = 2.0, 4.0, 1.0
    assert OM.allreduce_ab(OM.RING, 8, al, be, ga) == (28.0, 2 * 7 / 8 * 4.0 + 7 / 8 * 1.0)
    assert OM.allreduce_ab(OM.BINARY_TREE, 8, al, be, ga) == (12.0, 27.0)
    assert OM.allreduce_ab(OM.RECURSIVE_DOUBLING, 8, al, be, ga) == (6.0, 15.0)
    assert OM.allreduce_ab(OM.HALVING_DOUBLING, 8, al, be, ga) == (12.0, 8.0 - 9.0 / 8 + 1.0)
    # bandwidth-optimal algorithms approach 2*beta + gamma per byte; the ring's startup grows linearly
    a, b = OM.allreduce_ab(OM.RING, 2 ** 20, al, be, ga)
    assert b == pytest.approx(2 * be + ga, rel=1e-5) and a == pytest.approx(2 * al * 2 ** 20, rel=1e-5)
    _, b = OM.allreduce_ab(OM.HALVING_DOUBLING, 2 ** 20, al, be, ga)
    assert b == pytest.approx(2 * be + ga, rel=1e-5)
    # the ring's startup overhead quoted for cluster 1 (972 us) is 2(N-1) alpha
    a, _ = OM.allreduce_ab(OM.RING, 8, 972e-6 / 14, 0.0, 0.0)
    assert a == pytest.approx(972e-6)


def test_fit_recovers_lines_and_the_papers_example():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "allreduce_small_message_example.txt"))
            if l.strip() and not l.startswith("#")]
    a, b = OM.fit_ab([float(rows[0][0]), float(rows[1][0])], [float(rows[0][1]), float(rows[1][1])])
    assert a == pytest.approx(1.2e-3, rel=1e-9) and b == pytest.approx(1.5e-9, rel=1e-9)
    for line in open(os.path.join(GOLDEN, "fitted_allreduce_ab.txt")):
        if line.startswith("#") or not line.strip():
            continue
        _, a0, b0, _ = line.split()
        a0, b0 = float(a0), float(b0)
        sizes = [2 ** k for k in range(10, 28)]
        times = [OP.allreduce_time(a0, b0, s) for s in sizes]
        a, b = OM.fit_ab(sizes, times)
        assert a == pytest.approx(a0, rel=1e-8) and b == pytest.approx(b0, rel=1e-8)
    # noisy points: the fit is the least-squares minimiser (gradient of the squared error vanishes)
    rng = np.random.default_rng(0)
    M = rng.uniform(1e3, 1e8, 50)
    T = 2e-4 + 5e-10 * M + rng.normal(0, 1e-5, 50)
    a, b = OM.fit_ab(M, T)
    r = T - (a + b * M)
    assert abs(r.sum()) < 1e-9 and abs((r * M).sum()) < 1e-3


def test_simulation_reproduces_the_qualitative_claims_of_section_6_4():
    p = W.make_profile("resnet50")
    by = [int(x) for x in p.size_bytes]
    tb = [float(x) for x in p.t_backward]
    counts = [2 ** k for k in range(2, 12)]
    # ring over a slow network: alpha = 70 us, 10 Gb/s
    ring = OM.simulate(by, tb, 0.05, OM.RING, 70e-6, 8e-10, 1e-11, counts)
    groups = [r["groups"] for r in ring]
    assert all(g1 >= g2 for g1, g2 in zip(groups, groups[1:]))            # fewer and fewer messages
    assert groups[-1] == 1                                                  # converges to single-layer communication
    assert ring[-1]["t_mgwfbp"] == ring[-1]["t_single"]
    assert ring[0]["t_wfbp"] < ring[0]["t_single"] and ring[-1]["t_wfbp"] > ring[-1]["t_single"]   # the curves cross
    for r in ring:
        assert r["t_mgwfbp"] <= min(r["t_wfbp"], r["t_single"]) * (1 + 1e-12)
        assert r["speedup_mgwfbp"] <= r["N"] * (1 + 1e-12)
    # double binary trees with a small point-to-point latency: the startup grows only logarithmically, so
    # WFBP and MG-WFBP stay ahead of single-layer communication even at 2048 workers
    tree = OM.simulate(by, tb, 0.05, OM.DOUBLE_BINARY_TREES, 10e-6, 8e-10, 1e-11, [128, 256, 512, 1024, 2048])
    for r in tree:
        assert r["t_mgwfbp"] <= r["t_wfbp"] <= r["t_single"]
        assert r["groups"] > 1
