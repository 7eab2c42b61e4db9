"""Cost-model helpers of the library against the oracle (Table 2, the (a, b) fit, the worker-count sweep)."""
import numpy as np
import pytest

import paper_1912_09268_amd as M
import workloads as W
from oracle import model as OM


def test_allreduce_ab_matches_table2_oracle():
    rng = np.random.default_rng(0)
    for algo in range(5):
        for N in (1, 2, 3, 4, 8, 16, 64, 1000, 2048):
            al, be, ga = (float(10 ** rng.uniform(-7, -3)), float(10 ** rng.uniform(-11, -8)),
                          float(10 ** rng.uniform(-12, -9)))
            a, b = M.allreduce_ab(algo, N, al, be, ga)
            a0, b0 = OM.allreduce_ab(algo, N, al, be, ga)
            # the same handful of binary64 operations; allow the last bit of log2 / association
            assert a == pytest.approx(a0, rel=1e-15, abs=0) and b == pytest.approx(b0, rel=4e-16, abs=0)
    assert M.allreduce_ab(M.AR_RING, 2, 3.0, 5.0, 7.0) == (6.0, 8.5)
    assert M.allreduce_ab(M.AR_HALVING_DOUBLING, 2, 3.0, 5.0, 7.0) == (6.0, 8.5)
    for bad in ((9, 4, 1.0, 1.0, 1.0), (0, 0, 1.0, 1.0, 1.0), (0, 4, -1.0, 1.0, 1.0), (0, 4, 1.0, float("nan"), 1.0)):
        with pytest.raises(M.MgwfbpError):
            M.allreduce_ab(*bad)


def test_fit_ab_matches_oracle_and_the_papers_example():
    a, b = M.fit_ab([200000, 400000], [1.5e-3, 1.8e-3])
    assert a == pytest.approx(1.2e-3, rel=1e-12) and b == pytest.approx(1.5e-9, rel=1e-12)
    rng = np.random.default_rng(1)
    for _ in range(50):
        n = int(rng.integers(2, 40))
        sizes = np.unique(np.rint(10 ** rng.uniform(3, 9, n)).astype(np.uint64))
        if sizes.size < 2:
            continue
        a0, b0 = float(10 ** rng.uniform(-5, -3)), float(10 ** rng.uniform(-11, -9))
        times = a0 + b0 * sizes.astype(np.float64) * (1 + rng.normal(0, 0.02, sizes.size))
        a, b = M.fit_ab(sizes, times)
        ar, br = OM.fit_ab(sizes.astype(np.float64), times)
        # two different solvers of the same 2x2 least-squares problem: agreement far below the noise
        assert b == pytest.approx(br, rel=1e-9)
        assert a == pytest.approx(ar, rel=1e-7, abs=1e-12)
    with pytest.raises(M.MgwfbpError):
        M.fit_ab([5, 5], [1.0, 2.0])
    with pytest.raises(M.MgwfbpError):
        M.fit_ab([5], [1.0])


@pytest.mark.parametrize("algo", [OM.RING, OM.DOUBLE_BINARY_TREES, OM.HALVING_DOUBLING])
def test_simulate_matches_oracle(algo):
    p = W.make_profile("resnet50")
    by = [int(x) for x in p.size_bytes]
    tb = [float(x) for x in p.t_backward]
    counts = [2 ** k for k in range(2, 12)]
    tw, ts, tm, g = M.simulate(p.size_bytes, p.t_backward, 0.05, algo, 70e-6, 8e-10, 1e-11, counts)
    ref = OM.simulate(by, tb, 0.05, algo, 70e-6, 8e-10, 1e-11, counts)
    for k, r in enumerate(ref):
        a, b = M.allreduce_ab(algo, counts[k], 70e-6, 8e-10, 1e-11)
        if (a, b) == (r["a"], r["b"]):          # identical cost model -> identical bits
            assert (tw[k], ts[k], tm[k], g[k]) == (r["t_wfbp"], r["t_single"], r["t_mgwfbp"], r["groups"])
        else:
            assert tw[k] == pytest.approx(r["t_wfbp"], rel=1e-12) and tm[k] == pytest.approx(r["t_mgwfbp"], rel=1e-12)
    if algo == OM.RING:
        assert g[-1] == 1 and all(x >= y for x, y in zip(g, g[1:]))
