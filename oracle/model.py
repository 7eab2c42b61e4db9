"""Oracle for the cost-model helpers around the planner.  TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

  allreduce_ab      Table 2: startup a and per-byte cost b of five all-reduce algorithms from the
                    point-to-point latency alpha, per-byte time beta, per-byte summation time gamma and
                    the number of workers N (logarithms are base 2; the paper assumes N a power of two).
                    Reading: the table's "double binary trees" startup is printed as `2 log N` without
                    alpha; it is taken as 2*alpha*log N, like every other entry.
  fit_ab            Sec. 6.2 / Fig. 4: a and b are obtained by fitting the line a + b*M to measured
                    all-reduce times; ordinary least squares via numpy.polyfit.
  simulate          Sec. 6.4: iteration times of WFBP (every layer normal), single-layer communication
                    (everything merged, Eq. 9) and MG-WFBP (Algorithm 1) for a list of worker counts, with
                    (a, b) taken from Table 2 for each count; speedup over one worker is
                    N * (t_f + sum t_b) / t_iter (Eq. 4 with the overlapped iteration time).

Pins: tests/test_oracle_model.py (N = 1 and N = 2 identities between the algorithms, textbook limits,
exact recovery of lines, the 200 KB / 400 KB example of Sec. 1, the qualitative statements of Sec. 6.4).
The curves and group counts the paper prints need its measured traces: parity unpinned for those.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np

from . import plan as OP

BINARY_TREE, RECURSIVE_DOUBLING, HALVING_DOUBLING, DOUBLE_BINARY_TREES, RING = range(5)


def allreduce_ab(algorithm: int, N: int, alpha: float, beta: float, gamma: float) -> Tuple[float, float]:
    """(a, b) of Table 2."""
    if N < 1:
        raise ValueError("N >= 1")
    lg = math.log2(N)
    if algorithm == BINARY_TREE:
        return 2.0 * alpha * lg, (2.0 * beta + gamma) * lg
    if algorithm == RECURSIVE_DOUBLING:
        return alpha * lg, (beta + gamma) * lg
    if algorithm == HALVING_DOUBLING:
        return 2.0 * alpha * lg, 2.0 * beta - (1.0 / N) * (2.0 * beta + gamma) + gamma
    if algorithm == DOUBLE_BINARY_TREES:
        return 2.0 * alpha * lg, beta + gamma
    if algorithm == RING:
        return 2.0 * (N - 1) * alpha, (2.0 * (N - 1) / N) * beta + ((N - 1) / N) * gamma
    raise ValueError("unknown all-reduce algorithm")


def fit_ab(message_bytes: Sequence[float], seconds: Sequence[float]) -> Tuple[float, float]:
    """Least-squares line through (M, T): returns (a, b) with T ~ a + b*M."""
    b, a = np.polyfit(np.asarray(message_bytes, np.float64), np.asarray(seconds, np.float64), 1)
    return float(a), float(b)


def simulate(size_bytes: Sequence[int], t_backward: Sequence[float], t_forward: float, algorithm: int,
             alpha: float, beta: float, gamma: float, worker_counts: Sequence[int]) -> List[dict]:
    """One record per worker count: a, b, the three iteration times (forward time included), their
    speedups over a single worker, and the number of messages MG-WFBP sends."""
    out = []
    compute = t_forward + sum(float(x) for x in t_backward)
    for N in worker_counts:
        a, b = allreduce_ab(algorithm, N, alpha, beta, gamma)
        m = OP.plan_algorithm1(size_bytes, t_backward, a, b)
        t_w = t_forward + OP.wfbp_time(size_bytes, t_backward, a, b)
        t_s = t_forward + OP.single_layer_time(size_bytes, t_backward, a, b)
        t_m = t_forward + OP.iteration_time(m, size_bytes, t_backward, a, b)
        out.append({"N": N, "a": a, "b": b, "t_wfbp": t_w, "t_single": t_s, "t_mgwfbp": t_m,
                    "groups": len(m) - sum(m),
                    "speedup_wfbp": N * compute / t_w, "speedup_single": N * compute / t_s,
                    "speedup_mgwfbp": N * compute / t_m})
    return out
