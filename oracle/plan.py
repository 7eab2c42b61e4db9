"""Oracle for the planning half of MG-WFBP.  TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Everything is written in the paper's notation with 1-based layer numbers: layer 1 is the input
side, layer L the output side; backpropagation visits L, L-1, ..., 1.  Internally lists carry an
unused slot 0 so that `x[l]` reads like the paper's x^(l).  Public functions take and return
0-based sequences in forward order (position i holds layer l = i + 1).

All times are Python floats (IEEE binary64), one rounding per written operation, evaluated in the
order the paper writes them.  Message sizes are exact Python integers (bytes).

Readings taken where the paper leaves a choice:
  * b multiplies BYTES (Eq. 10 defines M in bytes); Algorithm 1's `b x p[l]` is read with p[l]
    expressed in bytes.
  * tau_b^(L) = 0, as Algorithm 1 initialises it (Eq. 6 has t_f there; a constant shift).
  * The merge test is the one Algorithm 1 spells out, `tau_b[l-1] + t_b[l-1] - tau_c[l] < a`,
    evaluated left to right, strict; equality keeps the layer normal (Case 3 uses ">=").
  * Layer 1 can never be merged (first property of a merged-gradient layer), so there are
    2^(L-1) candidate plans, not 2^L.
  * Inside a merge buffer tensors lie in arrival order (layer L-side first), densely (Sec. 5.3
    sizes the buffer as the plain sum of the member sizes).

Parity pins live in tests/test_oracle_plan.py (hand-evaluated timelines, closed forms for the
all-normal and all-merged plans, the paper's 200 KB / 400 KB example, exhaustive search,
limit cases, a group-level timeline simulation written independently of Eq. 7; group ready times
against the hand timeline and a library running sum).
The group counts the paper prints for its simulated clusters (Sec. 6.4) need backward-time traces
that are not available: parity unpinned for those.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

NORMAL = 0   # l_n
MERGED = 1   # l_m


# ------------------------------------------------------------------------------------------
# Eq. 10: all-reduce cost model
# ------------------------------------------------------------------------------------------

def allreduce_time(a: float, b: float, message_bytes: int) -> float:
    """T_ar(M) = a + b x M  (Eq. 10)."""
    return a + b * float(message_bytes)


# ------------------------------------------------------------------------------------------
# Eq. 6 / Eq. 7: the wait-free backpropagation timeline
# ------------------------------------------------------------------------------------------

def _one_based(seq: Sequence) -> list:
    return [None] + list(seq)


def backward_start_times(t_b1: list) -> list:
    """tau_b^(l) for l = 1..L with tau_b^(L) = 0 (Eq. 6, Algorithm 1 initialisation)."""
    L = len(t_b1) - 1
    tau_b = [None] * (L + 1)
    tau_b[L] = 0.0
    for l in range(L - 1, 0, -1):
        tau_b[l] = tau_b[l + 1] + t_b1[l + 1]
    return tau_b


def comm_start_times(t_c1: list, t_b1: list, tau_b1: list) -> list:
    """tau_c^(l) for l = 1..L (Eq. 7; procedure CalculateCommStart of Algorithm 1).

    Layer L may communicate once its own gradient exists; any lower layer needs both its own
    gradient and the end of the communication scheduled just before it."""
    L = len(t_b1) - 1
    tau_c = [None] * (L + 1)
    tau_c[L] = tau_b1[L] + t_b1[L]
    for l in range(L - 1, 0, -1):
        tau_c[l] = max(tau_c[l + 1] + t_c1[l + 1], tau_b1[l] + t_b1[l])
    return tau_c


# ------------------------------------------------------------------------------------------
# Eq. 8 with the merge properties Eq. 12-14: iteration time of a given plan
# ------------------------------------------------------------------------------------------

def timeline(merged: Sequence[int], size_bytes: Sequence[int], t_backward: Sequence[float],
             a: float, b: float) -> Tuple[list, list, list]:
    """The wait-free backpropagation timeline of the plan `merged` (0-based flags, merged[i] = 1 iff layer i+1
    is a merged-gradient layer): 1-based lists (tau_b, tau_c, t_c).

    A merged layer has no communication of its own (Eq. 12: t_c = 0) and hands its bytes to the layer below
    (Eq. 13); every other layer's message takes a + b x bytes (Eq. 10); backward passes start by Eq. 6 and
    communications by Eq. 7, which for the layer below a merged one is Eq. 14."""
    L = len(size_bytes)
    m = _one_based(merged)
    p = _one_based(int(x) for x in size_bytes)
    t_b = _one_based(float(x) for x in t_backward)
    for l in range(L, 1, -1):
        if m[l] == MERGED:
            p[l - 1] = p[l - 1] + p[l]
    t_c = [None] * (L + 1)
    for l in range(1, L + 1):
        t_c[l] = 0.0 if m[l] == MERGED else allreduce_time(a, b, p[l])
    tau_b = backward_start_times(t_b)
    tau_c = comm_start_times(t_c, t_b, tau_b)
    return tau_b, tau_c, t_c


def iteration_time(merged: Sequence[int], size_bytes: Sequence[int], t_backward: Sequence[float],
                   a: float, b: float) -> float:
    """t_iter - t_f for the plan `merged`: the iteration ends when layer 1's message ends (Eq. 8)."""
    if len(size_bytes) == 0:
        return 0.0
    if merged[0]:
        raise ValueError("layer 1 cannot be a merged-gradient layer")
    _, tau_c, t_c = timeline(merged, size_bytes, t_backward, a, b)
    return tau_c[1] + t_c[1]


def wfbp_time(size_bytes, t_backward, a, b) -> float:
    """Every layer normal: plain wait-free backpropagation."""
    return iteration_time([NORMAL] * len(size_bytes), size_bytes, t_backward, a, b)


def single_layer_time(size_bytes, t_backward, a, b) -> float:
    """Layers L..2 all merged: one message after the whole backward pass (single-layer S-SGD, Eq. 9)."""
    L = len(size_bytes)
    return iteration_time([NORMAL] + [MERGED] * (L - 1), size_bytes, t_backward, a, b)


# ------------------------------------------------------------------------------------------
# Algorithm 1
# ------------------------------------------------------------------------------------------

def plan_algorithm1(size_bytes: Sequence[int], t_backward: Sequence[float], a: float, b: float
                    ) -> List[int]:
    """The plan Algorithm 1 finds, stated through the definitions it rests on (O(L^2)).

    Layers are decided from L down to 2, every layer below the one under decision still normal.  Layer l
    becomes a merged-gradient layer iff, on the timeline of the plan decided so far (Eq. 6 and Eq. 7 under
    Eq. 12-14), the gradient of layer l-1 exists less than `a` after layer l could start to communicate:
    tau_b^(l-1) + t_b^(l-1) - tau_c^(l) < a, the layer-type rule of Lemma 1 / Theorem 1 in the form in which
    Algorithm 1 evaluates it (left to right, strict).  Layer 1 is always normal.

    Returns merged[0..L-1]; merged[0] is always 0."""
    L = len(size_bytes)
    t_b = _one_based(float(x) for x in t_backward)
    m = [NORMAL] * L                                  # m[l - 1] is the type of layer l
    for l in range(L, 1, -1):
        tau_b, tau_c, _ = timeline(m, size_bytes, t_backward, a, b)
        if tau_b[l - 1] + t_b[l - 1] - tau_c[l] < a:
            m[l - 1] = MERGED
    return m


def merge_rule_holds(l: int, tau_b1: list, t_b1: list, tau_c1: list, a: float) -> bool:
    """Lemma 1 / Theorem 1's layer-type rule in its printed form: tau_b^(l-1)+t_b^(l-1) < tau_c^(l)+a."""
    return tau_b1[l - 1] + t_b1[l - 1] < tau_c1[l] + a


# ------------------------------------------------------------------------------------------
# exhaustive search over the 2^(L-1) plans
# ------------------------------------------------------------------------------------------

def all_plans(L: int):
    """Every plan with layer 1 normal, as 0-based flag lists."""
    if L == 0:
        return
    for code in range(1 << (L - 1)):
        yield [NORMAL] + [(code >> (i - 1)) & 1 for i in range(1, L)]


def bruteforce_best(size_bytes, t_backward, a, b) -> Tuple[float, List[int]]:
    """Minimum iteration time over all plans, and one plan attaining it (first in enumeration order)."""
    L = len(size_bytes)
    if L > 20:
        raise ValueError("exhaustive search is meant for small L")
    best_t = None
    best_m = None
    for m in all_plans(L):
        t = iteration_time(m, size_bytes, t_backward, a, b)
        if best_t is None or t < best_t:
            best_t, best_m = t, m
    return best_t, best_m


# ------------------------------------------------------------------------------------------
# the true optimum of the paper's minimisation problem (Eq. 8 minimised over all plans), for any L
# ------------------------------------------------------------------------------------------

def plan_optimal(size_bytes: Sequence[int], t_backward: Sequence[float], a: float, b: float
                 ) -> Tuple[float, List[int]]:
    """Exact minimiser of t_iter - t_f over all 2^(L-1) plans, by dynamic programming over the
    arrival order.  Not in the paper (its Algorithm 1 is a greedy that Theorem 1 claims optimal; it is
    not always); the DEFINITION of the result is `bruteforce_best`, which pins this function for L <= 16.

    Let the layers arrive as k = 1..L (k = 1 is layer L).  A plan cuts this sequence into consecutive
    groups; the group holding arrivals i+1..k sends one message of their summed bytes, starting when
    arrival k's gradient exists and the previous group's message has ended.  The end time of a group is
    non-decreasing in the end time of the group before it, so
        F[0] = 0 ;  F[k] = min over 0 <= i < k of  max(F[i], ready[k]) + (a + b * bytes(i+1..k))
    and F[L] is the optimum.  Ties take the smallest i (the longest group).  Every candidate is formed
    with the same operations, in the same order, as `iteration_time` uses for that plan, so F[L] equals
    `iteration_time(plan)` bit for bit.

    Returns (F[L], merged[0..L-1])."""
    L = len(size_bytes)
    if L == 0:
        return 0.0, []
    t_b1 = _one_based(float(x) for x in t_backward)
    tau_b = backward_start_times(t_b1)
    # arrival k is paper layer L + 1 - k
    ready = [None] + [tau_b[L + 1 - k] + t_b1[L + 1 - k] for k in range(1, L + 1)]
    nbytes = [None] + [int(size_bytes[L - k]) for k in range(1, L + 1)]
    prefix = [0] * (L + 1)
    for k in range(1, L + 1):
        prefix[k] = prefix[k - 1] + nbytes[k]
    F = [0.0] * (L + 1)
    cut = [0] * (L + 1)
    for k in range(1, L + 1):
        best = None
        for i in range(0, k):
            start = F[i] if F[i] > ready[k] else ready[k]
            cand = start + allreduce_time(a, b, prefix[k] - prefix[i])
            if best is None or cand < best:
                best, cut[k] = cand, i
        F[k] = best
    merged = [MERGED] * L
    k = L
    while k > 0:
        # the group ending at arrival k closes at paper layer L + 1 - k, which is therefore normal
        merged[(L + 1 - k) - 1] = NORMAL
        k = cut[k]
    return F[L], merged


# ------------------------------------------------------------------------------------------
# Algorithm 2 (communication handler): which layers travel together; Sec. 5.3: buffer layout
# ------------------------------------------------------------------------------------------

def groups_in_arrival_order(merged: Sequence[int]) -> List[List[int]]:
    """Replay the communication handler: layers are pushed L, L-1, ..., 1 into a layer buffer and the
    buffer is all-reduced and cleared whenever the pushed layer is normal.

    Returns groups of 0-based tensor indices, first-communicated group first; inside a group the
    indices are in arrival order (descending)."""
    L = len(merged)
    groups: List[List[int]] = []
    lb: List[int] = []
    for l in range(L, 0, -1):
        lb.append(l - 1)
        if merged[l - 1] == NORMAL:
            groups.append(lb)
            lb = []
    if lb:
        raise ValueError("layer 1 must be normal")
    return groups


def group_ready_times(merged: Sequence[int], t_backward: Sequence[float]) -> List[float]:
    """When each group's buffer is full, in seconds from the start of the backward pass, first group first.

    The handler of Algorithm 2 sends a buffer when the layer it has just pushed is normal; that layer's
    gradient exists at tau_b^(l) + t_b^(l) (Eq. 6 with tau_b^(L) = 0)."""
    L = len(merged)
    t_b1 = _one_based(float(x) for x in t_backward)
    tau_b = backward_start_times(t_b1) if L else []
    ready = []
    for members in groups_in_arrival_order(merged):
        l = members[-1] + 1                      # the group's last arrival, a normal layer
        ready.append(tau_b[l] + t_b1[l])
    return ready


def merge_layout(n_elems: Sequence[int], merged: Sequence[int]):
    """Element layout of the pre-allocated merge buffers (Sec. 5.3).

    Returns (tensor_group[L], tensor_off[L], group_elems[G]): tensor i lives in buffer
    tensor_group[i] at element offset tensor_off[i]; a buffer holds exactly the sum of its members'
    elements, members in arrival order, no padding."""
    L = len(n_elems)
    tensor_group = [None] * L
    tensor_off = [None] * L
    group_elems = []
    for k, members in enumerate(groups_in_arrival_order(merged)):
        fill = 0
        for i in members:
            tensor_group[i] = k
            tensor_off[i] = fill
            fill += int(n_elems[i])
        group_elems.append(fill)
    return tensor_group, tensor_off, group_elems
