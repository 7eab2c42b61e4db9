"""Oracle for the data half of MG-WFBP: pack, reduce, unpack + update.
TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Plain numpy: one loop over tensors, one over workers, element-wise float32 ufuncs (each numpy
ufunc call rounds once to binary32, so `a * b + c` written as two calls is two roundings and can
never become a fused multiply-add).  No blocking, no fusion, no reordering.

What each function states:
  pack            Sec. 5.3: the gradients of a group's member layers are copied, in arrival order,
                  into one contiguous pre-allocated buffer of exactly the summed size.
  reduce_average  Eq. 2: (1/N) * sum over workers g = 1..N of the gradients.  The sum runs in worker
                  order 0, 1, ..., P-1 in binary32; the factor is one multiply by float32(1/P)
                  (the paper fixes neither order nor placement; this is the reading both sides use).
                  Half-precision gradients (Sec. 5.3, BytesPerElement = 2) are IEEE binary16 values
                  (numpy float16, the paper's FP16) or bfloat16 bit patterns (uint16, the benchmark
                  configuration's); both widen exactly to binary32 before the first add and the result
                  stays binary32.
  unpack_update   Eq. 2 / Algorithm 2 line 15 with a momentum buffer (the paper's update is plain
                  SGD; the momentum term comes from the benchmark configuration):
                      v <- mu * v + g ;  w <- w - eta * v      (four roundings, no FMA)
                  with g read from the reduced buffer at the tensor's offset.
  unmerged_step   The same iteration without any merging: every layer averaged and updated by
                  itself.  The paper states that merged aggregation gives the same gradients as plain
                  S-SGD (Sec. 6.3.2), so the merged path must reproduce this bit for bit.

Pins: tests/test_oracle_pipeline.py (binary64-then-round replay of every binary32 operation,
integer-valued data with exact sums, identical-copies identity, mu = 0 reduction to Eq. 2,
merged == unmerged, scalar struct-based replay on tiny inputs).
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> the binary32 values they denote (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def widen_f16(x: np.ndarray) -> np.ndarray:
    """IEEE binary16 values -> the same values in binary32 (exact: binary32 has more exponent and more
    fraction bits)."""
    return x.astype(np.float32)


def as_f32(x: np.ndarray) -> np.ndarray:
    if x.dtype == np.float32:
        return x
    if x.dtype == np.uint16:
        return widen_bf16(x)
    if x.dtype == np.float16:
        return widen_f16(x)
    raise TypeError(f"gradient dtype {x.dtype} not understood (float32, float16 or uint16 bfloat16 bits)")


# ------------------------------------------------------------------------------------------
# pack
# ------------------------------------------------------------------------------------------

def pack(grads: Sequence[np.ndarray], groups: Sequence[Sequence[int]]) -> List[np.ndarray]:
    """One worker's merge buffers: buffers[k] is the concatenation of grads[i] for i in groups[k],
    in the order listed (arrival order).  Bits are copied, never converted."""
    buffers = []
    for members in groups:
        total = sum(int(grads[i].size) for i in members)
        dtype = grads[members[0]].dtype
        buf = np.empty(total, dtype=dtype)
        fill = 0
        for i in members:
            n = int(grads[i].size)
            buf[fill:fill + n] = grads[i]
            fill += n
        buffers.append(buf)
    return buffers


def pack_as_gradients_arrive(grads: Sequence[np.ndarray], merged: Sequence[int]):
    """Algorithm 2's communication handler for one worker, one iteration: layers are popped in the order
    L, L-1, ..., 1; each is pushed to the layer buffer (its gradient is copied behind what the buffer
    already holds, Sec. 5.3), and when the pushed layer is a normal layer the buffer is full: it is
    handed to the all-reduce and a fresh buffer is started.

    Returns the list of full buffers in the order they were handed over, each with the 0-based tensor
    indices it holds: [(buffer, [indices]), ...]."""
    L = len(grads)
    sent = []
    parts: List[np.ndarray] = []
    members: List[int] = []
    for l in range(L, 0, -1):
        parts.append(grads[l - 1])            # lb.push(l)
        members.append(l - 1)
        if merged[l - 1] == 0:                # m[l] == l_n
            buf = np.concatenate(parts) if parts else np.empty(0, grads[0].dtype)
            sent.append((buf, members))
            parts, members = [], []
    if parts:
        raise ValueError("layer 1 must be a normal layer")
    return sent


# ------------------------------------------------------------------------------------------
# reduce
# ------------------------------------------------------------------------------------------

def reduce_average(worker_buffers: Sequence[np.ndarray]) -> np.ndarray:
    """Average of P equally long buffers (one per worker), summed in worker order."""
    P = len(worker_buffers)
    acc = as_f32(worker_buffers[0]).copy()
    for g in range(1, P):
        acc = np.add(acc, as_f32(worker_buffers[g]), dtype=np.float32)
    inv = np.float32(1.0) / np.float32(P)
    return np.multiply(acc, inv, dtype=np.float32)


# ------------------------------------------------------------------------------------------
# unpack + update
# ------------------------------------------------------------------------------------------

def sgd_momentum(w: np.ndarray, v: np.ndarray, g: np.ndarray, lr: float, momentum: float) -> None:
    """In place: v <- mu*v + g ; w <- w - eta*v, every operation rounded to binary32."""
    mu = np.float32(momentum)
    eta = np.float32(lr)
    t1 = np.multiply(v, mu, dtype=np.float32)
    v[...] = np.add(t1, g, dtype=np.float32)
    t2 = np.multiply(v, eta, dtype=np.float32)
    w[...] = np.subtract(w, t2, dtype=np.float32)


def unpack_update(reduced: Sequence[np.ndarray], groups: Sequence[Sequence[int]],
                  weights: Sequence[np.ndarray], momenta: Sequence[np.ndarray],
                  lr: float, momentum: float) -> None:
    """Walk every reduced buffer in layout order and update the member tensors in place."""
    for k, members in enumerate(groups):
        fill = 0
        for i in members:
            n = int(weights[i].size)
            sgd_momentum(weights[i], momenta[i], reduced[k][fill:fill + n], lr, momentum)
            fill += n


# ------------------------------------------------------------------------------------------
# whole iteration, merged and unmerged
# ------------------------------------------------------------------------------------------

def merged_step(worker_grads: Sequence[Sequence[np.ndarray]], groups: Sequence[Sequence[int]],
                weights: Sequence[np.ndarray], momenta: Sequence[np.ndarray],
                lr: float, momentum: float):
    """pack for every worker, reduce every group, unpack + update.  Returns (merge_buffers[P][G],
    reduced[G]); weights and momenta are updated in place."""
    merge_buffers = [pack(g, groups) for g in worker_grads]
    reduced = [reduce_average([merge_buffers[w][k] for w in range(len(worker_grads))])
               for k in range(len(groups))]
    unpack_update(reduced, groups, weights, momenta, lr, momentum)
    return merge_buffers, reduced


def unmerged_step(worker_grads: Sequence[Sequence[np.ndarray]],
                  weights: Sequence[np.ndarray], momenta: Sequence[np.ndarray],
                  lr: float, momentum: float) -> None:
    """Plain S-SGD: each layer's gradient is averaged over the workers and applied by itself."""
    P = len(worker_grads)
    for i in range(len(weights)):
        g = reduce_average([worker_grads[w][i] for w in range(P)])
        sgd_momentum(weights[i], momenta[i], g, lr, momentum)
