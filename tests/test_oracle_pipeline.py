"""Pins for oracle/pipeline.py and for the input helpers in workloads.py."""
import struct

import numpy as np
import pytest
import torch

import workloads as W
from oracle import pipeline as OD
from oracle import plan as OP


def _r32(x):
    """Round a binary64 value to binary32 and return it as a Python float."""
    return struct.unpack("f", struct.pack("f", x))[0]


# ----------------------------------------------------------------------------------------
# bfloat16 helpers against torch's own conversion (a library routine the oracle does not use)
# ----------------------------------------------------------------------------------------

def test_widen_bf16_known_patterns_and_against_torch():
    bits = np.array([0x3F80, 0xC000, 0x0000, 0x8000, 0x7F80, 0x0001, 0x3EAB, 0xFF80], dtype=np.uint16)
    got = OD.widen_bf16(bits)
    assert got[0] == 1.0 and got[1] == -2.0 and got[2] == 0.0 and np.signbit(got[3])
    assert np.isinf(got[4]) and got[5] == 2.0 ** -133 and np.isneginf(got[7])
    allbits = np.arange(65536, dtype=np.uint16)
    ref = torch.from_numpy(allbits.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    assert np.array_equal(OD.widen_bf16(allbits).view(np.uint32), ref.view(np.uint32))


def test_widen_f16_against_the_definition_of_binary16_for_every_pattern():
    """Pin: IEEE 754 binary16 is sign (1 bit), exponent (5 bits, bias 15), fraction (10 bits): a normal number is
    (-1)^s 2^(e-15) (1 + f/1024), a subnormal (e = 0) is (-1)^s 2^(-14) (f/1024), e = 31 is infinity (f = 0) or NaN.
    Every one of the 65536 patterns is evaluated by that formula in binary64 (exact) and compared with the
    oracle's widening; torch's own half -> float conversion is the second, independent witness."""
    allbits = np.arange(65536, dtype=np.uint16)
    got = OD.widen_f16(allbits.view(np.float16))
    assert got.dtype == np.float32
    s = (allbits >> 15).astype(np.float64)
    e = ((allbits >> 10) & 0x1F).astype(np.int64)
    f = (allbits & 0x3FF).astype(np.float64)
    want = np.where(e == 0, 2.0 ** -14 * (f / 1024.0), 2.0 ** (e - 15).astype(np.float64) * (1.0 + f / 1024.0))
    want = np.where(s == 1, -want, want)
    finite = e != 31
    assert np.array_equal(got[finite].astype(np.float64), want[finite])
    assert np.array_equal(np.signbit(got[finite]), s[finite] == 1)            # also for the two zeros
    inf = (e == 31) & (f == 0)
    assert np.all(np.isinf(got[inf])) and np.array_equal(np.signbit(got[inf]), s[inf] == 1)
    assert np.all(np.isnan(got[(e == 31) & (f != 0)]))
    ref = torch.from_numpy(allbits.view(np.int16).copy()).view(torch.float16).float().numpy()
    ok = ~np.isnan(ref)
    assert np.array_equal(got[ok].view(np.uint32), ref[ok].view(np.uint32)) and np.array_equal(np.isnan(got), np.isnan(ref))
    assert got[0x3C00] == 1.0 and got[0xC000] == -2.0 and got[0x0001] == 2.0 ** -24 and got[0x7BFF] == 65504.0


def test_reduce_f16_inputs_accumulate_in_binary32():
    """0.1 is not a binary16 number; three copies of its binary16 neighbour sum, in binary32, to a value that
    binary16 arithmetic could not hold, and the 1/3 factor is applied in binary32."""
    x = np.float16(0.1)
    bufs = [np.full(5, x, np.float16) for _ in range(3)]
    got = OD.reduce_average(bufs)
    v = np.float32(x)
    want = np.float32(np.float32(np.float32(v + v) + v) * (np.float32(1.0) / np.float32(3.0)))
    assert got.dtype == np.float32 and np.all(got == want)
    assert np.float16(np.float16(x + x) + x) != np.float32(np.float32(v + v) + v)      # binary16 adds would differ


def test_f32_to_bf16_bits_is_round_to_nearest_even():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(200_000).astype(np.float32) * np.float32(1e-3)
    x[:4] = [1.0, 1.00390625, 1.01171875, -3.0e-39]     # exact, tie to even (down), tie to even (up), subnormal
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(W.f32_to_bf16_bits(x), ref)


# ----------------------------------------------------------------------------------------
# pack
# ----------------------------------------------------------------------------------------

def test_pack_worked_example():
    grads = [np.array([1, 2], np.float32), np.array([3], np.float32), np.array([4, 5, 6], np.float32),
             np.array([], np.float32), np.array([7], np.float32)]
    m = [0, 1, 0, 1, 1]                                   # layers 5,4 merged into 3; layer 2 into 1
    groups = OP.groups_in_arrival_order(m)
    assert groups == [[4, 3, 2], [1, 0]]
    bufs = OD.pack(grads, groups)
    assert [b.tolist() for b in bufs] == [[7, 4, 5, 6], [3, 1, 2]]


def test_pack_round_trip_and_buffer_size():
    rng = np.random.default_rng(1)
    for dtype in (np.float32, np.uint16):
        L = 40
        n = rng.integers(0, 300, size=L)
        grads = [rng.integers(0, 60000, size=int(k)).astype(dtype) for k in n]
        m = [0] + [int(x) for x in rng.integers(0, 2, size=L - 1)]
        groups = OP.groups_in_arrival_order(m)
        tg, off, ge = OP.merge_layout([int(k) for k in n], m)
        bufs = OD.pack(grads, groups)
        assert [b.size for b in bufs] == ge
        assert sum(b.nbytes for b in bufs) == sum(g.nbytes for g in grads)    # Sec. 5.3 buffer bytes
        for i in range(L):
            assert np.array_equal(bufs[tg[i]][off[i]:off[i] + int(n[i])], grads[i])
            assert bufs[tg[i]].dtype == dtype


# ----------------------------------------------------------------------------------------
# reduce
# ----------------------------------------------------------------------------------------

def test_reduce_order_is_left_to_right():
    # 1e8 + 1 rounds back to 1e8 in binary32, so only the order 0,1,2,3 gives 0.25
    bufs = [np.array([v], np.float32) for v in (1e8, 1.0, -1e8, 1.0)]
    assert OD.reduce_average(bufs)[0] == np.float32(0.25)
    # any order that cancels the big terms first would have given 0.5
    assert OD.reduce_average([bufs[0], bufs[2], bufs[1], bufs[3]])[0] == np.float32(0.5)


def test_reduce_small_integers_are_exact():
    rng = np.random.default_rng(2)
    for P in (1, 2, 4, 8, 16):
        ints = rng.integers(-1000, 1000, size=(P, 5000))
        got = OD.reduce_average([ints[w].astype(np.float32) for w in range(P)])
        assert np.array_equal(got.astype(np.float64), ints.sum(axis=0) / P)


def test_reduce_identical_copies_returns_input():
    rng = np.random.default_rng(3)
    x = (rng.integers(-2 ** 19, 2 ** 19, size=4096).astype(np.float32)) * np.float32(2.0 ** -12)
    for P in (2, 4, 8, 16):
        assert np.array_equal(OD.reduce_average([x] * P), x)


def test_reduce_replayed_in_binary64_with_explicit_rounding():
    rng = np.random.default_rng(4)
    P, n = 8, 300
    bufs = [rng.standard_normal(n).astype(np.float32) * np.float32(1e-2) for _ in range(P)]
    got = OD.reduce_average(bufs)
    inv = _r32(1.0 / P)
    for j in range(n):
        acc = float(bufs[0][j])
        for w in range(1, P):
            acc = _r32(acc + float(bufs[w][j]))          # exact in binary64, then one rounding
        assert float(got[j]) == _r32(acc * inv)


def test_reduce_non_power_of_two_uses_reciprocal_multiply():
    # sum 5 over three workers: 5 * float32(1/3) and 5 / 3 round to different binary32 values
    bufs = [np.array([1.0], np.float32), np.array([1.0], np.float32), np.array([3.0], np.float32)]
    third = np.float32(1.0) / np.float32(3.0)
    assert np.float32(5.0) * third != np.float32(5.0) / np.float32(3.0)
    assert OD.reduce_average(bufs)[0] == np.float32(5.0) * third


def test_reduce_bf16_inputs_accumulate_in_binary32():
    rng = np.random.default_rng(5)
    P, n = 8, 2000
    f = [rng.standard_normal(n).astype(np.float32) * np.float32(1e-3) for _ in range(P)]
    bits = [W.f32_to_bf16_bits(x) for x in f]
    got = OD.reduce_average(bits)
    assert got.dtype == np.float32
    wide = [torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16).double().numpy() for b in bits]
    exact = np.sum(wide, axis=0) / P
    assert np.max(np.abs(got - exact)) <= 1e-6 * np.max(np.abs(exact)) + 1e-12
    # and it is the binary32 left-to-right sum of the widened values
    acc = wide[0].astype(np.float32)
    for w in range(1, P):
        acc = (acc.astype(np.float64) + wide[w]).astype(np.float32)
    assert np.array_equal(got, (acc.astype(np.float64) * 0.125).astype(np.float32))


# ----------------------------------------------------------------------------------------
# update
# ----------------------------------------------------------------------------------------

def test_update_replayed_in_binary64_with_explicit_rounding():
    rng = np.random.default_rng(6)
    n = 500
    w = rng.standard_normal(n).astype(np.float32)
    v = rng.standard_normal(n).astype(np.float32) * np.float32(1e-2)
    g = rng.standard_normal(n).astype(np.float32) * np.float32(1e-2)
    w0, v0 = w.copy(), v.copy()
    OD.sgd_momentum(w, v, g, 0.1, 0.9)
    mu, eta = _r32(0.9), _r32(0.1)
    for j in range(n):
        t1 = _r32(mu * float(v0[j]))
        vn = _r32(t1 + float(g[j]))
        t2 = _r32(eta * vn)
        wn = _r32(float(w0[j]) - t2)
        assert float(v[j]) == vn and float(w[j]) == wn


def test_update_differs_from_a_fused_multiply_add():
    # chosen so that round(mu*v) + g and fma(mu, v, g) differ: the pin that contraction is absent
    v = np.array([1.0 + 2.0 ** -23], np.float32)
    g = np.array([-0.9], np.float32)
    w = np.array([0.0], np.float32)
    v0 = float(v[0])
    OD.sgd_momentum(w, v, g, 1.0, 0.9)
    mu = _r32(0.9)
    two_roundings = _r32(_r32(mu * v0) + float(g[0]))
    fused = _r32(mu * v0 + float(g[0]))                  # exact product in binary64, one rounding
    assert two_roundings != fused
    assert float(v[0]) == two_roundings


def test_momentum_zero_reduces_to_plain_sgd():
    rng = np.random.default_rng(7)
    w = rng.standard_normal(1000).astype(np.float32)
    g = rng.standard_normal(1000).astype(np.float32)
    v = rng.standard_normal(1000).astype(np.float32)
    expect = (w.astype(np.float64) - (np.float32(0.1).astype(np.float64) * g.astype(np.float64))
              .astype(np.float32).astype(np.float64)).astype(np.float32)     # Eq. 2, one worker
    OD.sgd_momentum(w, v, g, 0.1, 0.0)
    assert np.array_equal(w, expect) and np.array_equal(v, g)


def test_zero_gradient_zero_momentum_leaves_weights():
    w = np.arange(10, dtype=np.float32)
    v = np.zeros(10, np.float32)
    OD.sgd_momentum(w, v, np.zeros(10, np.float32), 0.1, 0.9)
    assert np.array_equal(w, np.arange(10, dtype=np.float32)) and not v.any()


# ----------------------------------------------------------------------------------------
# merged iteration == unmerged S-SGD (Sec. 6.3.2: aggregated gradients are the same)
# ----------------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_merged_step_equals_unmerged_step(dtype):
    rng = np.random.default_rng(8)
    prof = W.make_random_profile(rng, 30, size_hi=700, P=4, grad_dtype=dtype, allow_empty=True)
    n = prof.n_elems
    grads = [W.split_by_layer(W.worker_gradient_flat(prof, w), n) for w in range(prof.P)]
    w1 = [x.copy() for x in W.split_by_layer(W.initial_weights_flat(prof), n)]
    v1 = [x.copy() for x in W.split_by_layer(W.initial_momentum_flat(prof), n)]
    w2 = [x.copy() for x in w1]
    v2 = [x.copy() for x in v1]
    m = OP.plan_algorithm1([int(x) for x in prof.size_bytes], [float(x) for x in prof.t_backward],
                           prof.a, prof.b)
    groups = OP.groups_in_arrival_order(m)
    merge, reduced = OD.merged_step(grads, groups, w1, v1, prof.lr, prof.momentum)
    OD.unmerged_step(grads, w2, v2, prof.lr, prof.momentum)
    for i in range(prof.L):
        assert np.array_equal(w1[i].view(np.uint32), w2[i].view(np.uint32))
        assert np.array_equal(v1[i].view(np.uint32), v2[i].view(np.uint32))
    assert len(merge) == prof.P and len(reduced) == len(groups)
    assert all(r.dtype == np.float32 for r in reduced)


def test_merged_step_tiny_case_by_hand():
    # two workers, two layers merged into one buffer; all values exact in binary32
    grads = [[np.array([2.0, 4.0], np.float32), np.array([8.0], np.float32)],
             [np.array([6.0, 0.0], np.float32), np.array([-4.0], np.float32)]]
    w = [np.array([1.0, 1.0], np.float32), np.array([1.0], np.float32)]
    v = [np.array([1.0, -2.0], np.float32), np.array([4.0], np.float32)]
    groups = OP.groups_in_arrival_order([0, 1])
    merge, reduced = OD.merged_step(grads, groups, w, v, 0.5, 0.5)
    assert merge[0][0].tolist() == [8.0, 2.0, 4.0] and merge[1][0].tolist() == [-4.0, 6.0, 0.0]
    assert reduced[0].tolist() == [2.0, 4.0, 2.0]
    assert v[1].tolist() == [4.0] and v[0].tolist() == [4.5, 1.0]          # 0.5*v + g
    assert w[1].tolist() == [-1.0] and w[0].tolist() == [-1.25, 0.5]       # w - 0.5*v


def test_arrival_driven_pack_equals_whole_group_pack():
    rng = np.random.default_rng(9)
    for _ in range(30):
        L = int(rng.integers(1, 40))
        n = rng.integers(0, 200, size=L)
        grads = [rng.integers(0, 1000, size=int(k)).astype(np.float32) for k in n]
        m = [0] + [int(x) for x in rng.integers(0, 2, size=L - 1)]
        groups = OP.groups_in_arrival_order(m)
        sent = OD.pack_as_gradients_arrive(grads, m)
        bufs = OD.pack(grads, groups)
        assert [idx for _, idx in sent] == groups
        for (buf, _), ref in zip(sent, bufs):
            assert np.array_equal(buf, ref)
    # by hand: layers 3,2 merged into 1 -> one buffer [g3 | g2 | g1]
    g = [np.array([1.0], np.float32), np.array([2.0, 3.0], np.float32), np.array([4.0], np.float32)]
    (buf, idx), = OD.pack_as_gradients_arrive(g, [0, 1, 1])
    assert buf.tolist() == [4.0, 2.0, 3.0, 1.0] and idx == [2, 1, 0]
