"""HIP path against the CPU oracle, element by element, through the C ABI.  Everything here is
bit-exact: pack is a copy, and reduce / update fix the operation order and rounding."""
import sys
import time

import numpy as np
import pytest

import workloads as W
from oracle import pipeline as OD
from oracle import plan as OP

pytestmark = pytest.mark.gpu

MODES = ("staged", "staged_per_group", "reduce_update", "pipeline", "pipeline_per_group", "pipeline_no_reduced",
         "pipeline_spans", "direct", "direct_per_group_with_reduced", "pipeline_two_streams",
         "handler_replay_at_once", "handler_replay_on_a_schedule", "handler_replay_one_launch_per_group")
NO_REDUCED = ("reduce_update", "pipeline_no_reduced", "direct")
NO_MERGE = ("direct", "direct_per_group_with_reduced")


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _bits(a):
    a = np.ascontiguousarray(a)
    return a.view(np.uint32) if a.dtype == np.float32 else a.view(np.uint16)


def _run_mode(dm, mode, lr, mu, G):
    if mode == "staged":
        dm.pack(); dm.reduce(); dm.unpack_update(lr, mu)
    elif mode == "staged_per_group":
        for k in range(G):
            dm.pack(k); dm.reduce(k); dm.unpack_update(lr, mu, k)
    elif mode == "reduce_update":
        dm.pack(); dm.reduce_update(lr, mu)
    elif mode == "pipeline":
        dm.group_pipeline(lr, mu)
    elif mode == "pipeline_per_group":
        for k in reversed(range(G)):          # groups are independent: any order gives the same bits
            dm.group_pipeline(lr, mu, k)
    elif mode == "pipeline_no_reduced":
        dm.group_pipeline(lr, mu, write_reduced=False)
    elif mode == "pipeline_spans":                # a few consecutive groups per launch, plus an empty span
        k = 0
        width = 1
        while k < G:
            n = min(width, G - k)
            dm.group_pipeline_span(lr, mu, k, n)
            k += n
            width = width % 3 + 1
        dm.group_pipeline_span(lr, mu, G, 0)
    elif mode == "pipeline_two_streams":          # groups touch disjoint elements: any streams, any overlap
        import torch
        main = torch.cuda.current_stream()
        side = [torch.cuda.Stream(), torch.cuda.Stream()]       # default priority
        for s in side:
            s.wait_stream(main)
        for k in range(G):
            with torch.cuda.stream(side[k % 2]):
                dm.group_pipeline(lr, mu, k)
        for s in side:
            main.wait_stream(s)
    elif mode == "handler_replay_at_once":        # every group full at t0: one launch on the current stream
        import torch
        stats = dm.handler_replay(lr, mu, np.linspace(0.0, 1e-3, G), 0.0,
                                  [int(torch.cuda.current_stream().cuda_stream)], write_reduced=True)
        assert stats[0] == (1 if G else 0) and stats[1] == 0.0 and stats[3] == stats[2] >= 0.0
    elif mode == "handler_replay_one_launch_per_group":   # all full at t0, never batched, four streams
        import torch
        main = torch.cuda.current_stream()
        side = [torch.cuda.Stream() for _ in range(4)]          # default priority
        for s in side:
            s.wait_stream(main)
        stats = dm.handler_replay(lr, mu, np.zeros(G), 0.0, [int(s.cuda_stream) for s in side], write_reduced=True,
                                  max_groups_per_launch=1)
        assert stats[0] == G
    elif mode == "handler_replay_on_a_schedule":  # a group every 40 us on three streams: several launches
        import torch
        main = torch.cuda.current_stream()
        side = [torch.cuda.Stream() for _ in range(3)]          # default priority
        for s in side:
            s.wait_stream(main)
        ready = 40e-6 * np.arange(G)
        stats = dm.handler_replay(lr, mu, ready, 1.0, [int(s.cuda_stream) for s in side], write_reduced=True)
        assert 1 <= stats[0] <= G or G == 0
        assert stats[1] == (ready[-1] if G else 0.0) and stats[2] >= stats[1]
        _say(f"[parity]   handler replay: {stats[0]} launches for {G} groups, exposed {1e6 * stats[3]:.0f} us")
    elif mode == "direct":                        # merge arenas never written
        dm.direct_update(lr, mu)
    elif mode == "direct_per_group_with_reduced":
        for k in range(G):
            dm.direct_update(lr, mu, k, write_reduced=True)
    else:
        raise KeyError(mode)


def check_case(profile, merged, mode, misalign=0, steps=1, seed=W.BASE_SEED, label="", launch=None, resident=None,
               pacing=None, small_launch=None):
    """Run `steps` iterations on the GPU and in the oracle from the same host arrays and compare every
    output: P merge arenas, the reduced arena, weights and momenta, and the padding of the arenas."""
    import torch
    import paper_1912_09268_amd as M
    from paper_1912_09268_amd import harness as H

    _say(f"[parity] {label or profile.name} L={profile.L} E={profile.total_elems} P={profile.P} "
         f"{profile.grad_dtype} mode={mode} misalign={misalign} seed={seed}")
    n = [int(x) for x in profile.n_elems]
    merged = [int(x) for x in merged]
    gdt = {"f32": M.F32, "bf16": M.BF16, "f16": M.F16}[profile.grad_dtype]
    ctx = M.Context(n, merged, profile.P, gdt)
    if launch is not None:
        ctx.set_launch(*launch)
    if resident is not None:
        ctx.set_resident_bytes(resident)
    if pacing is not None:
        ctx.set_pacing(*pacing)
    if small_launch is not None:
        ctx.set_small_launch(small_launch)
    dm = H.DeviceModel(ctx, n, misalign=misalign, fill_arena=True)
    off, grp, base, ge = ctx.layout()
    groups = OP.groups_in_arrival_order(merged)
    assert len(groups) == ctx.n_groups

    w_flat = W.initial_weights_flat(profile, seed)
    v_flat = W.initial_momentum_flat(profile, seed)
    dm.upload_weights(w_flat, v_flat)
    w_o = [x.copy() for x in W.split_by_layer(w_flat, profile.n_elems)]
    v_o = [x.copy() for x in W.split_by_layer(v_flat, profile.n_elems)]

    for step in range(steps):
        flats = [W.worker_gradient_flat(profile, w, seed + 1000 * step) for w in range(profile.P)]
        for w in range(profile.P):
            dm.upload_grads(w, flats[w])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        _run_mode(dm, mode, profile.lr, profile.momentum, ctx.n_groups)
        torch.cuda.synchronize()
        _say(f"[parity]   step {step}: device calls took {1e3 * (time.perf_counter() - t0):.2f} ms")

        grads = [W.split_by_layer(f, profile.n_elems) for f in flats]
        merge_dev = [dm.download_merge(w) for w in range(profile.P)]
        red_dev = dm.download_reduced()
        covered = np.zeros(max(ctx.arena_elems, 1), bool)
        red_o = []
        for k, members in enumerate(groups):
            lo, hi = int(base[k]), int(base[k]) + int(ge[k])
            covered[lo:hi] = True
            bufs = [OD.pack(grads[w], [members])[0] for w in range(profile.P)]
            if mode not in NO_MERGE:
                for w in range(profile.P):
                    assert np.array_equal(_bits(merge_dev[w][lo:hi]), _bits(bufs[w])), f"merge arena w={w} group={k}"
            r = OD.reduce_average(bufs)
            red_o.append(r)
            if mode not in NO_REDUCED:
                assert np.array_equal(_bits(red_dev[lo:hi]), _bits(r)), f"reduced group={k}"
        # padding between groups is never written
        pad = ~covered
        for w in range(profile.P):
            m = _bits(merge_dev[w])
            sent = H.SENTINEL32 if m.dtype == np.uint32 else H.SENTINEL16
            assert (m[pad] == sent).all(), "merge arena padding was written"
            if mode in NO_MERGE:
                assert (m == sent).all(), "merge arenas must stay untouched in this mode"
        r32 = _bits(red_dev)
        assert (r32[pad] == H.SENTINEL32).all(), "reduced arena padding was written"
        if mode in NO_REDUCED:
            assert (r32 == H.SENTINEL32).all(), "reduced arena must stay untouched in this mode"
        OD.unpack_update(red_o, groups, w_o, v_o, profile.lr, profile.momentum)
        w_dev = dm.download_weights()
        v_dev = dm.download_momenta()
        w_ref = np.concatenate(w_o) if w_o else np.zeros(0, np.float32)
        v_ref = np.concatenate(v_o) if v_o else np.zeros(0, np.float32)
        assert np.array_equal(_bits(v_dev), _bits(v_ref)), "momentum"
        assert np.array_equal(_bits(w_dev), _bits(w_ref)), "weights"
        assert dm.guard_bands_intact(), "a per-layer tensor was written outside its bounds"
        dm.fill_arenas()
    ctx.close()


def _plan_of(profile):
    import paper_1912_09268_amd as M
    merged, _ = M.plan(profile.size_bytes, profile.t_backward, profile.a, profile.b)
    ref = OP.plan_algorithm1([int(x) for x in profile.size_bytes], [float(x) for x in profile.t_backward],
                             profile.a, profile.b)
    assert merged.tolist() == ref
    return ref


# ------------------------------------------------------------------------------------------
# small and medium cases: several tiles, ragged tails, every mode
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("mode", MODES)
def test_toy_mlp_all_modes(mode):
    p = W.make_profile("toy_mlp")
    check_case(p, _plan_of(p), mode, steps=2)


@pytest.mark.parametrize("P", [1, 2, 3, 4, 8, 16])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_random_models_worker_counts(P, dtype):
    rng = np.random.default_rng(1000 + P)
    p = W.make_random_profile(rng, 50, size_hi=20000, P=P, grad_dtype=dtype, allow_empty=True)
    merged = [0] + [int(x) for x in (rng.random(p.L - 1) < 0.6)]
    for mode in ("staged", "pipeline", "reduce_update", "pipeline_spans", "direct_per_group_with_reduced"):
        check_case(p, merged, mode, label=f"random P={P}")


@pytest.mark.parametrize("P", [33, 64])
def test_largest_worker_counts(P):
    import paper_1912_09268_amd as M
    rng = np.random.default_rng(2000 + P)
    p = W.make_random_profile(rng, 12, size_hi=9000, P=P, grad_dtype="bf16" if P == 33 else "f32")
    merged = [0] + [int(x) for x in (rng.random(p.L - 1) < 0.5)]
    for mode in ("staged", "pipeline", "direct"):
        check_case(p, merged, mode, label=f"P={P}")
    with pytest.raises(M.MgwfbpError):
        M.Context([4, 4], [0, 1], 65, M.F32)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("mode", ["staged", "pipeline", "direct_per_group_with_reduced"])
def test_misaligned_sources_and_odd_sizes(dtype, mode):
    rng = np.random.default_rng(7)
    p = W.make_random_profile(rng, 80, size_lo=1, size_hi=9000, P=4, grad_dtype=dtype)
    merged = [0] + [int(x) for x in (rng.random(p.L - 1) < 0.7)]
    check_case(p, merged, mode, misalign=3, steps=2, label="misaligned")


@pytest.mark.parametrize("mode", ["staged", "pipeline", "direct"])
def test_thousands_of_one_element_tensors(mode):
    """More segments in one tile than the kernel stages in LDS, plus straddling vectors everywhere."""
    sizes = [1] * 3000 + [5, 1, 1, 7] * 50 + [4100, 3]
    rng = np.random.default_rng(8)
    p = W.Profile("ones", np.asarray(sizes, np.uint64), rng.uniform(1e-6, 1e-5, len(sizes)), 1e-4, 1e-9, 2,
                  "f32", 1.0)
    merged = [0] + [1] * (len(sizes) - 1)
    check_case(p, merged, mode)
    merged = [0] + [int(x) for x in (rng.random(len(sizes) - 1) < 0.97)]
    check_case(p, merged, mode)


def test_single_layer_and_all_normal_and_all_merged():
    rng = np.random.default_rng(9)
    one = W.Profile("one", np.asarray([70001], np.uint64), np.asarray([1e-3]), 1e-5, 1e-9, 8, "f32", 1.0)
    check_case(one, [0], "pipeline")
    check_case(one, [0], "staged")
    p = W.make_random_profile(rng, 12, size_hi=30000, P=8)
    check_case(p, [0] * p.L, "pipeline", label="all normal")
    check_case(p, [0] + [1] * (p.L - 1), "pipeline", label="all merged")
    check_case(p, [0] + [1] * (p.L - 1), "staged_per_group", label="all merged")


def test_empty_model_and_empty_groups_are_no_ops():
    empty = W.Profile("empty", np.zeros(3, np.uint64), np.asarray([1e-3] * 3), 1e-5, 1e-9, 2, "f32", 1.0)
    check_case(empty, [0, 1, 0], "staged")
    check_case(empty, [0, 1, 0], "pipeline_per_group")
    mixed = W.Profile("mixed", np.asarray([0, 0, 9, 0, 5000, 0], np.uint64), np.asarray([1e-3] * 6), 1e-5, 1e-9, 2,
                      "f32", 1.0)
    check_case(mixed, [0, 1, 0, 0, 1, 0], "staged_per_group")
    check_case(mixed, [0, 1, 0, 0, 1, 0], "pipeline")


def test_special_values_propagate_like_ieee():
    """Subnormals, signed zeros, infinities and NaNs go through pack untouched and through reduce /
    update with IEEE semantics (no flush to zero)."""
    import torch
    import paper_1912_09268_amd as M
    from paper_1912_09268_amd import harness as H
    n = [5000]
    ctx = M.Context(n, [0], 2, M.F32)
    dm = H.DeviceModel(ctx, n, fill_arena=True)
    g0 = np.full(5000, 1e-40, np.float32)           # subnormal
    g1 = np.full(5000, 2e-40, np.float32)
    g0[1], g1[1] = np.inf, 1.0
    g0[2], g1[2] = np.inf, -np.inf                  # NaN
    g0[3], g1[3] = -0.0, -0.0
    g0[4], g1[4] = 3.0e38, 3.0e38                   # overflows to +inf in the sum
    w = np.ones(5000, np.float32)
    v = np.full(5000, 1e-41, np.float32)
    dm.upload_grads(0, g0); dm.upload_grads(1, g1); dm.upload_weights(w, v)
    dm.group_pipeline(0.1, 0.9)
    torch.cuda.synchronize()
    bufs = [g0, g1]
    r = OD.reduce_average(bufs)
    wo, vo = w.copy(), v.copy()
    OD.sgd_momentum(wo, vo, r, 0.1, 0.9)
    def same(dev, ref):
        # IEEE 754 fixes which results are NaN but not a NaN's sign or payload: compare NaN positions,
        # and bits everywhere else
        nan = np.isnan(ref)
        return np.array_equal(np.isnan(dev), nan) and np.array_equal(_bits(dev)[~nan], _bits(ref)[~nan])

    assert np.array_equal(_bits(dm.download_merge(0)[:5000]), _bits(g0))       # a copy keeps every bit
    assert same(dm.download_reduced()[:5000], r)
    assert same(dm.download_momenta(), vo)
    assert same(dm.download_weights(), wo)
    assert r[0] != 0 and np.isnan(r[2]) and np.isinf(r[4])
    ctx.close()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_every_sixteen_bit_pattern_through_pack_and_reduce(dtype):
    """All 65536 patterns of a 16-bit gradient format (subnormals, both zeros, infinities, quiet and signalling
    NaNs) go through pack bit for bit, and through reduce as the values the format defines."""
    import torch
    import paper_1912_09268_amd as M
    from paper_1912_09268_amd import harness as H
    n = [65536]
    ctx = M.Context(n, [0], 2, M.F16 if dtype == "f16" else M.BF16)
    dm = H.DeviceModel(ctx, n, fill_arena=True)
    patterns = np.arange(65536, dtype=np.uint16)
    g0 = patterns.view(np.float16) if dtype == "f16" else patterns
    half = np.float16(0.5) if dtype == "f16" else np.uint16(0x3F00)
    g1 = np.full(65536, half, dtype=g0.dtype)
    _say(f"[parity] all 65536 {dtype} patterns, P=2")
    dm.upload_grads(0, g0); dm.upload_grads(1, g1)
    dm.upload_weights(np.zeros(65536, np.float32), np.zeros(65536, np.float32))
    dm.pack(); dm.reduce()
    torch.cuda.synchronize()
    assert np.array_equal(_bits(dm.download_merge(0)[:65536]), patterns)
    r = OD.reduce_average([g0, g1])
    dev = dm.download_reduced()[:65536]
    nan = np.isnan(r)
    assert np.array_equal(np.isnan(dev), nan) and np.array_equal(_bits(dev)[~nan], _bits(r)[~nan])
    ctx.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("kind", ["pack", "reduce", "unpack_update", "reduce_update", "pipeline", "direct", "span",
                                  "static"])
def test_a_call_for_one_group_touches_only_that_group(kind, dtype):
    """Groups lie end to end in the arena and share tiles with their neighbours.  A call for group k (or for a
    run of groups) must produce the oracle's result for k and leave every other group's arena elements,
    weights and momenta exactly as they were, whatever the offsets of its two ends inside a tile."""
    import torch
    import paper_1912_09268_amd as M
    from paper_1912_09268_amd import harness as H

    rng = np.random.default_rng(77)
    # odd sizes around the tile (2048) and the vector (4); groups of one to three tensors
    sizes = [1, 3, 2047, 2049, 5, 4096, 17, 1023, 6000, 2, 2048, 511, 7, 3000, 1025, 64]
    merged = [0, 1, 0, 0, 1, 1, 0, 0, 1, 0, 0, 1, 0, 1, 1, 0]
    prof = W.make_random_profile(rng, len(sizes), P=3, grad_dtype=dtype)
    import dataclasses
    prof = dataclasses.replace(prof, n_elems=np.asarray(sizes, np.uint64))
    gdt = {"f32": M.F32, "bf16": M.BF16}[dtype]
    n = [int(x) for x in sizes]
    host_only = kind == "static"
    ctx = M.Context(n, merged, prof.P, gdt, host_only=host_only)
    layout_ctx = ctx
    dm = H.DeviceModel(ctx, n, misalign=3, fill_arena=True)
    off, grp, base, ge = layout_ctx.layout()
    groups = OP.groups_in_arrival_order(merged)
    G = len(groups)
    seed = 4242
    flats = [W.worker_gradient_flat(prof, w, seed) for w in range(prof.P)]
    grads = [W.split_by_layer(f, prof.n_elems) for f in flats]
    for w in range(prof.P):
        dm.upload_grads(w, flats[w])
    w_flat, v_flat = W.initial_weights_flat(prof, seed), W.initial_momentum_flat(prof, seed)

    for k in range(G):
        first, count = (k, min(2, G - k)) if kind == "span" else (k, 1)
        chosen = list(range(first, first + count))
        _say(f"[parity] one group alone: kind={kind} {dtype} groups {chosen} of {G}, base {int(base[k])}")
        dm.upload_weights(w_flat, v_flat)
        w_o = [x.copy() for x in W.split_by_layer(w_flat, prof.n_elems)]
        v_o = [x.copy() for x in W.split_by_layer(v_flat, prof.n_elems)]
        dm.fill_arenas()
        if kind in ("reduce", "reduce_update", "unpack_update"):     # these read arenas: fill them for every group
            dm.pack()
            if kind == "unpack_update":
                dm.reduce()
        torch.cuda.synchronize()
        merge_before = [dm.download_merge(w).copy() for w in range(prof.P)]
        red_before = dm.download_reduced().copy()
        if kind == "pack":
            dm.pack(k)
        elif kind == "reduce":
            dm.reduce(k)
        elif kind == "unpack_update":
            dm.unpack_update(prof.lr, prof.momentum, k)
        elif kind == "reduce_update":
            dm.reduce_update(prof.lr, prof.momentum, k)
        elif kind == "pipeline":
            dm.group_pipeline(prof.lr, prof.momentum, k)
        elif kind == "direct":
            dm.direct_update(prof.lr, prof.momentum, k, write_reduced=True)
        elif kind == "span":
            dm.group_pipeline_span(prof.lr, prof.momentum, first, count)
        elif kind == "static":
            dm.group_pipeline_static(prof.lr, prof.momentum, k)
        torch.cuda.synchronize()
        merge_dev = [dm.download_merge(w) for w in range(prof.P)]
        red_dev = dm.download_reduced()
        inside = np.zeros(max(layout_ctx.arena_elems, 1), bool)
        red_o = [None] * G
        for g in chosen:
            lo, hi = int(base[g]), int(base[g]) + int(ge[g])
            inside[lo:hi] = True
            bufs = [OD.pack(grads[w], [groups[g]])[0] for w in range(prof.P)]
            red_o[g] = OD.reduce_average(bufs)
            if kind in ("pack", "pipeline", "span", "static"):
                for w in range(prof.P):
                    assert np.array_equal(_bits(merge_dev[w][lo:hi]), _bits(bufs[w])), f"merge arena w={w} group={g}"
            if kind in ("reduce", "pipeline", "direct", "span", "static"):
                assert np.array_equal(_bits(red_dev[lo:hi]), _bits(red_o[g])), f"reduced group={g}"
        for w in range(prof.P):           # every arena element outside the chosen groups is as it was
            assert np.array_equal(_bits(merge_dev[w])[~inside], _bits(merge_before[w])[~inside]), f"merge arena w={w}"
        assert np.array_equal(_bits(red_dev)[~inside], _bits(red_before)[~inside]), "reduced arena"
        if kind not in ("pack", "reduce"):
            OD.unpack_update([red_o[g] for g in chosen], [groups[g] for g in chosen], w_o, v_o, prof.lr,
                             prof.momentum)
        assert np.array_equal(_bits(dm.download_momenta()), _bits(np.concatenate(v_o))), "momentum"
        assert np.array_equal(_bits(dm.download_weights()), _bits(np.concatenate(w_o))), "weights"
        assert dm.guard_bands_intact()
    ctx.close()


def test_device_entry_points_reject_bad_arguments():
    import paper_1912_09268_amd as M
    from paper_1912_09268_amd import harness as H
    ctx = M.Context([100, 100], [0, 1], 2, M.F32)
    dm = H.DeviceModel(ctx, [100, 100])
    with pytest.raises(M.MgwfbpError):
        dm.pack(5)                                   # group out of range
    with pytest.raises(M.MgwfbpError):
        ctx.pack(0, 0, dm.merge_ptrs.data_ptr())     # null pointer table
    with pytest.raises(M.MgwfbpError):
        ctx.reduce(0, dm.merge_ptrs.data_ptr(), 0)   # null reduced arena
    with pytest.raises(M.MgwfbpError):
        dm.group_pipeline_span(0.1, 0.9, 1, 1)       # the model has one group only
    with pytest.raises(M.MgwfbpError):
        dm.group_pipeline_span(0.1, 0.9, -1, 1)
    ctx.close()
    # the handler replay checks its schedule and its streams before it launches anything
    ctx = M.Context([100, 100, 100], [0, 0, 0], 2, M.F32)
    dm = H.DeviceModel(ctx, [100, 100, 100])
    for ready, scale, streams, most in (([0.0, 2e-6, 1e-6], 1.0, [0], 0), ([0.0, 1e-6, float("nan")], 1.0, [0], 0),
                                        ([-1e-6, 0.0, 1e-6], 1.0, [0], 0), ([0.0, 1e-6, 2e-6], -1.0, [0], 0),
                                        ([0.0, 1e-6, 2e-6], float("inf"), [0], 0), ([0.0, 1e-6, 2e-6], 1.0, [], 0),
                                        ([0.0, 1e-6, 2e-6], 1.0, [0] * 17, 0), ([0.0, 1e-6, 2e-6], 1.0, [0], -1)):
        with pytest.raises(M.MgwfbpError):
            dm.handler_replay(0.1, 0.9, ready, scale, streams, max_groups_per_launch=most)
    ctx.close()


@pytest.mark.parametrize("launch", [(1, False, 0), (2, True, 0), (0, True, 0), (0, False, 2), (0, False, 4),
                                    (3, True, 3), (4096, False, 1024)])
def test_results_do_not_depend_on_launch_shape(launch):
    """Grid cap, die-contiguous numbering, tiles per workgroup and the cacheable share of w and v change how
    the work is dealt out, never what is computed."""
    rng = np.random.default_rng(77)
    p = W.make_random_profile(rng, 60, size_lo=1, size_hi=40000, P=8, allow_empty=True)
    merged = [0] + [int(x) for x in (rng.random(p.L - 1) < 0.5)]
    for mode, resident in (("pipeline", 0), ("staged", 1 << 20), ("reduce_update", None), ("staged_per_group", 3 << 18),
                           ("direct", 1 << 19)):
        check_case(p, merged, mode, launch=launch, resident=resident, label=f"launch={launch}")


@pytest.mark.parametrize("pacing", [(-1, 1), (2, 1), (3, 0), (5, 1), (7, 1), (1, 0), (12, 0), (16, 1), (20, 0), (31, 1),
                                    (64, 0), (0, -1), (3, -1)])
def test_results_do_not_depend_on_pacing(pacing):
    """The cap on workgroups per compute unit (an amount of unused LDS per launch) and the vectors a lane moves
    per step (-1: every load of a tile at once, the form small launches take by default) change when bytes move,
    never which bytes or what is computed from them."""
    rng = np.random.default_rng(78)
    p = W.make_random_profile(rng, 50, size_lo=1, size_hi=40000, P=8, allow_empty=True)
    merged = [0] + [int(x) for x in (rng.random(p.L - 1) < 0.5)]
    q = W.make_random_profile(rng, 20, size_lo=1, size_hi=30000, P=3, grad_dtype="bf16")
    merged_q = [0] + [int(x) for x in (rng.random(q.L - 1) < 0.5)]
    for mode in ("pipeline", "staged", "reduce_update", "direct"):
        check_case(p, merged, mode, pacing=pacing, label=f"pacing={pacing}")
    check_case(q, merged_q, "pipeline", pacing=pacing, misalign=3, label=f"pacing={pacing} bf16")


def test_pacing_arguments_are_checked():
    import paper_1912_09268_amd as M
    ctx = M.Context([100, 100], [0, 1], 2, M.F32, host_only=True)
    for bad in ((65, 0), (2, -2), (2, 3), (0, 5)):
        with pytest.raises(M.MgwfbpError):
            ctx.set_pacing(*bad)
    ctx.set_pacing(0, 0)
    ctx.set_pacing(-5, 1)
    ctx.set_pacing(2, -1)
    ctx.set_small_launch(0)
    ctx.set_small_launch(-1)
    ctx.close()


@pytest.mark.parametrize("max_tiles", [0, 7, 1 << 30])
def test_results_do_not_depend_on_the_small_launch_threshold(max_tiles):
    """Launches of at most `max_tiles` tiles take the burst form, larger ones the paced form: 0 sends every
    launch down the paced path, 7 splits the per-group launches of this model between the two, 2^30 sends all
    of them down the burst path."""
    rng = np.random.default_rng(79)
    p = W.make_random_profile(rng, 40, size_lo=1, size_hi=60000, P=4, allow_empty=True)
    merged = [0] + [int(x) for x in (rng.random(p.L - 1) < 0.4)]
    for mode in ("pipeline", "pipeline_per_group", "staged_per_group", "direct_per_group_with_reduced"):
        check_case(p, merged, mode, small_launch=max_tiles, label=f"small launch <= {max_tiles} tiles")


# ------------------------------------------------------------------------------------------
# the benchmark configurations at full size, in the launch configuration bench.py times
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("name,mode", [("resnet50", "pipeline"), ("resnet50", "staged"),
                                       ("tiny_layers", "pipeline"), ("tiny_layers", "staged_per_group"),
                                       ("vgg16", "pipeline"), ("vgg16", "staged"),
                                       ("transformer", "pipeline"), ("transformer", "staged"),
                                       ("resnet50", "pipeline_two_streams"),
                                       ("resnet50", "direct"), ("vgg16", "direct"), ("transformer", "direct"),
                                       ("tiny_layers", "direct")])
def test_full_size_profiles(name, mode):
    p = W.make_profile(name)
    check_case(p, _plan_of(p), mode, steps=1)


@pytest.mark.parametrize("name,wgs", [("resnet50", 0), ("resnet50", 14), ("resnet50", 18), ("resnet50", 21),
                                      ("resnet50", -1), ("vgg16", 0), ("vgg16", 14), ("vgg16", 18), ("vgg16", 21),
                                      ("vgg16", -1)])
def test_full_size_in_the_benchmarks_own_launch_configuration(name, wgs):
    """bench.py times the fused pipeline without the optional reduced arena and with the cap on workgroups per
    compute unit that its tuning step picks among the library default (0), 14, 18, 21 and none."""
    p = W.make_profile(name)
    check_case(p, _plan_of(p), "pipeline_no_reduced", steps=1, pacing=(wgs, 0))


# ------------------------------------------------------------------------------------------
# arrival-driven packing (Algorithm 2's handler): tensor by tensor, and in random runs
# ------------------------------------------------------------------------------------------

def _check_incremental(profile, merged, splitter, misalign=0, label=""):
    import torch
    import paper_1912_09268_amd as M
    from paper_1912_09268_amd import harness as H
    _say(f"[incremental] {label or profile.name} L={profile.L} E={profile.total_elems} P={profile.P} {profile.grad_dtype}")
    n = [int(x) for x in profile.n_elems]
    merged = [int(x) for x in merged]
    ctx = M.Context(n, merged, profile.P, {"f32": M.F32, "bf16": M.BF16, "f16": M.F16}[profile.grad_dtype])
    dm = H.DeviceModel(ctx, n, misalign=misalign, fill_arena=True)
    off, grp, base, ge = ctx.layout()
    flats = [W.worker_gradient_flat(profile, w) for w in range(profile.P)]
    for w in range(profile.P):
        dm.upload_grads(w, flats[w])
    w_flat, v_flat = W.initial_weights_flat(profile), W.initial_momentum_flat(profile)
    dm.upload_weights(w_flat, v_flat)
    grads = [W.split_by_layer(f, profile.n_elems) for f in flats]
    # device: push runs of tensors as they "arrive"; when a run contains a group's normal layer the
    # group's buffer is full -> reduce + update that group
    L = profile.L
    hi = L - 1
    closed = 0
    for run_len in splitter(L):
        lo = max(hi - run_len + 1, 0)
        dm.pack_tensors(hi, lo)
        while closed < ctx.n_groups and all(grp[i] != closed or i >= lo for i in range(L)):
            dm.reduce(closed)
            dm.unpack_update(profile.lr, profile.momentum, closed)
            closed += 1
        hi = lo - 1
        if hi < 0:
            break
    assert closed == ctx.n_groups
    torch.cuda.synchronize()
    # oracle: the handler's buffers, in the order they fill
    sent = [OD.pack_as_gradients_arrive(grads[w], merged) for w in range(profile.P)]
    w_o = [x.copy() for x in W.split_by_layer(w_flat, profile.n_elems)]
    v_o = [x.copy() for x in W.split_by_layer(v_flat, profile.n_elems)]
    merge_dev = [dm.download_merge(w) for w in range(profile.P)]
    red_dev = dm.download_reduced()
    covered = np.zeros(max(ctx.arena_elems, 1), bool)
    groups, reduced = [], []
    for k in range(ctx.n_groups):
        lo_e, hi_e = int(base[k]), int(base[k]) + int(ge[k])
        covered[lo_e:hi_e] = True
        bufs = [sent[w][k][0] for w in range(profile.P)]
        for w in range(profile.P):
            assert np.array_equal(_bits(merge_dev[w][lo_e:hi_e]), _bits(bufs[w])), f"merge w={w} group={k}"
        r = OD.reduce_average(bufs)
        assert np.array_equal(_bits(red_dev[lo_e:hi_e]), _bits(r))
        groups.append(sent[0][k][1])
        reduced.append(r)
    for w in range(profile.P):
        m = _bits(merge_dev[w])
        assert (m[~covered] == (H.SENTINEL32 if m.dtype == np.uint32 else H.SENTINEL16)).all()
    OD.unpack_update(reduced, groups, w_o, v_o, profile.lr, profile.momentum)
    assert np.array_equal(_bits(dm.download_weights()), _bits(np.concatenate(w_o)))
    assert np.array_equal(_bits(dm.download_momenta()), _bits(np.concatenate(v_o)))
    ctx.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_pack_tensor_by_tensor_as_gradients_arrive(dtype):
    rng = np.random.default_rng(31)
    p = W.make_random_profile(rng, 70, size_lo=1, size_hi=12000, P=4, grad_dtype=dtype, allow_empty=True)
    merged = [0] + [int(x) for x in (rng.random(p.L - 1) < 0.6)]
    _check_incremental(p, merged, lambda L: [1] * L, label="one tensor per call")
    _check_incremental(p, merged, lambda L: [1] * L, misalign=5, label="one tensor per call, misaligned")
    _check_incremental(p, merged, lambda L: [int(x) for x in np.random.default_rng(5).integers(1, 9, size=L)],
                       label="random runs")
    _check_incremental(p, merged, lambda L: [L], label="everything in one run")


def test_pack_tensors_on_toy_and_tiny_profiles():
    p = W.make_profile("toy_mlp")
    _check_incremental(p, _plan_of(p), lambda L: [1] * L)
    rng = np.random.default_rng(32)
    sizes = [1] * 700 + [3, 1, 2, 5] * 40 + [9000]
    q = W.Profile("ones", np.asarray(sizes, np.uint64), rng.uniform(1e-6, 1e-5, len(sizes)), 1e-4, 1e-9, 2, "f32", 1.0)
    merged = [0] + [int(x) for x in (rng.random(len(sizes) - 1) < 0.95)]
    _check_incremental(q, merged, lambda L: [int(x) for x in np.random.default_rng(6).integers(1, 40, size=L)],
                       label="many one-element tensors")


def test_pack_tensors_rejects_bad_runs():
    import paper_1912_09268_amd as M
    from paper_1912_09268_amd import harness as H
    ctx = M.Context([100, 0, 100], [0, 1, 1], 2, M.F32)
    dm = H.DeviceModel(ctx, [100, 0, 100])
    for first, last in ((0, 1), (3, 0), (1, -1)):
        with pytest.raises(M.MgwfbpError):
            dm.pack_tensors(first, last)
    dm.pack_tensors(1, 1)            # an empty tensor: accepted, nothing to do
    ctx.close()


# ------------------------------------------------------------------------------------------
# HIP graph: one launch per group captured once, replayed with eager work in between
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("fork", [1, 4])
def test_per_group_launches_replay_correctly_from_a_hip_graph(fork):
    """One launch per group recorded into a HIP graph, on one stream (fork = 1) or forked over four streams and
    joined again (the form bench.py times); every replay is compared with the oracle's next step."""
    import torch
    import paper_1912_09268_amd as M
    from paper_1912_09268_amd import harness as H
    p = W.make_profile("toy_mlp")
    rng = np.random.default_rng(40)
    q = W.make_random_profile(rng, 40, size_hi=15000, P=8)
    for prof, merged in ((p, _plan_of(p)), (q, [0] + [int(x) for x in (rng.random(q.L - 1) < 0.5)])):
        n = [int(x) for x in prof.n_elems]
        ctx = M.Context(n, merged, prof.P, M.F32)
        dm = H.DeviceModel(ctx, n, fill_arena=True)
        flats = [W.worker_gradient_flat(prof, w) for w in range(prof.P)]
        for w in range(prof.P):
            dm.upload_grads(w, flats[w])
        w_flat, v_flat = W.initial_weights_flat(prof), W.initial_momentum_flat(prof)
        dm.upload_weights(w_flat, v_flat)
        torch.cuda.synchronize()
        side = [torch.cuda.Stream() for _ in range(fork)] if fork > 1 else []     # default priority
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):                      # capture only: nothing runs here
            if fork == 1:
                for k in range(ctx.n_groups):
                    dm.group_pipeline(prof.lr, prof.momentum, k)
            else:
                origin = torch.cuda.current_stream()
                for s in side:
                    s.wait_stream(origin)
                for k in range(ctx.n_groups):
                    with torch.cuda.stream(side[k % fork]):
                        dm.group_pipeline(prof.lr, prof.momentum, k)
                for s in side:
                    origin.wait_stream(s)
        grads = [W.split_by_layer(f, prof.n_elems) for f in flats]
        groups = OP.groups_in_arrival_order(merged)
        w_o = [x.copy() for x in W.split_by_layer(w_flat, prof.n_elems)]
        v_o = [x.copy() for x in W.split_by_layer(v_flat, prof.n_elems)]
        scratch = torch.zeros(1 << 20, device="cuda")
        for replay in range(4):
            graph.replay()
            scratch.add_(1.0)                              # the program's own eager work between replays
            torch.cuda.synchronize()
            OD.merged_step(grads, groups, w_o, v_o, prof.lr, prof.momentum)
            assert np.array_equal(_bits(dm.download_weights()), _bits(np.concatenate(w_o))), f"replay {replay}"
            assert np.array_equal(_bits(dm.download_momenta()), _bits(np.concatenate(v_o))), f"replay {replay}"
        assert float(scratch[0]) == 4.0
        ctx.close()


# ------------------------------------------------------------------------------------------
# maximum sizes: a tensor with more than 2^31 elements (64-bit offsets everywhere)
# ------------------------------------------------------------------------------------------

def test_tensor_with_more_than_two_to_the_31_elements():
    """Inputs are drawn on the device with torch's seeded generator (not by the library); the oracle
    recomputes windows of the result element by element from downloaded windows of those inputs."""
    import torch
    import paper_1912_09268_amd as M
    from paper_1912_09268_amd import harness as H
    big = 2 ** 31 + 10007
    n = [3001, big, 17]
    merged = [0, 1, 1]                      # one group: tensor 2 at offset 0, the big tensor at 17, tensor 0 behind it
    P = 2
    _say(f"[parity] huge tensor: {big} bf16 elements, P={P}")
    ctx = M.Context(n, merged, P, M.BF16)
    off, grp, base, ge = ctx.layout()
    assert off.tolist() == [17 + big, 17, 0] and int(ge[0]) == sum(n)
    dm = H.DeviceModel(ctx, n, fill_arena=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1912)
    for w in range(P):
        for t in dm.grads[w]:
            t.random_(0x3A00, 0x3C00, generator=gen)          # bfloat16 patterns of small positive values
            t[::2].neg_()                                       # flip the sign bit of every other one... of the int16
    for t in dm.w:
        t.normal_(generator=gen)
    for t in dm.v:
        t.normal_(0.0, 1e-2, generator=gen)
    torch.cuda.synchronize()

    def window(t, lo, hi):
        a = t[lo:hi].cpu().numpy()
        return a.view(np.uint16) if a.dtype == np.int16 else a

    # windows inside the big tensor (start, around 2^31 elements and 2^32 bytes, end) and the small tensors
    spans = {1: [(0, 6000), (2 ** 30 - 3000, 2 ** 30 + 3000), (2 ** 31 - 3000, 2 ** 31 + 3000), (big - 6000, big)],
             0: [(0, 3001)], 2: [(0, 17)]}
    before = {}
    for i, lst in spans.items():
        for lo, hi in lst:
            before[(i, lo)] = ([window(dm.grads[w][i], lo, hi) for w in range(P)],
                               window(dm.w[i], lo, hi).copy(), window(dm.v[i], lo, hi).copy())
    dm.group_pipeline(0.1, 0.9)
    torch.cuda.synchronize()
    for i, lst in spans.items():
        for lo, hi in lst:
            g, w0, v0 = before[(i, lo)]
            a_lo = int(base[0]) + int(off[i]) + lo
            for w in range(P):
                assert np.array_equal(window(dm.merge[w], a_lo, a_lo + hi - lo), g[w]), (i, lo, w)
            r = OD.reduce_average(g)
            assert np.array_equal(_bits(window(dm.reduced, a_lo, a_lo + hi - lo)), _bits(r)), (i, lo)
            OD.sgd_momentum(w0, v0, r, 0.1, 0.9)
            assert np.array_equal(_bits(window(dm.v[i], lo, hi)), _bits(v0)), (i, lo)
            assert np.array_equal(_bits(window(dm.w[i], lo, hi)), _bits(w0)), (i, lo)
    # the padding behind the group is untouched
    end = int(base[0]) + int(ge[0])
    tail = window(dm.merge[0], end, ctx.arena_elems)
    assert (tail == H.SENTINEL16).all()
    ctx.close()


# ------------------------------------------------------------------------------------------
# the cost model fitted to a measured size sweep of the reduce step (Sec. 6.2's method, one GPU)
# ------------------------------------------------------------------------------------------

def test_fit_ab_on_a_measured_reduce_sweep():
    """Time mgwfbp_reduce over single-group models of growing size and fit T = a + b*M as the paper does for
    its all-reduce (Fig. 4).  What is asserted is parity: the library's fit of the measured points equals the
    oracle's fit of the same points.  The fitted values themselves depend on the machine and are only printed."""
    import torch
    import paper_1912_09268_amd as M
    from oracle import model as OM
    from paper_1912_09268_amd import harness as H
    P = 8
    sizes, times = [], []
    for n in (1 << 16, 1 << 18, 1 << 20, 1 << 22, 1 << 24, 1 << 25, 1 << 26):
        ctx = M.Context([n], [0], P, M.F32)
        dm = H.DeviceModel(ctx, [n])
        for m in dm.merge:
            m.normal_()
        for _ in range(5):
            dm.reduce(0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 30
        e0.record()
        for _ in range(reps):
            dm.reduce(0)
        e1.record()
        torch.cuda.synchronize()
        sizes.append(n * 4)                                   # message bytes of one worker's slice
        times.append(e0.elapsed_time(e1) * 1e-3 / reps)
        ctx.close()
    a, b = M.fit_ab(sizes, times)
    a_ref, b_ref = OM.fit_ab(np.asarray(sizes, np.float64), np.asarray(times, np.float64))
    assert b == pytest.approx(b_ref, rel=1e-9)                # two solvers of one 2x2 least-squares problem
    assert a == pytest.approx(a_ref, rel=1e-7, abs=1e-12)
    rate = (P * 4 + 4) / 4 / b / 1e12 if b > 0 else float("nan")   # bytes moved per message byte, over b
    worst = max(abs(a + b * s - t) / t for s, t in zip(sizes[3:], times[3:]))
    _say(f"[fit] reduce sweep: a = {a * 1e6:.2f} us, b = {b * 1e12:.3f} ps/B -> {rate:.2f} TB/s of traffic; "
         f"times {[round(t * 1e6, 1) for t in times]} us; worst residual above 16 MiB {100 * worst:.1f} %")


# ------------------------------------------------------------------------------------------
# broad randomised coverage: many small models with random shapes, plans, worker counts and alignments
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("block", range(6))
def test_many_random_models(block):
    rng = np.random.default_rng(9000 + block)
    for case in range(10):
        L = int(rng.integers(1, 90))
        hi = int(rng.choice([8, 300, 3000, 30000]))
        P = int(rng.choice([1, 2, 3, 4, 5, 8, 16]))
        dtype = str(rng.choice(["f32", "bf16", "f16"]))
        p = W.make_random_profile(rng, L, size_lo=1, size_hi=hi, P=P, grad_dtype=dtype, allow_empty=bool(rng.integers(0, 2)))
        merged = [0] + [int(x) for x in (rng.random(L - 1) < rng.choice([0.1, 0.5, 0.9]))]
        mode = str(rng.choice(["staged", "staged_per_group", "reduce_update", "pipeline", "pipeline_per_group",
                               "pipeline_spans", "direct", "direct_per_group_with_reduced"]))
        launch = (int(rng.choice([0, 1, 3])), bool(rng.integers(0, 2)), int(rng.choice([0, 1, 2, 5])))
        check_case(p, merged, mode, misalign=int(rng.choice([0, 0, 3, 5])), launch=launch,
                   resident=int(rng.choice([0, 1 << 16, 1 << 30])), seed=int(rng.integers(1, 10 ** 6)),
                   label=f"random block {block} case {case}")


def test_random_models_for_a_while():
    """The same checker driven by a random generator over every mode, launch shape, pacing and small-launch
    setting, for MGWFBP_RANDOM_SECONDS seconds (default 5) from seed MGWFBP_RANDOM_SEED (default 31337); set the
    two variables to sweep longer or elsewhere."""
    import os
    budget = float(os.environ.get("MGWFBP_RANDOM_SECONDS", "5"))
    seed0 = int(os.environ.get("MGWFBP_RANDOM_SEED", "31337"))
    rng = np.random.default_rng(seed0)
    t0 = time.time()
    cases = 0
    while cases == 0 or time.time() - t0 < budget:
        L = int(rng.integers(1, 120))
        hi = int(rng.choice([8, 300, 3000, 30000, 200000]))
        P = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 16, 17]))
        dtype = str(rng.choice(["f32", "bf16", "f16"]))
        p = W.make_random_profile(rng, L, size_lo=1, size_hi=hi, P=P, grad_dtype=dtype,
                                  allow_empty=bool(rng.integers(0, 2)))
        merged = [0] + [int(x) for x in (rng.random(L - 1) < rng.choice([0.1, 0.5, 0.9]))]
        mode = str(rng.choice(list(MODES)))
        launch = (int(rng.choice([0, 1, 3])), bool(rng.integers(0, 2)), int(rng.choice([0, 1, 2, 5])))
        pacing = (int(rng.choice([0, -1, 2, 3, 5, 14, 20])), int(rng.choice([0, 0, -1, 1])))
        check_case(p, merged, mode, misalign=int(rng.choice([0, 0, 3, 5])), launch=launch, pacing=pacing,
                   small_launch=int(rng.choice([-1, 0, 3, 40, 1 << 30])),
                   resident=int(rng.choice([0, 1 << 16, 1 << 30])), seed=int(rng.integers(1, 10 ** 6)),
                   steps=int(rng.choice([1, 1, 2])), label=f"random sweep {seed0} case {cases}")
        cases += 1
    _say(f"[parity] random sweep from seed {seed0}: {cases} cases in {time.time() - t0:.0f} s, all bit-exact")

