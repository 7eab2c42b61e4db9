"""mgwfbp_group_pipeline_static, the entry point for callers that must not allocate device memory: its kernels
read the group/offset/tile tables from a fixed array inside the loaded library instead of the context's own
device tables.  Checked through the C ABI against mgwfbp_group_pipeline on the same inputs, bit for bit, on two
calls in a row (the second with a smaller model, so the array still holds the first call's longer tables), on a
repeated call that skips the table copy, on a model whose tables do not fit, and recorded into a HIP graph."""
import sys

import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _both_ways(profile, merged, seed, repeats=1):
    """Existing entry point on a device context vs the static entry point on a host-only context."""
    import torch
    import paper_1912_09268_amd as M
    from paper_1912_09268_amd import harness as H
    n = [int(x) for x in profile.n_elems]
    gdt = {"f32": M.F32, "bf16": M.BF16, "f16": M.F16}[profile.grad_dtype]
    ctx_dev = M.Context(n, merged, profile.P, gdt)
    ctx_host = M.Context(n, merged, profile.P, gdt, host_only=True)
    ref = H.DeviceModel(ctx_dev, n, fill_arena=True)
    new = H.DeviceModel(ctx_host, n, fill_arena=True)
    w0, v0 = W.initial_weights_flat(profile, seed), W.initial_momentum_flat(profile, seed)
    for dm in (ref, new):
        dm.upload_weights(w0, v0)
    for rep in range(repeats):
        for w in range(profile.P):
            g = W.worker_gradient_flat(profile, w, seed + 31 * rep)
            ref.upload_grads(w, g)
            new.upload_grads(w, g)
        torch.cuda.synchronize()
        _say(f"[no-alloc] {profile.name} L={profile.L} E={profile.total_elems} P={profile.P} {profile.grad_dtype} "
             f"tiles={ctx_host.n_tiles} repeat={rep}")
        ref.group_pipeline(profile.lr, profile.momentum)
        new.group_pipeline_static(profile.lr, profile.momentum)
        torch.cuda.synchronize()
        def raw(t):                                       # bit patterns: the arenas' padding holds NaN sentinels
            return t.view(torch.int32) if t.dtype == torch.float32 else t
        for a, b, what in ([(x, y, f"merge arena {i}") for i, (x, y) in enumerate(zip(ref.merge, new.merge))] +
                           [(ref.reduced, new.reduced, "reduced arena")]):
            assert torch.equal(raw(a), raw(b)), what
        assert np.array_equal(ref.download_weights().view(np.uint32), new.download_weights().view(np.uint32))
        assert np.array_equal(ref.download_momenta().view(np.uint32), new.download_momenta().view(np.uint32))
    ctx_dev.close()
    ctx_host.close()


def test_static_table_entry_point_matches_the_allocating_one_on_two_calls_in_a_row():
    rng = np.random.default_rng(2024)
    big = W.make_random_profile(rng, 60, size_lo=1, size_hi=40000, P=4, a=2e-5, b=1e-9)
    merged_big = [0] + [int(x) for x in rng.integers(0, 2, size=big.L - 1)]
    small = W.make_random_profile(rng, 9, size_lo=1, size_hi=6000, P=2, grad_dtype="bf16", a=2e-5, b=1e-9)
    merged_small = [0] + [int(x) for x in rng.integers(0, 2, size=small.L - 1)]
    _both_ways(big, merged_big, seed=11)
    _both_ways(small, merged_small, seed=12, repeats=2)      # second repeat reuses the tables already in place


def test_static_table_entry_point_rejects_models_whose_tables_do_not_fit():
    import paper_1912_09268_amd as M
    n = [(1 << 30) + 5]                                       # 524289 tiles of 32 bytes > 8 MiB
    ctx = M.Context(n, [0], 2, M.F32, host_only=True)
    with pytest.raises(M.MgwfbpError) as e:
        ctx.group_pipeline_static(-1, 256, 256, 0, 256, 256, 0.1, 0.9, 0)   # rejected before any pointer is used
    assert e.value.status == -4
    with pytest.raises(M.MgwfbpError) as e:
        ctx.group_pipeline_static(3, 256, 256, 0, 256, 256, 0.1, 0.9, 0)    # group out of range
    assert e.value.status == -1
    ctx.close()


def test_static_table_entry_point_replays_from_a_hip_graph():
    """The use the entry point names first: after one ordinary call on the capture stream has put the tables in
    place, the call is recorded into a HIP graph (nothing but the kernel launch is captured) and every replay,
    with the program's own eager work in between, is compared with the oracle's next step."""
    import torch
    import paper_1912_09268_amd as M
    from paper_1912_09268_amd import harness as H
    from oracle import pipeline as OD
    from oracle import plan as OP
    rng = np.random.default_rng(515)
    prof = W.make_random_profile(rng, 30, size_lo=1, size_hi=20000, P=4, a=2e-5, b=1e-9)
    merged = [0] + [int(x) for x in rng.integers(0, 2, size=prof.L - 1)]
    n = [int(x) for x in prof.n_elems]
    ctx = M.Context(n, merged, prof.P, M.F32, host_only=True)
    dm = H.DeviceModel(ctx, n, fill_arena=True)
    flats = [W.worker_gradient_flat(prof, w, 9) for w in range(prof.P)]
    for w in range(prof.P):
        dm.upload_grads(w, flats[w])
    w_flat, v_flat = W.initial_weights_flat(prof, 9), W.initial_momentum_flat(prof, 9)
    dm.upload_weights(w_flat, v_flat)
    grads = [W.split_by_layer(f, prof.n_elems) for f in flats]
    groups = OP.groups_in_arrival_order(merged)
    w_o = [x.copy() for x in W.split_by_layer(w_flat, prof.n_elems)]
    v_o = [x.copy() for x in W.split_by_layer(v_flat, prof.n_elems)]
    torch.cuda.synchronize()
    s = torch.cuda.Stream()                                   # default priority
    _say(f"[no-alloc] graph: L={prof.L} E={prof.total_elems} P={prof.P} tiles={ctx.n_tiles}")
    with torch.cuda.stream(s):
        dm.group_pipeline_static(prof.lr, prof.momentum)      # ordinary call: copies the tables, runs step 1
    s.synchronize()
    OD.merged_step(grads, groups, w_o, v_o, prof.lr, prof.momentum)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):                   # capture only: nothing runs here
        dm.group_pipeline_static(prof.lr, prof.momentum)
    eager = torch.zeros(1 << 20, device="cuda")
    for replay in range(3):
        graph.replay()
        eager.add_(1.0)                                       # the program's own eager work between replays
        torch.cuda.synchronize()
        OD.merged_step(grads, groups, w_o, v_o, prof.lr, prof.momentum)
        assert np.array_equal(dm.download_weights().view(np.uint32), np.concatenate(w_o).view(np.uint32)), replay
        assert np.array_equal(dm.download_momenta().view(np.uint32), np.concatenate(v_o).view(np.uint32)), replay
    assert float(eager[0]) == 3.0
    ctx.close()
