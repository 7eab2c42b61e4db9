"""Benchmark of the merged-gradient hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload vgg16] [--also resnet50,transformer,...]

A step is one pass of the whole device path over one synthetic batch of gradients: every group of the plan is
packed into the P merge arenas, reduced (sum over the P simulated workers, times 1/P) and applied to the
per-layer weights and momenta -- the fused pack + reduce + update kernel, all groups in ONE launch.  Inputs are
resident in HBM before the timed region.  The plan itself is computed once per training run; its time is
reported separately as `plan_us`.

How a step is timed.  In training a forward and a backward pass run between two updates (Algorithm 2), so
nothing the previous update touched is still in the GPU's 256 MB memory-side cache.  Every timed step therefore
(1) is preceded by an untimed scrub that reads 512 MiB and writes 512 MiB of unrelated memory, and (2) has its
own pair of HIP events on the stream the kernel is launched on; the figure reported is the MEDIAN over the K
steps.  `value`, `ms_per_step`, `pct_of_8TBps` and `roofline` all come from that cold timing.  The same K steps
issued back to back without scrubs are reported beside it (`back_to_back`), as context only.

`value` is the algorithmic bytes of the fused pipeline (2*P*g + 16 per element, g = gradient bytes) divided by
the median cold time per step, on the headline workload (the VGG-16 shape, the larger of the two shapes the
target names).  The other workloads are timed the same way in the same run and reported under `workloads`;
`target_70pct` lists the two shapes the target names.  For each workload the line also carries the launch forms
a training loop would use as groups fill during the backward pass (`launch_forms`): one launch per group on one
stream, one launch per group over four streams, and the communication handler replaying the profile's own
backward schedule (real time, and compressed until the arrivals outrun the launches).

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import dataclasses
import hashlib
import json
import os
import statistics
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
SCRUB_BYTES = 1 << 30            # half is read, half is written, before every cold step
ALL_WORKLOADS = ("vgg16", "resnet50", "transformer", "tiny_layers", "toy_mlp")

# Bytes that crossed the L2 <-> fabric boundary per pipeline launch, from two rocprofv3 --pmc runs (FETCH_SIZE,
# then WRITE_SIZE), each scaled by what the same counter reads for a plain device copy of known size; the runs
# are summarised in profiles/.  These counters sit in front of the memory-side cache, so this is what the
# kernel asks of the memory system, not a count of DRAM transactions.  A figure is only valid for the kernel
# source it was measured on: the key is the git blob hash of csrc/kernels.hip, and bench.py reports null when
# the file has changed since.
MEASURED_FABRIC_BYTES = {
    "fd3d0ccd1e08a7bcb203b5eab8bf6a152efaba89": {
        ("vgg16", "pipeline"): 1.11378e+10,
        ("resnet50", "pipeline"): 2.05763e+09,
        ("transformer", "pipeline"): 1.62547e+10,
        ("tiny_layers", "pipeline"): 1.89362e+09,
    },
}

# The paper's own numbers (other hardware, whole training iterations over a network): context, not a target.
PAPER_CONTEXT = {
    "this_path": "the paper times neither the merge copies, the reduction arithmetic, the update nor Algorithm 1; "
                 "it quotes 900 GB/s peak memory bandwidth of a Tesla V100 for the copies (Sec. 5.3) and calls the "
                 "plan a one-time O(L^2) computation (Sec. 4.2)",
    "allreduce_fit_a_s_b_s_per_byte": {
        "8 nodes x Tesla K80 (16 GPUs), 10GbE": [9.72e-4, 1.97e-9],
        "4 nodes x 4 Tesla V100 PCIe, 10GbE": [9.08e-4, 7.4e-10],
        "4 nodes x 4 Tesla V100 PCIe, 56Gb InfiniBand": [2.36e-4, 4.06e-10]},
    "iteration_time_gains": {
        "16 K80 GPUs, 10GbE, GoogleNet and ResNet-50 (Sec. 1, Sec. 6.3)":
            "about 1.2x over WFBP and about 1.36x over single-layer communication (SyncEASGD)",
        "16 V100 GPUs, ResNet-152 / DenseNet-161 / DenseNet-201 / Inception-v4 (Sec. 6.3)":
            "18.8 % faster than both baselines on average; up to 70 % on 10GbE and up to 26 % on 56Gb InfiniBand"},
    "simulated_scaling": {
        "64 workers, ring all-reduce, K80 backward times with the 10GbE cluster's a and b (Sec. 6.4)":
            "GoogleNet 1.78x over WFBP and 1.35x over SyncEASGD; ResNet-50 about 1.75x and 1.45x; MG-WFBP stays "
            "near linear while the baselines reach about 55 % scaling efficiency"},
}


def bytes_per_element(mode: str, P: int, g: int) -> int:
    """Algorithmic HBM bytes per gradient element for the path a mode runs (g = gradient bytes).
    pack 2*P*g | reduce P*g + 4 | unpack_update 20 | fused forms drop the intermediate traffic."""
    if mode in ("pipeline", "pipeline_per_group"):
        return 2 * P * g + 16            # read P grads, write P merge, read+write w and v
    if mode == "direct":
        return P * g + 16                # read P grads, read+write w and v; no merge arenas
    if mode == "pack":
        return 2 * P * g
    if mode == "reduce":
        return P * g + 4
    if mode == "unpack_update":
        return 20
    if mode == "reduce_update":
        return 2 * P * g + (P * g + 16)  # pack, then merge -> w, v
    if mode in ("staged", "staged_per_group"):
        return 3 * P * g + 24
    raise KeyError(mode)


def launches_per_step(mode: str, G: int) -> int:
    return {"pipeline": 1, "pipeline_per_group": G, "direct": 1, "pack": 1, "reduce": 1, "unpack_update": 1,
            "reduce_update": 2, "staged": 3, "staged_per_group": 3 * G}[mode]


def run_step(dm, mode: str, lr: float, mu: float, G: int) -> None:
    if mode == "pipeline":
        dm.group_pipeline(lr, mu, -1, write_reduced=False)
    elif mode == "pipeline_per_group":
        for k in range(G):
            dm.group_pipeline(lr, mu, k, write_reduced=False)
    elif mode == "direct":
        dm.direct_update(lr, mu, -1)
    elif mode == "pack":
        dm.pack(-1)
    elif mode == "reduce":
        dm.reduce(-1)
    elif mode == "unpack_update":
        dm.unpack_update(lr, mu, -1)
    elif mode == "reduce_update":
        dm.pack(-1); dm.reduce_update(lr, mu, -1)
    elif mode == "staged":
        dm.pack(-1); dm.reduce(-1); dm.unpack_update(lr, mu, -1)
    elif mode == "staged_per_group":
        for k in range(G):
            dm.pack(k); dm.reduce(k); dm.unpack_update(lr, mu, k)
    else:
        raise KeyError(mode)


class Scrubber:
    """Empties the memory-side cache: bench_aid_cache_scrub over a 1 GiB buffer on torch's current stream."""

    def __init__(self):
        import torch
        import bench_aid
        self._aid = bench_aid
        self._buf = torch.zeros(SCRUB_BYTES // 4, dtype=torch.float32, device="cuda")

    def __call__(self) -> None:
        import torch
        self._aid.cache_scrub(self._buf.data_ptr(), SCRUB_BYTES, int(torch.cuda.current_stream().cuda_stream))


def time_cold(step, scrub, steps: int, warmup: int):
    """K steps, each after a scrub, each between its own two HIP events on torch's current stream (the stream
    the library launches on).  Returns the list of per-step milliseconds."""
    import torch
    for _ in range(warmup):
        scrub()
        step()
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    for e0, e1 in pairs:
        scrub()
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    return [e0.elapsed_time(e1) for e0, e1 in pairs]


def time_back_to_back(step, steps: int, warmup: int):
    """The same K steps issued without anything between them: (wall ms per step, HIP-event ms per step)."""
    import torch
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


def pattern_ceiling(P: int, reps: int = 8):
    """What the bare read/write mix of the fused pipeline (P read-only, P write-only, 2 updated arrays) reaches on
    this GPU: bench_aid_stream_probe over binary32 arrays of 128 Mi elements each (more than 10 GB in all, so no
    cache holds any of it), HIP events.  Returns GB/s, or None if the mix has no probe instance."""
    import torch
    import bench_aid as A
    if P not in (1, 2, 4, 8, 16):
        return None
    n = 128 << 20
    mix = (P, P, 2)
    tensors = [[torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(c)] for c in mix]
    ptrs = [[t.data_ptr() for t in group] for group in tensors]
    stream = int(torch.cuda.current_stream().cuda_stream)
    for _ in range(2):
        A.stream_probe(ptrs[0], ptrs[1], ptrs[2], n, stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        A.stream_probe(ptrs[0], ptrs[1], ptrs[2], n, stream)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    del tensors
    torch.cuda.empty_cache()
    return 4 * n * (mix[0] + mix[1] + 2 * mix[2]) / (ms * 1e-3) / 1e9


def achievable_references(P: int, reps: int = 6):
    """Two more figures of the same GPU to read the kernel against: the same P + P + 2 mix walked the way the
    kernels walk it (one array at a time, workgroups of one wavefront with one 16-byte vector per lane in flight,
    sixteen of them per compute unit), and a
    plain copy of one array onto another.  GB/s each (None where the aid has no instance)."""
    import torch
    import bench_aid as A
    n = 64 << 20
    stream = int(torch.cuda.current_stream().cuda_stream)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    out = {"paced_pattern_GBps": None, "plain_copy_GBps": None}
    if P in (1, 2, 4, 8, 16):
        t = [[torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(c)] for c in (P, P, 2)]
        ptrs = [[x.data_ptr() for x in g] for g in t]
        ms = timed(lambda: A.paced_probe(ptrs[0], ptrs[1], ptrs[2], n, 64, 1, 10176, stream))
        out["paced_pattern_GBps"] = round(4 * n * (2 * P + 4) / (ms * 1e-3) / 1e9, 1)
        del t
    t = [[torch.zeros(2 * n, dtype=torch.float32, device="cuda")] for _ in range(2)]
    ms = timed(lambda: A.stream_probe([t[0][0].data_ptr()], [t[1][0].data_ptr()], [], 2 * n, stream))
    out["plain_copy_GBps"] = round(4 * 2 * n * 2 / (ms * 1e-3) / 1e9, 1)
    del t
    torch.cuda.empty_cache()
    return out


def kernel_source_hash() -> str:
    """git's blob hash of the kernel source, computed without git."""
    data = open(os.path.join(ROOT, "paper_1912_09268_amd", "csrc", "kernels.hip"), "rb").read()
    return hashlib.sha1(b"blob %d\0" % len(data) + data).hexdigest()


def _cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(profile, merged, flats, bytes_per_step, budget_s=12.0):
    """The oracle as it stands, timed on this host for whole steps until `budget_s` is used up."""
    import workloads as W
    from oracle import pipeline as OD
    from oracle import plan as OP
    groups = OP.groups_in_arrival_order([int(x) for x in merged])
    grads = [W.split_by_layer(f, profile.n_elems) for f in flats]
    w = [x.copy() for x in W.split_by_layer(W.initial_weights_flat(profile), profile.n_elems)]
    v = [x.copy() for x in W.split_by_layer(W.initial_momentum_flat(profile), profile.n_elems)]
    times = []
    t_all = time.perf_counter()
    while not times or time.perf_counter() - t_all < budget_s:
        t0 = time.perf_counter()
        OD.merged_step(grads, groups, w, v, profile.lr, profile.momentum)
        times.append(time.perf_counter() - t0)
    best = min(times)
    by = [int(x) for x in profile.size_bytes]
    tb = [float(x) for x in profile.t_backward]
    plan_times = []
    for _ in range(5):
        t0 = time.perf_counter()
        OP.plan_algorithm1(by, tb, profile.a, profile.b)
        plan_times.append((time.perf_counter() - t0) * 1e6)
    return {"value": round(bytes_per_step / best / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{len(times)} full step(s) of the {profile.name} workload (all groups, P={profile.P}) in "
                      f"{sum(times):.1f} s of CPU time; best {best * 1e3:.0f} ms/step; same byte count as `value`",
            "ms_per_step": round(best * 1e3, 1), "plan_us": round(statistics.median(plan_times), 1),
            "host_cpus": os.cpu_count(), "cpu_model": _cpu_model()}


def time_plan(p):
    """Median microseconds of the bare C-ABI call (arguments marshalled beforehand) and of the call through the
    Python binding (marshalling included)."""
    import ctypes as C
    import numpy as np
    import paper_1912_09268_amd as M
    through = []
    for _ in range(200):
        t0 = time.perf_counter()
        merged, first = M.plan(p.size_bytes, p.t_backward, p.a, p.b)
        through.append((time.perf_counter() - t0) * 1e6)
    sz = np.ascontiguousarray(p.size_bytes, np.uint64)
    tb = np.ascontiguousarray(p.t_backward, np.float64)
    m_out = np.zeros(p.L, np.uint8)
    f_out = np.zeros(p.L + 1, np.int32)
    g_out = C.c_int32(0)
    raw = M.lib().mgwfbp_plan
    c_args = (sz.ctypes.data_as(C.POINTER(C.c_uint64)), tb.ctypes.data_as(C.POINTER(C.c_double)), p.L,
              C.c_double(p.a), C.c_double(p.b), m_out.ctypes.data_as(C.POINTER(C.c_uint8)),
              f_out.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(g_out))
    bare = []
    for _ in range(200):
        t0 = time.perf_counter()
        for _ in range(20):
            raw(*c_args)
        bare.append((time.perf_counter() - t0) * 1e6 / 20)
    assert m_out.tolist() == merged.tolist()
    return merged, first, statistics.median(bare), statistics.median(through)


def launch_forms(dm, p, merged, G, scrub, one_launch_ms, reps):
    """The forms a training loop uses while groups fill during the backward pass, all through the library's own
    handler (mgwfbp_handler_replay: host clock from the call to the moment every stream has drained, so launch
    and synchronisation overheads are inside the figures).  Every repetition starts from a scrubbed cache."""
    import numpy as np
    import torch
    import paper_1912_09268_amd as M
    main = torch.cuda.current_stream()
    side = [torch.cuda.Stream() for _ in range(4)]                 # default priority
    h_main = [int(main.cuda_stream)]
    h_side = [int(s.cuda_stream) for s in side]
    ready = M.group_ready_times(merged, p.t_backward)
    backward_s = float(ready[-1]) if G else 0.0

    def replay(scale, most, streams, n):
        out = []
        for _ in range(n):
            scrub()
            torch.cuda.synchronize()
            out.append(dm.handler_replay(p.lr, p.momentum, ready, scale, streams, max_groups_per_launch=most))
        return out

    def med(rows, j):
        return statistics.median(r[j] for r in rows)

    replay(0.0, 0, h_main, 2)                                      # warm-up
    once = replay(0.0, 0, h_main, reps)                            # everything full: one launch, host-clocked
    per_group_1 = replay(0.0, 1, h_main, reps)
    per_group_4 = replay(0.0, 1, h_side, reps)
    once_ms = med(once, 2) * 1e3

    # the same G launches recorded once into a HIP graph that forks over the four streams and joins again;
    # a replay costs the host one call
    def fork_join():
        for s in side:
            s.wait_stream(main)
        for k in range(G):
            with torch.cuda.stream(side[k % 4]):
                dm.group_pipeline(p.lr, p.momentum, k, write_reduced=False)
        for s in side:
            main.wait_stream(s)
    graph_ms = None
    if G <= 1024:
        fork_join()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            main_in_capture = torch.cuda.current_stream()
            for s in side:
                s.wait_stream(main_in_capture)
            for k in range(G):
                with torch.cuda.stream(side[k % 4]):
                    dm.group_pipeline(p.lr, p.momentum, k, write_reduced=False)
            for s in side:
                main_in_capture.wait_stream(s)
        graph.replay()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            scrub()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            graph.replay()
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - t0) * 1e3)
        graph_ms = statistics.median(ts)
        del graph
    out = {
        "how": "host clock around mgwfbp_handler_replay (launches + drain of every stream), cache scrubbed first; "
               "medians of %d" % reps,
        "one_launch_all_groups_ms": round(once_ms, 4),
        "one_launch_per_group": {
            "launches": G,
            "one_stream_ms": round(med(per_group_1, 2) * 1e3, 4),
            "one_stream_vs_one_launch": round(med(per_group_1, 2) * 1e3 / once_ms, 3),
            "four_streams_ms": round(med(per_group_4, 2) * 1e3, 4),
            "four_streams_vs_one_launch": round(med(per_group_4, 2) * 1e3 / once_ms, 3),
            "hip_graph_four_streams_ms": None if graph_ms is None else round(graph_ms, 4),
            "hip_graph_four_streams_vs_one_launch": None if graph_ms is None else round(graph_ms / once_ms, 3)},
    }
    # the profile's own backward schedule (Eq. 6), in real time: groups arrive far apart, every group gets its
    # own launch, and what is left exposed after the last gradient is one small launch
    n_real = 3 if backward_s < 0.25 else 1
    real = replay(1.0, 0, h_side, n_real)
    out["arrival_replay_real_time"] = {
        "backward_pass_ms": round(backward_s * 1e3, 3), "launches": int(med(real, 0)),
        "exposed_after_last_gradient_us": round(med(real, 3) * 1e6, 1), "repetitions": n_real}
    # the same schedule compressed until the whole backward pass lasts twice the one-launch time: arrivals now
    # outrun the launches and the handler batches what filled meanwhile
    if backward_s > 0:
        scale = 2.0 * (once_ms * 1e-3) / backward_s
        fast = replay(scale, 0, h_side, reps)
        out["arrival_replay_compressed"] = {
            "backward_pass_ms": round(backward_s * scale * 1e3, 4), "launches": int(med(fast, 0)),
            "total_ms": round(med(fast, 2) * 1e3, 4),
            "exposed_after_last_gradient_us": round(med(fast, 3) * 1e6, 1),
            "total_vs_backward_pass": round(med(fast, 2) / (backward_s * scale), 3)}
    return out


def make_inputs(p):
    """Seeded host arrays of the profile, drawn in parallel (one generator per worker, as the recipe says)."""
    import workloads as W
    with ThreadPoolExecutor(max_workers=min(8, p.P)) as ex:
        flats = list(ex.map(lambda w: W.worker_gradient_flat(p, w), range(p.P)))
    return flats, W.initial_weights_flat(p), W.initial_momentum_flat(p, zero=True)


def measure_workload(name, args, scrub, headline: bool):
    import torch
    import paper_1912_09268_amd as M
    import workloads as W
    from paper_1912_09268_amd import harness as H

    p = W.make_profile(name)
    if args.workers > 0:
        p = dataclasses.replace(p, P=args.workers)
    if args.grad_dtype != "profile":
        p = dataclasses.replace(p, grad_dtype=args.grad_dtype)
    n = [int(x) for x in p.n_elems]
    g = p.elem_bytes
    merged, first, plan_us, plan_us_binding = time_plan(p)
    G = int(first.shape[0])
    ctx = M.Context(n, merged, p.P, {"f32": M.F32, "bf16": M.BF16, "f16": M.F16}[p.grad_dtype])
    if args.resident_mib >= 0:
        ctx.set_resident_bytes(args.resident_mib << 20)
    dm = H.DeviceModel(ctx, n)
    flats, w0, v0 = make_inputs(p)
    for w in range(p.P):
        dm.upload_grads(w, flats[w])
    dm.upload_weights(w0, v0)
    if not (headline and not args.no_cpu_baseline):
        flats = None
    dm.pack(-1); dm.reduce(-1)                  # so that modes that start mid-path read real data
    torch.cuda.synchronize()

    mode = args.mode

    def step():
        run_step(dm, mode, p.lr, p.momentum, G)

    # Pacing (workgroups per compute unit): results never depend on it, so it is picked by timing a few cold
    # steps, as a training loop can do during its first iterations.  "default" is the library's own choice.
    ctx.set_launch(args.blocks_per_cu, args.xcd_contiguous, max(args.tiles_per_workgroup, 0))
    tuned = None
    if args.workgroups_per_cu == "auto" and "per_group" not in mode:
        best, tuned = "default", {}
        for k in ("default", 14, 18, 21, -1):
            ctx.set_pacing(0 if k == "default" else k, args.vectors_per_step)
            tuned[str(k)] = round(statistics.median(time_cold(step, scrub, 7, 2)), 5)
            if tuned[str(k)] < tuned[str(best)] * 0.995:      # prefer the earlier on a tie
                best = k
        wgs = best
    else:
        wgs = "default" if args.workgroups_per_cu in ("auto", "default") else int(args.workgroups_per_cu)
    ctx.set_pacing(0 if wgs == "default" else wgs, args.vectors_per_step)
    tpw = max(args.tiles_per_workgroup, 0)

    cold = time_cold(step, scrub, args.steps, args.warmup)
    cold_ms = statistics.median(cold)
    wall_b2b, ev_b2b = (float("nan"), float("nan")) if args.no_back_to_back else \
        time_back_to_back(step, args.steps, args.warmup)
    E = p.total_elems
    bpe = bytes_per_element(mode, p.P, g)
    step_bytes = bpe * E
    nl = launches_per_step(mode, G)
    gbps = step_bytes / (cold_ms * 1e-3) / 1e9
    res = {
        "workload": name, "tensors": p.L, "elements": E, "groups": G, "P": p.P,
        "dtype": "f32" if g == 4 else "%s gradients, f32 accumulate/update" % p.grad_dtype,
        "mode": mode, "launches_per_step": nl, "bytes_per_element": bpe, "bytes_per_step": step_bytes,
        "tile_elems": ctx.tile_elems, "tiles_per_workgroup": tpw or "default", "workgroups_per_cu": wgs,
        "vectors_per_step": args.vectors_per_step or "default", "autotune_cold_ms": tuned,
        "ms_per_step": round(cold_ms, 5), "ms_per_step_min": round(min(cold), 5),
        "ms_per_step_max": round(max(cold), 5), "GBps": round(gbps, 1),
        "frac_of_8TBps": round(gbps / HBM_PEAK_GBPS, 4),
        "back_to_back": None if args.no_back_to_back else {
            "ms_per_step": round(wall_b2b, 5), "event_ms_per_step": round(ev_b2b, 5),
            "GBps": round(step_bytes / (wall_b2b * 1e-3) / 1e9, 1)},
        "plan_us": round(plan_us, 2), "plan_us_through_python_binding": round(plan_us_binding, 2),
    }
    if not args.no_launch_forms and mode == "pipeline" and G > 0:
        res["launch_forms"] = launch_forms(dm, p, merged, G, scrub, cold_ms, max(5, args.steps // 3))
    if args.all_modes or (headline and not args.no_other_modes):
        ctx.set_pacing(0, args.vectors_per_step)          # every other kind at the library's own pacing
        others = {}
        for m in ("pipeline", "direct", "pack", "reduce", "unpack_update", "reduce_update", "staged"):
            if m == mode:
                continue
            ms = statistics.median(time_cold(lambda: run_step(dm, m, p.lr, p.momentum, G), scrub,
                                             max(10, args.steps // 2), 2))
            b = bytes_per_element(m, p.P, g) * E
            others[m] = {"ms_per_step": round(ms, 5), "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                         "frac_of_8TBps": round(b / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                         "bytes_per_element": bytes_per_element(m, p.P, g), "launches_per_step": launches_per_step(m, G)}
        res["other_modes_cold"] = others
    extra = {"profile": p, "merged": merged, "flats": flats, "step_bytes": step_bytes}
    ctx.close()
    del dm
    torch.cuda.empty_cache()
    return res, extra


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30, help="timed steps per measurement (each with its own events)")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vgg16", help="headline workload")
    ap.add_argument("--also", default="resnet50,transformer,tiny_layers,toy_mlp",
                    help="comma-separated workloads timed the same way and reported under `workloads` ('' = none)")
    ap.add_argument("--mode", default="pipeline",
                    choices=["pipeline", "pipeline_per_group", "direct", "pack", "reduce", "unpack_update",
                             "reduce_update", "staged", "staged_per_group"])
    ap.add_argument("--workers", type=int, default=0,
                    help="override the profile's worker count P (1 = the share one GPU of a data-parallel job holds)")
    ap.add_argument("--all-modes", action="store_true",
                    help="time the other modes (pack, reduce, unpack_update, ... each alone), cold, for every workload "
                         "and not only for the headline one")
    ap.add_argument("--no-other-modes", action="store_true", help="skip the other modes also for the headline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-launch-forms", action="store_true")
    ap.add_argument("--no-ceiling", action="store_true")
    ap.add_argument("--no-back-to-back", action="store_true",
                    help="skip the back-to-back loop (a profiler then sees cold launches only)")
    ap.add_argument("--blocks-per-cu", type=int, default=0)
    ap.add_argument("--xcd-contiguous", action="store_true")
    ap.add_argument("--tiles-per-workgroup", type=int, default=0,
                    help="consecutive tiles per workgroup; 0 = library default")
    ap.add_argument("--workgroups-per-cu", default="auto",
                    help="pacing: workgroups (of one wavefront) a compute unit may hold; 'auto' = pick among the library "
                         "default, 14, 18, 21 and no cap by timing a few cold steps first, 'default' = library default, "
                         "n = fixed, -1 = no cap")
    ap.add_argument("--vectors-per-step", type=int, default=0,
                    help="pacing: 0 = library default, 1 = paced walk for every launch, -1 = burst form for every launch")
    ap.add_argument("--resident-mib", type=int, default=-1,
                    help="MiB of w+v kept cacheable (library default, 0, if negative)")
    ap.add_argument("--copy-calibration", type=float, default=0.0, metavar="GiB",
                    help="instead of the benchmark, run a plain device copy of this many GiB `--steps` times "
                         "(reference dispatch of known size for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--grad-dtype", default="profile", choices=("profile", "f32", "bf16", "f16"),
                    help="gradient type of every workload: the profile's own, or binary32 / bfloat16 / IEEE binary16 "
                         "(the half precision of the paper's mixed-precision runs)")
    ap.add_argument("--small-launch-study", action="store_true",
                    help="instead of the benchmark, time single launches of the fused pipeline over 2 Ki .. 8 Mi "
                         "elements (one tensor, P = 8, binary32, cold cache, HIP events) in the paced and in the "
                         "burst form: where the library's threshold for small launches comes from")
    ap.add_argument("--probe-mix", default="", metavar="R,W,X",
                    help="instead of the benchmark, run the bench aid's bare stream pattern with R read-only, W "
                         "write-only and X updated arrays of 512 MiB each `--steps` times (reference dispatches "
                         "for counter studies)")
    ap.add_argument("--probe-paced", default="", metavar="LANES,VECTORS,LDS_KIB",
                    help="with --probe-mix: walk the arrays one at a time in workgroups of LANES lanes and VECTORS "
                         "vectors per lane, with LDS_KIB KiB of unused LDS per workgroup as occupancy cap")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path is per-GPU; nothing is sharded or "
              "exchanged between GPUs). Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    if args.copy_calibration > 0:
        nbytes = int(args.copy_calibration * (1 << 30))
        src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        print(json.dumps({"calibration": "plain device copy", "bytes_read": nbytes, "bytes_written": nbytes,
                          "launches": args.steps, "ms_per_copy": round(ms, 4),
                          "GBps": round(2 * nbytes / ms / 1e6, 1)}))
        return 0

    if args.small_launch_study:
        import statistics
        import paper_1912_09268_amd as M
        from paper_1912_09268_amd import harness as H
        scrub = Scrubber()
        rows = []
        for kelems in (2, 32, 128, 256, 512, 768, 1024, 1536, 2048, 4096, 8192):     # Ki elements in the launch
            ctx = M.Context([kelems * 1024], [0], 8, M.F32)
            dm = H.DeviceModel(ctx, [kelems * 1024])
            tiles = ctx.n_tiles
            for w in range(8):
                dm.grads[w][0].normal_(0.0, 1e-2)
            dm.w[0].normal_()
            dm.v[0].zero_()
            row = {"tiles": tiles, "elements": kelems * 1024}
            for form, vectors in (("paced", 0), ("burst", -1)):
                ctx.set_small_launch(0)
                ctx.set_pacing(0, vectors)
                ms = time_cold(lambda: run_step(dm, "pipeline", 0.1, 0.9, 1), scrub, args.steps, args.warmup)
                row[form + "_us"] = round(1e3 * statistics.median(ms), 2)
            rows.append(row)
            ctx.close()
            del dm
        print(json.dumps({"small_launch_study": "fused pipeline, one tensor of `tiles` tiles, P = 8, "
                          "binary32, one launch per step, cache scrubbed before each, median of per-step HIP-event "
                          "pairs (which include a few us of launch floor)", "steps": args.steps, "rows": rows}))
        return 0

    if args.probe_mix:
        import bench_aid as A
        mix = [int(x) for x in args.probe_mix.split(",")]
        n = 128 << 20
        tensors = [[torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(c)] for c in mix]
        ptrs = [[t.data_ptr() for t in group] for group in tensors]
        stream = int(torch.cuda.current_stream().cuda_stream)
        if args.probe_paced:
            lanes, vecs, kib = [int(x) for x in args.probe_paced.split(",")]

            def probe():
                A.paced_probe(ptrs[0], ptrs[1], ptrs[2], n, lanes, vecs, kib << 10, stream)
        else:
            def probe():
                A.stream_probe(ptrs[0], ptrs[1], ptrs[2], n, stream)
        probe()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            probe()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        nbytes = 4 * n * (mix[0] + mix[1] + 2 * mix[2])
        print(json.dumps({"probe_mix": mix, "paced": args.probe_paced or None, "bytes_per_launch": nbytes,
                          "launches": args.steps + 1,
                          "ms_per_launch": round(ms, 4), "GBps": round(nbytes / ms / 1e6, 1)}))
        return 0

    scrub = Scrubber()
    head, extra = measure_workload(args.workload, args, scrub, headline=True)
    others = {}
    for name in [x for x in args.also.split(",") if x and x != args.workload]:
        others[name], _ = measure_workload(name, args, scrub, headline=False)

    ceiling = None if args.no_ceiling else pattern_ceiling(head["P"])
    refs = {} if args.no_ceiling else achievable_references(head["P"])
    nl = head["launches_per_step"]
    kernel_ms = head["ms_per_step"] / nl
    achieved = (head["bytes_per_step"] / nl) / (kernel_ms * 1e-3) / 1e9
    khash = kernel_source_hash()
    as_measured = args.workers == 0 and args.grad_dtype == "profile"      # the stored figures are for the profiles as they are
    traffic = MEASURED_FABRIC_BYTES.get(khash, {}).get((args.workload, args.mode)) if as_measured else None
    by_name = dict(others)
    by_name[args.workload] = head
    out = {
        "metric": "pack+reduce+unpack GB/s and % of HBM peak on 1 MI355X; plan time (us)",
        "value": head["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if head["dtype"] == "f32" else head["dtype"], "data": "synthetic",
        "config": {"workload": args.workload, "tensors": head["tensors"], "elements": head["elements"],
                   "groups": head["groups"], "P": head["P"], "mode": args.mode, "launches_per_step": nl,
                   "bytes_per_element": head["bytes_per_element"], "tile_elems": head["tile_elems"],
                   "tiles_per_workgroup": head["tiles_per_workgroup"], "workgroups_per_cu": head["workgroups_per_cu"],
                   "vectors_per_step": head["vectors_per_step"], "autotune_cold_ms": head["autotune_cold_ms"],
                   "blocks_per_cu": args.blocks_per_cu or "default", "xcd_contiguous": bool(args.xcd_contiguous),
                   "timing": "median of %d steps, each between its own HIP events on the launch stream and each "
                             "preceded by an untimed 1 GiB cache scrub (512 MiB read + 512 MiB written)" % args.steps},
        "pct_of_8TBps": round(100.0 * head["GBps"] / HBM_PEAK_GBPS, 2),
        "back_to_back": head["back_to_back"],
        "plan_us": head["plan_us"], "plan_us_through_python_binding": head["plan_us_through_python_binding"],
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_is": "bytes at the L2-fabric boundary per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, "
                                   "scaled by a plain copy), in front of the memory-side cache; null if "
                                   "csrc/kernels.hip changed since it was measured",
                     "kernel_source_blob": khash,
                     "kernel": "mgwfbp_stream_kernel<%s>" % args.mode, "avg_launch_ms": round(kernel_ms, 5),
                     "algorithmic_bytes_per_launch": head["bytes_per_step"] // nl,
                     "bare_pattern_GBps": None if ceiling is None else round(ceiling, 1),
                     **refs},
        "target_70pct": {k: by_name[k]["frac_of_8TBps"] for k in ("resnet50", "vgg16") if k in by_name},
        "launch_forms": head.get("launch_forms"),
        "workloads": others,
        "paper_context": PAPER_CONTEXT,
    }
    if "other_modes_cold" in head:
        out["other_modes_cold"] = head["other_modes_cold"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(extra["profile"], extra["merged"], extra["flats"], extra["step_bytes"])
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
