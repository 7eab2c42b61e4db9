"""Benchmark of the merged-gradient hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet50] [--mode pipeline]

A step is one pass of the whole device path over one synthetic batch of gradients: every group of the
plan is packed into the P merge arenas, reduced (sum over the P simulated workers, times 1/P) and
applied to the per-layer weights and momenta.  Inputs are resident in HBM before the timed region.
The plan itself is computed once per training run; its time is reported separately as `plan_us`.

Prints ONE JSON line.  `value` is algorithmic bytes of the path that ran divided by the time per step.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM-side bytes per launch measured with rocprofv3 (--pmc FETCH_SIZE, then --pmc WRITE_SIZE, each scaled
# by the same counter's reading for a plain 1 GiB device copy); the runs and the scale factors are in
# profiles/mgwfbp_stream_kernel_<workload>_*.txt.  Only the single-kernel mode has one figure.
MEASURED_TRAFFIC_BYTES = {
    ("resnet50", "pipeline"): 2.0466e9,
    ("vgg16", "pipeline"): 11.0736e9,
    ("transformer", "pipeline"): 16.1089e9,
    ("tiny_layers", "pipeline"): 1.8816e9,
    ("resnet50", "direct"): 1.2287e9,
    ("vgg16", "direct"): 6.6498e9,
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
    mode = mode[:-len("_graph")] if mode.endswith("_graph") else mode
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


def stream_mix(mode: str, P: int):
    """(read-only, write-only, updated-in-place) arrays a single-launch mode streams, or None."""
    return {"pipeline": (P, P, 2), "direct": (P, 0, 2), "pack": (P, P, 0), "reduce": (P, 1, 0),
            "unpack_update": (1, 0, 2)}.get(mode)


def pattern_ceiling(mode: str, P: int, reps: int = 10):
    """What the bare read/write mix of `mode` reaches on this GPU: bench_aid_stream_probe over freshly allocated
    binary32 arrays of 128 Mi elements each (for 16-bit gradients the stream counts are the same, the arrays
    are not halved), timed with HIP events.  Returns GB/s, or None if the mix has no probe instance."""
    import torch
    import bench_aid as A
    mix = stream_mix(mode, P)
    if mix is None or mix[0] not in (0, 1, 2, 4, 8, 16) or mix[1] not in (0, 1, 2, 4, 8, 16):
        return None
    n = 128 << 20
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
    return 4 * n * (mix[0] + mix[1] + 2 * mix[2]) / (ms * 1e-3) / 1e9


def launches_per_step(mode: str, G: int) -> int:
    mode = mode[:-len("_graph")] if mode.endswith("_graph") else mode
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


def time_mode(dm, mode, lr, mu, G, steps, warmup):
    """Returns (wall ms per step, HIP-event ms per step).  Events sit on torch's current stream, which
    is the stream handed to the library.  A mode ending in `_graph` captures one step of the base mode
    into a HIP graph once and replays it."""
    import torch
    if mode.endswith("_graph"):
        base = mode[:-len("_graph")]
        run_step(dm, base, lr, mu, G)            # warm up outside capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run_step(dm, base, lr, mu, G)
        step = graph.replay
    else:
        def step():
            run_step(dm, mode, lr, mu, G)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return wall, e0.elapsed_time(e1) / steps


def autotune_launch(ctx, dm, mode, lr, mu, G, blocks_per_cu, xcd, candidates=(1, 2, 4), steps=8):
    """Pick tiles-per-workgroup by timing real steps.  Results do not depend on the launch shape (every
    element is computed by the same instruction sequence whatever workgroup handles it), so a training
    loop can do the same during its first iterations at no cost."""
    best, best_ms, seen = candidates[0], None, {}
    for k in candidates:
        ctx.set_launch(blocks_per_cu, xcd, k)
        _, ms = time_mode(dm, mode, lr, mu, G, steps, 2)
        seen[k] = round(ms, 5)
        if best_ms is None or ms < best_ms * 0.995:      # prefer the earlier candidate on a tie
            best, best_ms = k, ms
    ctx.set_launch(blocks_per_cu, xcd, best)
    return best, seen


def _cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(profile, merged, bytes_per_step, budget_s=10.0):
    """The oracle as it stands, timed on this host for whole steps until `budget_s` is used up."""
    import numpy as np
    import workloads as W
    from oracle import pipeline as OD
    from oracle import plan as OP
    groups = OP.groups_in_arrival_order([int(x) for x in merged])
    flats = [W.worker_gradient_flat(profile, w) for w in range(profile.P)]
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
    return {"plan_us": round(statistics.median(plan_times), 1), "value": bytes_per_step / best / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{len(times)} full step(s) of the {profile.name} workload (all groups, P={profile.P}) in "
                      f"{sum(times):.1f} s of CPU time; "
                      f"best {best * 1e3:.0f} ms/step; same byte count as `value`",
            "ms_per_step": best * 1e3, "host_cpus": os.cpu_count(), "cpu_model": _cpu_model()}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet50")
    ap.add_argument("--mode", default="pipeline",
                    choices=["pipeline", "pipeline_per_group", "direct", "pack", "reduce", "unpack_update",
                             "reduce_update", "staged", "staged_per_group",
                             "pipeline_per_group_graph", "staged_per_group_graph"])
    ap.add_argument("--workers", type=int, default=0,
                    help="override the profile's worker count P (1 = the share one GPU of a data-parallel job holds)")
    ap.add_argument("--all-modes", action="store_true", help="also time the other launch modes (extra keys)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--blocks-per-cu", type=int, default=0)
    ap.add_argument("--xcd-contiguous", action="store_true")
    ap.add_argument("--tiles-per-workgroup", type=int, default=-1,
                    help="consecutive tiles per workgroup; 0 = library default, negative = pick 1, 2 or 4 by "
                         "timing a few untimed steps first")
    ap.add_argument("--resident-mib", type=int, default=-1,
                    help="MiB of w+v kept cacheable (library default if negative)")
    ap.add_argument("--copy-calibration", type=float, default=0.0, metavar="GiB",
                    help="instead of the benchmark, run a plain device copy of this many GiB `--steps` times "
                         "(reference dispatch of known size for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path is per-GPU; nothing is sharded or "
              "exchanged between GPUs). Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_1912_09268_amd as M
    import workloads as W
    from paper_1912_09268_amd import harness as H

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

    p = W.make_profile(args.workload)
    if args.workers > 0:
        p = dataclasses.replace(p, P=args.workers)
    n = [int(x) for x in p.n_elems]
    g = p.elem_bytes

    # plan: one-time host computation, timed on its own -- once through the Python binding (argument
    # marshalling included) and once as the bare C-ABI call with the arguments marshalled beforehand
    import ctypes as C
    plan_times = []
    for _ in range(1000 if p.L <= 1000 else 100):
        t0 = time.perf_counter()
        merged, first = M.plan(p.size_bytes, p.t_backward, p.a, p.b)
        plan_times.append((time.perf_counter() - t0) * 1e6)
    plan_us_binding = statistics.median(plan_times)
    sz = np.ascontiguousarray(p.size_bytes, np.uint64)
    tb = np.ascontiguousarray(p.t_backward, np.float64)
    m_out = np.zeros(p.L, np.uint8)
    f_out = np.zeros(p.L + 1, np.int32)
    g_out = C.c_int32(0)
    raw = M.lib().mgwfbp_plan
    c_args = (sz.ctypes.data_as(C.POINTER(C.c_uint64)), tb.ctypes.data_as(C.POINTER(C.c_double)), p.L,
              C.c_double(p.a), C.c_double(p.b), m_out.ctypes.data_as(C.POINTER(C.c_uint8)),
              f_out.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(g_out))
    plan_times = []
    for _ in range(200):
        t0 = time.perf_counter()
        for _ in range(20):
            raw(*c_args)
        plan_times.append((time.perf_counter() - t0) * 1e6 / 20)
    plan_us = statistics.median(plan_times)
    assert m_out.tolist() == merged.tolist()
    G = int(first.shape[0])

    ctx = M.Context(n, merged, p.P, M.BF16 if p.grad_dtype == "bf16" else M.F32)
    ctx.set_launch(args.blocks_per_cu, args.xcd_contiguous, max(args.tiles_per_workgroup, 0))
    if args.resident_mib >= 0:
        ctx.set_resident_bytes(args.resident_mib << 20)
    dm = H.DeviceModel(ctx, n)
    for w in range(p.P):
        dm.upload_grads(w, W.worker_gradient_flat(p, w))
    dm.upload_weights(W.initial_weights_flat(p), W.initial_momentum_flat(p, zero=True))
    torch.cuda.synchronize()

    dm.pack(-1); dm.reduce(-1)                  # so that modes that start mid-path read real data
    torch.cuda.synchronize()

    E = p.total_elems
    tuned = None
    if args.tiles_per_workgroup < 0 and "per_group" not in args.mode:
        tpw, tuned = autotune_launch(ctx, dm, args.mode, p.lr, p.momentum, G, args.blocks_per_cu, args.xcd_contiguous)
    else:
        tpw = max(args.tiles_per_workgroup, 0)
    wall_ms, event_ms = time_mode(dm, args.mode, p.lr, p.momentum, G, args.steps, args.warmup)
    bpe = bytes_per_element(args.mode, p.P, g)
    step_bytes = bpe * E
    value = step_bytes / (wall_ms * 1e-3) / 1e9
    nl = launches_per_step(args.mode, G)
    kernel_ms = event_ms / nl
    achieved = (step_bytes / nl) / (kernel_ms * 1e-3) / 1e9

    # what the same mix of read-only / write-only / updated streams reaches with nothing else in the kernel
    ceiling = pattern_ceiling(args.mode, p.P)

    out = {
        "metric": "pack+reduce+unpack GB/s and % of HBM peak on 1 MI355X; plan time (us)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if g == 4 else "bf16 gradients, f32 accumulate/update", "data": "synthetic",
        "config": {"workload": args.workload, "tensors": p.L, "elements": E, "groups": G, "P": p.P,
                   "mode": args.mode, "launches_per_step": nl, "bytes_per_element": bpe,
                   "tile_elems": ctx.tile_elems, "blocks_per_cu": args.blocks_per_cu or "default",
                   "xcd_contiguous": bool(args.xcd_contiguous),
                   "tiles_per_workgroup": tpw or "default", "autotune_ms": tuned},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "plan_us": round(plan_us, 2), "plan_us_through_python_binding": round(plan_us_binding, 2),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "bare_pattern_GBps": None if ceiling is None else round(ceiling, 1),
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": None if args.workers > 0 else MEASURED_TRAFFIC_BYTES.get((args.workload, args.mode)),
                     "kernel": f"mgwfbp_stream_kernel<{args.mode}>", "avg_launch_ms": round(kernel_ms, 5),
                     "algorithmic_bytes_per_launch": step_bytes // nl},
    }
    out["paper_context"] = PAPER_CONTEXT
    if args.all_modes:
        others = {}
        for mode in ("pipeline", "pipeline_per_group", "pipeline_per_group_graph", "direct", "pack", "reduce",
                     "unpack_update", "reduce_update", "staged",
                     "staged_per_group", "staged_per_group_graph"):
            if mode == args.mode:
                continue
            k = max(10, args.steps // (4 if "per_group" in mode else 1))
            wl, ev = time_mode(dm, mode, p.lr, p.momentum, G, k, max(2, args.warmup // 4))
            b = bytes_per_element(mode, p.P, g) * E
            others[mode] = {"ms_per_step": round(wl, 5), "GBps": round(b / (wl * 1e-3) / 1e9, 1),
                            "bytes_per_element": bytes_per_element(mode, p.P, g),
                            "launches_per_step": launches_per_step(mode, G)}
        out["other_modes"] = others
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(p, merged, step_bytes)
    ctx.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
