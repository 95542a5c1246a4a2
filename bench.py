#!/usr/bin/env python3
"""Benchmark of libheinsen on one MI355X.

A step is one pass of the whole hot path (one heinsen_scan call: load + encode, fused scan, carry,
decode + store) over one batch of synthetic input that is already resident in HBM.  The headline
workload is the largest single-GPU configuration, [B=16, n=16384, D=2048] float32 with mixed signs
(configuration 5); the other configurations are timed the same way and reported under
"other_workloads", each with a roofline block of its own.

Prints ONE JSON line: recurrence elements per second, the HBM roofline of the dominant (only) kernel
measured with HIP events on the launch stream, streaming yardsticks measured in the same run through
torch alone (out = a + b, copy), and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth



def measured_traffic(index):
    """HBM bytes per launch of configuration `index` as measured with rocprofv3 --pmc (FETCH_SIZE and
    WRITE_SIZE, scaled by what the same counters read for a copy of known size), read from the summary
    under profiles/ (a line `TRAFFIC_BYTES_PER_LAUNCH read=<int> write=<int>`); None if there is none."""
    import re

    path = os.path.join(ROOT, "profiles", f"hbm_traffic_cfg{index}.txt")
    try:
        m = re.search(r"TRAFFIC_BYTES_PER_LAUNCH\s+read=(\d+)\s+write=(\d+)", open(path).read())
    except OSError:
        return None
    return int(m.group(1)) + int(m.group(2)) if m else None


def device_inputs(cfg, torch, distinct=2):
    """Full-size device tensors for `cfg`: `distinct` generated batch items, repeated to B items.

    Generating every batch item on the host would take minutes for the 5e8-element workloads; the
    repeated items have the same distributions and the kernels do not depend on the values."""
    import numpy as np

    from paper_2311_06281_amd import workloads

    k = min(distinct, cfg.B)
    batch = workloads.generate(cfg, 0, k)
    reps = (cfg.B + k - 1) // k

    def up(arr, dtype=None):
        t = torch.from_numpy(arr).cuda()
        t = t.repeat((reps,) + (1,) * (t.dim() - 1))[: cfg.B].contiguous()
        return t

    if cfg.bf16:
        a = up(batch.a_bits.view(np.int16))
        b = up(batch.b_bits.view(np.int16))
    else:
        a = up(batch.a)
        b = up(batch.b)
    if cfg.x0_scalar:
        x0 = torch.from_numpy(batch.x0).cuda()
    else:
        x0 = torch.from_numpy(batch.x0).cuda().reshape(k, cfg.D).repeat(reps, 1)[: cfg.B].contiguous().reshape(-1)
    out = torch.empty(a.shape, dtype=torch.float32, device="cuda")
    return a, b, x0, out


def time_workload(cfg, torch, hb, steps, warmup, yardsticks=True):
    """Times `steps` calls after `warmup` untimed ones.  Returns a dict: wall ms per step (host clock around
    the synchronised region), mean kernel ms over the timed region (one pair of HIP events on the launch
    stream around the `steps` launches), per-launch event statistics from a second pass, and, for float32
    workloads, what torch's own out = a + b and copy reach on the same buffers."""
    a, b, x0, out = device_inputs(cfg, torch)
    layout = hb.LAYOUTS[cfg.layout]
    flags = hb.flags_from_names(cfg.flags)
    stream = torch.cuda.current_stream()

    def step():
        hb.heinsen_scan(a, b, x0, out, cfg.B, cfg.D, cfg.n, layout, flags, stream)

    def region(fn, n):
        first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        first.record(stream)
        for _ in range(n):
            fn()
        last.record(stream)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n, first.elapsed_time(last) / n

    # Settling: after an idle spell the first dozen launches run up to 10 % slower than the steady state (the
    # chip's power management is still moving its clocks: the per-launch times fall from launch to launch and
    # level off after about 15 launches).  What is measured here is sustained throughput, so the clocks are
    # given about 40 ms of this kernel to settle before the W warm-up steps and the K timed ones.
    t0 = time.perf_counter()
    for _ in range(5):
        step()
    torch.cuda.synchronize()
    est = max((time.perf_counter() - t0) / 5, 1e-6)
    settle = int(min(2000, max(20, 0.04 / est)))
    for _ in range(settle):
        step()
    torch.cuda.synchronize()
    for _ in range(warmup):
        step()
    wall_ms, kern_ms = region(step, steps)
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    for i in range(steps):
        starts[i].record(stream)
        step()
        ends[i].record(stream)
    torch.cuda.synchronize()
    each = sorted(s.elapsed_time(e) for s, e in zip(starts, ends))
    res = {"wall_ms": wall_ms, "kernel_ms": kern_ms, "each_mean": sum(each) / len(each),
           "each_median": each[len(each) // 2], "each_min": each[0], "stream": None, "settle_launches": settle + 5}
    if yardsticks and not cfg.bf16:
        reps = max(3, min(steps, 10))
        for _ in range(20):
            torch.add(a, b, out=out)
        _, add_ms = region(lambda: torch.add(a, b, out=out), reps)
        for _ in range(20):
            out.copy_(a)
        _, copy_ms = region(lambda: out.copy_(a), reps)
        E = cfg.elements
        res["stream"] = {"torch_add_GBps": 12 * E / (add_ms * 1e-3) / 1e9, "torch_copy_GBps": 8 * E / (copy_ms * 1e-3) / 1e9,
                         "note": "torch.add(a, b, out=o) and o.copy_(a) on this workload's own buffers, same run"}
    del a, b, x0, out
    torch.cuda.empty_cache()
    return res


def roofline_block(cfg, hb, t):
    """The roofline entry of one workload from time_workload's result."""
    alg_bytes = cfg.bytes_per_element * cfg.elements
    achieved = alg_bytes / (t["kernel_ms"] * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": measured_traffic(cfg.index), "algorithmic_bytes": alg_bytes,
            "kernel": hb.heinsen_kernel_name(cfg.B, cfg.D, cfg.n, hb.LAYOUTS[cfg.layout], hb.flags_from_names(cfg.flags)),
            "kernel_ms_mean": t["kernel_ms"], "kernel_ms_each_mean": t["each_mean"], "kernel_ms_each_median": t["each_median"],
            "kernel_ms_each_min": t["each_min"], "untimed_settling_launches": t["settle_launches"],
            "stream_ceiling": t["stream"]}


def arithmetic_dtype(cfg):
    return "f32" if not cfg.bf16 else "f32 (a, b stored as bf16)"


def cpu_baseline(cfg):
    """The CPU oracle as it stands, on the host cores, on the same workload (bounded sample)."""
    import oracle
    from paper_2311_06281_amd import workloads

    nb = min(cfg.B, 2)
    batch = workloads.generate(cfg, 0, nb)
    layout = oracle.LAYOUT_BND if cfg.layout == "BND" else oracle.LAYOUT_BDN
    fn = oracle.sequential_log if cfg.log_domain else oracle.sequential
    elements = nb * cfg.D * cfg.n
    cores = max(1, min(oracle.max_threads(), os.cpu_count() or 1))
    fn(batch.a, batch.b, batch.x0, layout=layout, threads=cores)  # warm the pages
    best = {}
    for threads in (1, cores):
        reps, t_best, t_total = 0, float("inf"), 0.0
        while reps < 3 or (t_total < 5.0 and reps < 50):
            t0 = time.perf_counter()
            fn(batch.a, batch.b, batch.x0, layout=layout, threads=threads)
            dt = time.perf_counter() - t0
            t_best = min(t_best, dt)
            t_total += dt
            reps += 1
        best[threads] = elements / t_best
    return {"value": best[cores], "unit": "elements/s", "cores": cores, "kind": "oracle",
            "sample": f"float64 sequential recurrence on {nb} of {cfg.B} batch items of the same workload "
                      f"({elements} elements), best of repeated runs, channels split over {cores} threads",
            "single_thread_value": best[1]}


def fig1_sweep(torch, hb, runs=30):
    """The paper's one experiment (Sec. 4, Fig. 1) on this GPU: time to compute n elements sequentially
    relative to the parallel computation, one sequence, n = 2^4 .. 2^26, mean of `runs` runs per point
    (fewer for the long sequential runs).  Inputs: the single-sequence workload (a ~ U(0.5,1),
    b ~ U(0,1), x0 = 1).  Also timed: the float64 CPU oracle on one host thread."""
    import math

    import oracle
    from paper_2311_06281_amd import workloads

    base = workloads.CONFIGS[1]
    stream = torch.cuda.current_stream()
    flags = hb.flags_from_names(base.flags)
    points = []
    for lg in range(4, 27):
        n = 1 << lg
        cfg = base.scaled(n=n)
        batch = workloads.generate(cfg)
        a = torch.from_numpy(batch.a).cuda()
        b = torch.from_numpy(batch.b).cuda()
        x0 = torch.from_numpy(batch.x0).cuda()
        out = torch.empty_like(a)

        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for s, e in ev:
                s.record(stream)
                fn()
                e.record(stream)
            torch.cuda.synchronize()
            return sum(s.elapsed_time(e) for s, e in ev) / reps * 1e3  # microseconds

        t_par = timed(lambda: hb.heinsen_scan(a, b, x0, out, 1, 1, n, hb.HEINSEN_LAYOUT_BDN, flags, stream), runs)
        seq_reps = runs if lg <= 20 else (5 if lg <= 23 else 2)
        t_seq = timed(lambda: hb.heinsen_sequential(a, b, x0, out, n, stream), seq_reps)
        a64 = batch.a.reshape(-1).astype("float64")
        b64 = batch.b.reshape(-1).astype("float64")
        t_cpu = float("inf")
        for _ in range(3):
            t0 = time.perf_counter()
            oracle.seq_f64(a64, b64, 1.0)
            t_cpu = min(t_cpu, (time.perf_counter() - t0) * 1e6)
        points.append({"n": n, "parallel_us": t_par, "sequential_gpu_us": t_seq, "sequential_cpu_us": t_cpu,
                       "ratio_gpu": t_seq / t_par, "ratio_cpu": t_cpu / t_par, "n_over_log2n": n / math.log2(n),
                       "sequential_runs": seq_reps})
        del a, b, x0, out
    return points


def tile_timeline(cfg, torch, hb, launches=4):
    """Per-tile view of one launch of a carry-chained kernel (heinsen_set_timeline): where a tile's life
    goes between its workgroup's start and its last store, and how the launch ramps up and drains.
    Returns a text report (times in microseconds; the GPU's wall clock ticks at 100 MHz)."""
    import numpy as np

    a, b, x0, out = device_inputs(cfg, torch)
    layout, flags = hb.LAYOUTS[cfg.layout], hb.flags_from_names(cfg.flags)
    stream = torch.cuda.current_stream()
    cap = 1 << 20
    stamps = torch.zeros(cap * 8, dtype=torch.int64, device="cuda")
    for _ in range(3):
        hb.heinsen_scan(a, b, x0, out, cfg.B, cfg.D, cfg.n, layout, flags, stream)
    torch.cuda.synchronize()
    hb.heinsen_set_timeline(stamps, cap)
    try:
        for _ in range(launches):
            stamps.zero_()
            hb.heinsen_scan(a, b, x0, out, cfg.B, cfg.D, cfg.n, layout, flags, stream)
            torch.cuda.synchronize()
    finally:
        hb.heinsen_set_timeline(None, 0)
    t = stamps.cpu().numpy().reshape(cap, 8).astype(np.float64)
    t = t[t[:, 7] > 0]
    nt = t.shape[0]
    t = (t - t[:, 0].min()) * 0.01
    names = ["workgroup start -> ticket drawn", "ticket -> inputs loaded and scanned", "scanned -> summary handed on",
             "summary -> carry records in", "records in -> start state known", "state -> outputs issued",
             "outputs issued -> end"]
    lines = [f"workload cfg{cfg.index} {cfg.shape()} {cfg.layout}: {nt} tiles stamped, kernel "
             f"{hb.heinsen_kernel_name(cfg.B, cfg.D, cfg.n, layout, flags)}",
             f"launch span (first workgroup start -> last tile end): {t[:, 7].max():.1f} us",
             f"{'phase':46s} {'mean':>7s} {'p50':>7s} {'p90':>7s} {'max':>7s}"]
    for i, nm in enumerate(names):
        d = t[:, i + 1] - t[:, i]
        lines.append(f"{nm:46s} {d.mean():7.2f} {np.median(d):7.2f} {np.percentile(d, 90):7.2f} {d.max():7.2f}")
    if cfg.layout == "BDN" and cfg.B * cfg.D == 1:
        # one row: tile i needs the summaries of all tiles before it.  How long after the last of them was
        # handed on does tile i know its start state?  (the latency of the carry tree itself, as opposed to
        # waiting for predecessors that are still loading)
        handed = np.maximum.accumulate(t[:, 3])
        lag = (t[:, 5] - np.maximum(handed, t[:, 3]))[1:]
        own = (handed - t[:, 3])[1:]
        lines.append(f"{'own summary -> summary of the last predecessor':46s} {own.mean():7.2f} {np.median(own):7.2f} {np.percentile(own, 90):7.2f} {own.max():7.2f}")
        lines.append(f"{'all summaries handed on -> start state known':46s} {lag.mean():7.2f} {np.median(lag):7.2f} {np.percentile(lag, 90):7.2f} {lag.max():7.2f}")
    life = t[:, 7] - t[:, 0]
    lines.append(f"{'tile life (start -> end)':46s} {life.mean():7.2f} {np.median(life):7.2f} {np.percentile(life, 90):7.2f} {life.max():7.2f}")
    starts, ends = np.sort(t[:, 0]), np.sort(t[:, 7])
    resident = int(np.sum(starts <= starts[0] + 1e-9 + np.median(life) * 0.25))
    k = min(nt - 1, 511)
    lines.append(f"ramp: workgroup start of tile #1 at 0.0, #{k + 1} at {starts[k]:.1f} us; first ticket at {np.sort(t[:, 1])[0]:.1f}, "
                 f"#{k + 1} ticket at {np.sort(t[:, 1])[k]:.1f} us  ({resident} workgroups started within a quarter of a tile life)")
    lines.append(f"drain: last workgroup start at {starts[-1]:.1f} us, first tile end {ends[0]:.1f}, median end {np.median(ends):.1f}, "
                 f"last end {ends[-1]:.1f} us -> {ends[-1] - starts[-1]:.1f} us with no new tile starting")
    grid = np.linspace(0, ends[-1], 21)
    alive = [int(np.sum((t[:, 0] <= g) & (t[:, 7] > g))) for g in grid]
    lines.append("tiles alive at 5 % steps of the span: " + " ".join(str(v) for v in alive))
    del a, b, x0, out, stamps
    torch.cuda.empty_cache()
    return "\n".join(lines)


def stream_probe(cfg, torch, hb, runs=20):
    """Ceilings of the access patterns (heinsen_stream_probe: out = a + b, nothing else) on buffers of
    configuration `cfg`'s size, beside torch's own add and copy.  Returns a text report."""
    B, n, D = cfg.B, cfg.n, cfg.D
    E = B * n * D
    a = torch.rand(E, dtype=torch.float32, device="cuda")
    b = torch.rand(E, dtype=torch.float32, device="cuda")
    out = torch.empty_like(a)
    stream = torch.cuda.current_stream()

    def timed(fn, nbytes):
        for _ in range(40):
            fn()
        first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        first.record(stream)
        for _ in range(runs):
            fn()
        last.record(stream)
        torch.cuda.synchronize()
        ms = first.elapsed_time(last) / runs
        return ms * 1e3, nbytes / (ms * 1e-3) / 1e9

    names = ["one long vector, 16 B per lane", "tiles 64 ch x 256 steps (rows of 256 B)", "tiles 128 ch x 128 steps (rows of 512 B)",
             "tiles 256 ch x 64 steps (rows of 1 KiB)", "64 x 256, stores after all loads", "128 x 128, stores after all loads",
             "256 x 64, stores after all loads"]
    lines = [f"out = a + b on [B={B}, n={n}, D={D}] float32 ({12 * E / 1e6:.0f} MB per launch), mean of {runs} launches after 40 untimed ones"]
    for pat, nm in enumerate(names):
        if cfg.layout == "BDN" and pat > 0:
            continue  # the tile patterns are those of the [B, n, D] kernel
        if hb.heinsen_stream_probe_status(a, b, out, B, n, D, pat, stream) != hb.HEINSEN_OK:
            lines.append(f"  heinsen_stream_probe {pat}: {nm:44s} not applicable to this shape")
            continue
        us, gbs = timed(lambda: hb.heinsen_stream_probe_status(a, b, out, B, n, D, pat, stream), 12 * E)
        lines.append(f"  heinsen_stream_probe {pat}: {nm:44s} {us:8.1f} us  {gbs:6.0f} GB/s  {gbs / HBM_PEAK_GBS:.3f} of peak")
    if cfg.bf16:
        ah, bh = a.to(torch.bfloat16), b.to(torch.bfloat16)
        us, gbs = timed(lambda: hb.heinsen_stream_probe_status(ah, bh, out, B, n, D, 7, stream), 8 * E)
        lines.append(f"  heinsen_stream_probe 7: {'one long vector, bf16 in, float32 out (8 B/element)':44s} {us:8.1f} us  {gbs:6.0f} GB/s  "
                     f"{gbs / HBM_PEAK_GBS:.3f} of peak")
        del ah, bh
    us, gbs = timed(lambda: torch.add(a, b, out=out), 12 * E)
    lines.append(f"  torch.add(a, b, out=o)  {'':47s} {us:8.1f} us  {gbs:6.0f} GB/s  {gbs / HBM_PEAK_GBS:.3f} of peak")
    us, gbs = timed(lambda: out.copy_(a), 8 * E)
    lines.append(f"  o.copy_(a)              {'':47s} {us:8.1f} us  {gbs:6.0f} GB/s  {gbs / HBM_PEAK_GBS:.3f} of peak")
    return "\n".join(lines)


def flag_sweep(cfg, torch, hb, runs=30):
    """The workload's shape, layout and storage type with other flag sets, i.e. the same bytes with less (or
    other) arithmetic: tells whether the kernel is bound by memory or by its instructions.  Inputs are the
    workload's own buffers, read as whatever the flags say (timing only).  Returns a text report."""
    a, b, x0, out = device_inputs(cfg, torch)
    stream = torch.cuda.current_stream()
    layout = hb.LAYOUTS[cfg.layout]
    store = hb.HEINSEN_IN_BF16 if cfg.bf16 else 0
    sets = [("the workload's own flags", hb.flags_from_names(cfg.flags)),
            ("LOG_INPUTS (logs in, x out: one log-add-exp less per element)", hb.HEINSEN_LOG_INPUTS | store),
            ("POSITIVE (x in, x out)", hb.HEINSEN_POSITIVE | store),
            ("signed (x in, x out, signs tracked)", store),
            ("LINEAR (no logarithm or exponential at all)", hb.HEINSEN_LINEAR | store)]
    lines = [f"workload cfg{cfg.index} {cfg.shape()} {cfg.layout}, {cfg.bytes_per_element} B/element, mean of {runs} launches after 50 ms of untimed ones"]
    for name, flags in sets:
        fn = lambda: hb.heinsen_scan(a, b, x0, out, cfg.B, cfg.D, cfg.n, layout, flags, stream)
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < 0.05:  # let the clocks settle (see time_workload)
            for _ in range(20):
                fn()
            torch.cuda.synchronize()
        first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        first.record(stream)
        for _ in range(runs):
            fn()
        last.record(stream)
        torch.cuda.synchronize()
        ms = first.elapsed_time(last) / runs
        gbs = cfg.bytes_per_element * cfg.elements / (ms * 1e-3) / 1e9
        lines.append(f"  {name:64s} {ms * 1e3:8.1f} us  {gbs:6.0f} GB/s  {gbs / HBM_PEAK_GBS:.3f} of peak  "
                     f"({hb.heinsen_kernel_name(cfg.B, cfg.D, cfg.n, layout, flags)})")
    del a, b, x0, out
    torch.cuda.empty_cache()
    return "\n".join(lines)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)   # the paper's protocol: mean of 30 runs (Fig. 1)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=5, help="headline benchmark configuration 1..5 (default 5, the largest)")
    ap.add_argument("--no-others", action="store_true", help="time only the headline workload")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--fig1", action="store_true",
                    help="instead of the benchmark, run the paper's sequential-vs-parallel sweep over n (Fig. 1)")
    ap.add_argument("--timeline", type=int, default=0, metavar="CFG",
                    help="instead of the benchmark, print the per-tile timeline of one launch of configuration CFG (2, 3 or 5)")
    ap.add_argument("--stream-probe", type=int, default=0, metavar="CFG",
                    help="instead of the benchmark, measure the streaming ceilings of the access patterns on CFG's size")
    ap.add_argument("--flag-sweep", type=int, default=0, metavar="CFG",
                    help="instead of the benchmark, time configuration CFG's shape with flag sets of less arithmetic")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain device copies of a known size (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2

    import torch

    from paper_2311_06281_amd import binding as hb
    from paper_2311_06281_amd import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    hb.load()  # no fallback: raises if the HIP library is missing
    torch.cuda.set_device(0)

    if args.fig1:
        print(json.dumps({"experiment": "time(sequential) / time(parallel) vs n, one sequence, one MI355X",
                          "runs_per_point": 30, "points": fig1_sweep(torch, hb)}))
        return 0

    if args.timeline:
        print(tile_timeline(workloads.CONFIGS[args.timeline], torch, hb))
        return 0

    if args.stream_probe:
        print(stream_probe(workloads.CONFIGS[args.stream_probe], torch, hb))
        return 0

    if args.flag_sweep:
        print(flag_sweep(workloads.CONFIGS[args.flag_sweep], torch, hb))
        return 0

    if args.copy_calibration:
        # 5 plain copies of 2^25 float32 (128 MiB read + 128 MiB written each): the HBM byte counters of
        # this kernel, divided by its known size, give the scale factor for the scan kernel's counters
        src = torch.ones(1 << 25, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cfg = workloads.CONFIGS[args.workload]
    # under a counter-collecting profiler (--copy-calibration) only the library's own kernels and the copies run
    t = time_workload(cfg, torch, hb, args.steps, args.warmup, yardsticks=not args.copy_calibration)
    E = cfg.elements
    result = {
        "metric": "recurrence elements/sec",
        "value": E / (t["wall_ms"] * 1e-3),
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": t["wall_ms"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": arithmetic_dtype(cfg),
        "data": "synthetic",
        "config": {"workload": f"cfg{cfg.index}: {cfg.name}", "B": cfg.B, "D": cfg.D, "n": cfg.n,
                   "layout": cfg.layout, "flags": list(cfg.flags), "bytes_per_element": cfg.bytes_per_element},
        "roofline": roofline_block(cfg, hb, t),
    }
    props = torch.cuda.get_device_properties(0)
    result["device"] = {"name": props.name, "arch": getattr(props, "gcnArchName", None), "compute_units": props.multi_processor_count}
    if not args.no_others:
        others = []
        for idx in (2, 4, 3, 1, 5):
            if idx == cfg.index:
                continue
            c = workloads.CONFIGS[idx]
            to = time_workload(c, torch, hb, args.steps, args.warmup)
            others.append({"workload": f"cfg{idx}: {c.name}", "dtype": arithmetic_dtype(c),
                           "elements_per_s": c.elements / (to["wall_ms"] * 1e-3), "ms_per_step": to["wall_ms"],
                           "bytes_per_element": c.bytes_per_element, "roofline": roofline_block(c, hb, to)})
        result["other_workloads"] = others
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
