#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload default]

A "step" is one pass of the whole hot path over one batch of synthetic input.  For the default
workload that is benchmark configuration 2, the one the metric is quoted on: one 8192x8192 fp32
2D filter pass for each of the seven filter shapes.  The headline `value` is the whole-job
GStencil/s (output points x sweeps / second) of K such steps, timed with the inputs resident in
HBM and rotated among four copies of the image, so that no launch finds its input in the 256 MB
memory-side cache ("cold"); per-kernel figures are given cold and, for context, warm (one input
tensor).  The same default run then times the other benchmark configurations (1, 3, 4, 5), each
case alone for at least --min-case-seconds, one sweep per launch and the way
ssam_stencil_iterate runs it by default, and reports them under "kernels".  Per-launch figures
are medians over groups of launches bracketed by HIP events on the launch stream.

Prints ONE JSON line: metric / value, "roofline" of the dominant kernel of the headline (HIP
events around its launches inside the timed region), "kernels", "parity" (the GPU output of every
configuration-2 case compared in this process with the field the CPU oracle computes for the
"cpu_baseline" leg) and "cpu_baseline" (the oracle timed on a bounded sample).

Other workloads: --workload config1 .. config5, filter_sweep, table3, conv3d (a step is then the whole
configuration: every case, all its sweeps), scan.  --tune "<knob>=v1,v2;<knob2>=..." times the
selected cases under every combination of tuning overrides (ssam_set_tuning) instead, one after the
other in this process (the clock differs between processes and boxes by several per cent, so variants
are only comparable within one run); with --cold the single-pass cases rotate their input as the
default workload does.  The two grids of an iterated case are carved from one allocation, back to back.
"""
from __future__ import annotations

import argparse
import itertools
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0                          # MI355X HBM3E, published
ALU_PEAK_TFLOPS = {"f32": 157.3, "f64": 78.6}   # published vector peaks (fp32 figure assumes packed FMA)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "measured_traffic.json")
COLD_COPIES = 4                                 # distinct input tensors a single-pass case rotates through


def dtype_tag(dt) -> str:
    return "f32" if np.dtype(dt) == np.float32 else "f64"


def case_coef(case):
    return case.coef if case.kind != "stencil2d" else case.coef[0]


def measured_traffic():
    """HBM bytes per launch from rocprofv3 counters, keyed "<kernel instance>@<grid>"; written by
    `python -m paper_1907_06154_amd.profiling` from the counter CSVs (see profiles/)."""
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f).get("bytes_per_launch", {})
    except (OSError, ValueError):
        return {}


def grid_tag(shape) -> str:
    return "x".join(str(s) for s in shape)


class Timer:
    """HIP-event timing on the launch stream."""

    def __init__(self, torch):
        self.torch = torch
        self.stream = torch.cuda.current_stream()

    def pair(self):
        return self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)


def run_single(ssam, case, d_in, d_out):
    if case.kind == "conv2d":
        ssam.ssam_conv2d(d_in, case.coef, case.boundary, d_out=d_out)
    elif case.kind == "conv3d":
        ssam.ssam_conv3d(d_in, case.coef, case.boundary, d_out=d_out)
    elif case.kind == "stencil2d":
        ssam.ssam_stencil2d(d_in, case_coef(case), case.boundary, d_out=d_out)
    else:
        ssam.ssam_stencil3d(d_in, case_coef(case), case.boundary, d_out=d_out)


def grids_back_to_back(torch, like, count):
    """`count` uninitialised grids shaped like `like`, carved from ONE allocation, one after the other --
    the way the two arrays of a Jacobi iteration are normally laid out.  Where separately allocated buffers
    end up is up to the allocator's history, and the time of the bandwidth-bound 3D kernels depends on the
    distance between input and output (512^3 fp64: 361 us back to back, 416 us when 17 MiB further apart)."""
    n = like.numel()
    pool = torch.empty(count * n, dtype=like.dtype, device=like.device)
    return [pool[i * n:(i + 1) * n].view(like.shape) for i in range(count)]


def launches_of(ssam, case):
    """(launches, name of the instance that does most of them, every launch's instance name in order)
    for one ssam_stencil_iterate run of the case under the current tuning, from the planning query (a
    "..._fusedS" launch performs S sweeps)."""
    kind = {"stencil2d": "iterate2d", "stencil3d": "iterate3d"}[case.kind]
    single = ssam.ssam_describe(case.kind, case.shape, case_coef(case), case.boundary).split()[0]
    names, t = [], 0
    while t < case.steps:
        if kind == "iterate2d":
            nm = ssam.ssam_describe(kind, case.shape, case_coef(case), case.boundary, remaining=case.steps - t).split()[0]
        else:   # 3D: pairs of sweeps while two or more remain
            nm = ssam.ssam_describe(kind, case.shape, case_coef(case), case.boundary).split()[0] if case.steps - t >= 2 else single
        t += int(nm.rsplit("_fused", 1)[1]) if "_fused" in nm else 1
        names.append(nm)
    return len(names), max(set(names), key=names.count), names


def time_groups(timer, enqueue_group, launches_per_group: int, min_seconds: float, min_groups: int = 9):
    """Runs groups of launches (enqueue_group() enqueues one group), each bracketed by an event pair,
    until min_seconds of GPU time and min_groups groups are in; returns per-launch milliseconds of
    every group."""
    torch = timer.torch
    per_launch, total_ms = [], 0.0
    while total_ms < min_seconds * 1e3 or len(per_launch) < min_groups:
        batch = []
        for _ in range(8):
            s, e = timer.pair()
            s.record(timer.stream)
            enqueue_group()
            e.record(timer.stream)
            batch.append((s, e))
        torch.cuda.synchronize()
        for s, e in batch:
            ms = s.elapsed_time(e)
            per_launch.append(ms / launches_per_group)
            total_ms += ms
    return per_launch


def kernel_entry(case, kname, launch_ms, launches, traffic, extra=None):
    esz = np.dtype(case.dtype).itemsize
    alg_bytes = case.points * 2 * esz
    flops = case.points * (2 * case.taps - 1) * case.steps / launches
    tag = dtype_tag(case.dtype)
    gbps = alg_bytes / (launch_ms * 1e-3) / 1e9
    tflops = flops / (launch_ms * 1e-3) / 1e12
    t_hbm = alg_bytes / (HBM_PEAK_GBPS * 1e9)
    t_alu = flops / (ALU_PEAK_TFLOPS[tag] * 1e12)
    k = {"case": case.name, "kernel": kname, "launch_ms": launch_ms, "launches_per_step": launches,
         "sweeps_per_launch": case.steps / launches, "gstencil_per_s": case.points * case.steps / (launch_ms * launches) / 1e6,
         "hbm_GBps": gbps, "hbm_frac": gbps / HBM_PEAK_GBPS, "alu_TFLOPs": tflops, "alu_frac": tflops / ALU_PEAK_TFLOPS[tag],
         # arithmetic-bound kernels whose products run on the matrix cores ("...mx") are priced
         # against the dense fp32 MFMA peak, which equals the published fp32 vector peak
         "bound": "hbm" if t_hbm >= t_alu else ("mfma" if kname.split("+")[0].endswith("mx") else "alu"),
         "traffic": traffic.get(f"{kname}@{grid_tag(case.shape)}")}
    if extra:
        k.update(extra)
    return k


def time_single_pass_case(ssam, timer, case, inputs, d_out, min_seconds, traffic):
    """A one-launch case (2D filter, single sweep): cold = inputs rotated per launch, warm = one input."""
    kname = ssam.ssam_describe(case.kind, case.shape, case_coef(case), case.boundary).split()[0]
    n = len(inputs)

    def cold():
        for d_in in inputs:
            run_single(ssam, case, d_in, d_out)

    def warm():
        for _ in range(n):
            run_single(ssam, case, inputs[0], d_out)

    for _ in range(2):
        cold()
    cold_ms = float(np.median(time_groups(timer, cold, n, min_seconds)))
    extra = {"mode": "single_pass", "input": f"rotated among {n} tensors (cold)"}
    if n > 1:
        warm_ms = float(np.median(time_groups(timer, warm, n, min_seconds / 2)))
        esz = np.dtype(case.dtype).itemsize
        extra.update({"launch_ms_warm": warm_ms, "hbm_frac_warm": case.points * 2 * esz / (warm_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS})
    return kernel_entry(case, kname, cold_ms, 1, traffic, extra)


def time_iterative_case(ssam, timer, case, a, b, fuse, min_seconds, traffic):
    """All sweeps of an iterative case per group; fuse = 0: one sweep per launch, -1: the library's choice.
    Runs carry on from the field the previous run left (same arithmetic on the same grid)."""
    ssam.ssam_set_tuning("fuse_sweeps", fuse)
    try:
        launches, kname, _ = launches_of(ssam, case)
        state = {"a": a, "b": b}

        def group():
            res = ssam.ssam_stencil_iterate(state["a"], state["b"], case_coef(case), case.steps, case.boundary)
            if res is not state["a"]:
                state["a"], state["b"] = state["b"], state["a"]

        group()
        ms = float(np.median(time_groups(timer, group, launches, min_seconds, min_groups=5)))
    finally:
        ssam.ssam_set_tuning("fuse_sweeps", -1)
    return kernel_entry(case, kname, ms, launches, traffic,
                        {"mode": "one_sweep_per_launch" if fuse == 0 else "default"})


def cpu_baseline_and_parity(ssam, torch, cases, outputs, target_seconds: float):
    """Times the oracle, as it stands, on a bounded sample -- the leading rows of each case's grid, one
    pass each, sized from a short calibration run for about `target_seconds` of oracle time in all --
    and compares the GPU output of the same cases with the fields the oracle computed: the rows of the
    sample that do not depend on rows beyond it (the sample ends inside the grid, so its last rows see
    the oracle's boundary rule where the full grid continues)."""
    import oracle
    import workloads as wl

    def run(case, lead):
        shape = (lead,) + tuple(case.shape[1:])
        # the leading block of the row-major field is a prefix of the same counter stream
        sample = wl.uniform_field(shape, case.field_range[0], case.field_range[1], case.field_seed, case.dtype)
        t0 = time.perf_counter()
        if case.kind == "conv2d":
            res = oracle.conv2d(sample, case.coef, case.boundary)
        elif case.kind == "conv3d":
            res = oracle.conv3d(sample, case.coef, case.boundary)
        else:
            res = oracle.stencil(sample, case_coef(case), case.boundary)
        return time.perf_counter() - t0, int(np.prod(shape)), res

    c0 = cases[0]
    inner0 = int(np.prod(c0.shape[1:]))
    lead0 = max(1, min(c0.shape[0], int(2e8 / max(1, c0.taps) / inner0)))
    dt, n, _ = run(c0, lead0)
    taps_per_s = n * c0.taps / max(dt, 1e-6)

    pts, secs, desc = 0, 0.0, []
    worst, checked, tol = 0.0, 0, 0.0
    for case in cases:
        inner = int(np.prod(case.shape[1:]))
        want_pts = target_seconds / len(cases) * taps_per_s / max(1, case.taps)
        lead = max(1, min(case.shape[0], int(want_pts // inner)))
        dt, n, ref = run(case, lead)
        secs += dt
        pts += n
        desc.append("x".join(str(v) for v in (lead,) + tuple(case.shape[1:])))
        if case.name in outputs:
            reach = case.coef.shape[0] - 1 - case.coef.shape[0] // 2     # rows below an output row that it reads
            rows = lead if lead == case.shape[0] else lead - reach
            if rows > 0:
                got = outputs[case.name][:rows].cpu().numpy()
                scale = float(np.abs(case.coef.astype(np.float64)).sum()) * max(abs(case.field_range[0]), abs(case.field_range[1]))
                err = float(np.max(np.abs(got.astype(np.float64) - ref[:rows].astype(np.float64)))) / scale
                worst = max(worst, err)
                checked += got.size
                tol = 1e-5 if np.dtype(case.dtype) == np.float32 else 1e-12
    threads = oracle.num_threads()
    oracle.set_num_threads(1)
    dt1, n1, _ = run(c0, max(1, lead0 // max(1, threads)))
    oracle.set_num_threads(threads)
    base = {"value": pts / secs / 1e9, "unit": "GStencil/s", "cores": threads, "kind": "oracle",
            "single_thread_ns_per_point": dt1 / n1 * 1e9, "single_thread_case": c0.name,
            "sample": f"one pass of each of the {len(cases)} cases on the leading block of its grid "
                      f"({', '.join(desc)}; {pts} points, {secs:.1f} s of oracle time)"}
    parity = {"max_norm_err": worst, "tol": tol, "checked_points": checked, "ok": bool(checked > 0 and worst <= tol),
              "against": "the oracle fields of the cpu_baseline sample (leading rows of every case), element by element, "
                         "normalised by sum|w| * max|in|"}
    return base, parity


# ---- the default workload ---------------------------------------------------------------------

def bench_default(ssam, wl, torch, args) -> int:
    traffic = measured_traffic()
    timer = Timer(torch)
    cases = wl.config2()
    if args.cases:
        keys = args.cases.split(",")
        cases = [c for c in cases if any(k in c.name for k in keys)]
    c0 = cases[0]
    image = wl.uniform_field_on("cuda", c0.shape, c0.field_range[0], c0.field_range[1], c0.field_seed, c0.dtype)
    inputs = [image] + [image.clone() for _ in range(COLD_COPIES - 1)]
    d_out = torch.empty_like(image)

    # plain grid-stride copy of the same size (1 read + 1 write), cold, for context
    def copies():
        for d_in in inputs:
            ssam.ssam_probe_copy(d_in, d_out)
    copies()
    copy_ms = float(np.median(time_groups(timer, copies, len(inputs), 0.1)))
    copy_gbps = 2 * image.numel() * image.element_size() / (copy_ms * 1e-3) / 1e9

    # per-kernel figures, every case alone
    kernels = [time_single_pass_case(ssam, timer, c, inputs, d_out, args.min_case_seconds, traffic) for c in cases]
    dom_case = max(zip(cases, kernels), key=lambda ck: ck[1]["launch_ms"])[0]

    # the headline: K steps of all cases, inputs rotated per launch, events around the dominant kernel only
    step_ms_guess = sum(k["launch_ms"] for k in kernels)
    steps = args.steps if args.steps is not None else max(20, min(5000, int(math.ceil(3200.0 / step_ms_guess))))
    warmup = args.warmup if args.warmup is not None else 20
    launch = itertools.count()

    def one_step(events=None):
        for c in cases:
            d_in = inputs[next(launch) % len(inputs)]
            if events is not None and c is dom_case:
                s, e = timer.pair()
                s.record(timer.stream)
                run_single(ssam, c, d_in, d_out)
                e.record(timer.stream)
                events.append((s, e))
            else:
                run_single(ssam, c, d_in, d_out)

    for _ in range(warmup):
        one_step()
    torch.cuda.synchronize()
    dom_events = []
    t0 = time.perf_counter()
    for _ in range(steps):
        one_step(dom_events)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dom_ms = float(np.mean([s.elapsed_time(e) for s, e in dom_events]))
    dom = kernel_entry(dom_case, next(k["kernel"] for k in kernels if k["case"] == dom_case.name), dom_ms, 1, traffic)
    if dom["bound"] == "hbm":
        roof = {"bound": "hbm", "achieved": dom["hbm_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": dom["hbm_frac"]}
    else:
        roof = {"bound": dom["bound"], "achieved": dom["alu_TFLOPs"], "peak": ALU_PEAK_TFLOPS["f32"], "unit": "TFLOP/s", "frac": dom["alu_frac"]}
    roof.update({"traffic": dom["traffic"], "kernel": dom["kernel"], "case": dom["case"], "launch_ms_mean": dom_ms,
                 "launches_timed": len(dom_events)})
    total_pts = sum(c.points for c in cases)

    # the GPU outputs the parity check compares (one more launch per case, kept on the device)
    outputs = {}
    if not args.no_cpu_baseline:
        for c in cases:
            o = torch.empty_like(image)
            run_single(ssam, c, image, o)
            outputs[c.name] = o
        torch.cuda.synchronize()

    out = {
        "metric": "GStencil/s", "value": total_pts / (wall / steps) / 1e9, "unit": "GStencil/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": wall / steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config2: " + ", ".join(c.name for c in cases), "grid": grid_tag(c0.shape),
                   "boundary": c0.boundary, "sweeps_per_case": 1,
                   "input": f"rotated among {len(inputs)} copies of the image per launch (cold in the memory-side cache)"},
        "roofline": roof,
        "consistency": {"timed_region_s": wall, "sum_of_median_launches_ms": step_ms_guess},
        "plain_copy_GBps": copy_gbps,
    }
    del inputs[1:]
    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["parity"] = cpu_baseline_and_parity(ssam, torch, cases, outputs, args.cpu_seconds)
    outputs.clear()
    del d_out, image
    torch.cuda.empty_cache()

    # the other configurations, every case alone: one sweep per launch, and the library's default
    if not args.cases and not args.headline_only:
        for cfg in ("config1", "config3", "config4", "config5"):
            for c in wl.all_configs()[cfg]:
                src = wl.uniform_field_on("cuda", c.shape, c.field_range[0], c.field_range[1], c.field_seed, c.dtype)
                a, b = grids_back_to_back(torch, src, 2)
                a.copy_(src)
                del src
                if c.steps == 1:
                    k = time_single_pass_case(ssam, timer, c, [a], b, args.min_case_seconds, traffic)
                    k["input"] = "one tensor"
                    kernels.append(k)
                    big = wl.Case(c.name + "_x6sweeps", c.kind, c.dtype, c.shape, c.field_range, c.field_seed, c.coef, c.boundary, 6)
                    kernels.append(time_iterative_case(ssam, timer, big, a, b, -1, args.min_case_seconds, traffic))
                else:
                    kernels.append(time_iterative_case(ssam, timer, c, a, b, 0, args.min_case_seconds, traffic))
                    kd = time_iterative_case(ssam, timer, c, a, b, -1, args.min_case_seconds, traffic)
                    if kd["kernel"] != kernels[-1]["kernel"]:
                        kernels.append(kd)
                del a, b
                torch.cuda.empty_cache()
    out["kernels"] = kernels
    print(json.dumps(out))
    return 0


# ---- one configuration as the workload -----------------------------------------------------------

def bench_config(ssam, wl, torch, args) -> int:
    traffic = measured_traffic()
    timer = Timer(torch)
    cases = wl.all_configs()[args.workload]
    if args.cases:
        keys = args.cases.split(",")
        cases = [c for c in cases if any(k in c.name for k in keys)]
    ssam.ssam_set_tuning("fuse_sweeps", args.fuse_sweeps)
    iterative = cases[0].steps > 1
    steps = args.steps if args.steps is not None else (3 if iterative else 20)
    warmup = args.warmup if args.warmup is not None else (1 if iterative else 3)

    fields, bufs = {}, {}
    for c in cases:
        key = (dtype_tag(c.dtype), c.shape, c.field_seed)
        if key not in fields:
            fields[key] = wl.uniform_field_on("cuda", c.shape, c.field_range[0], c.field_range[1], c.field_seed, c.dtype)
        bufs[c.name] = key
    work = {k: tuple(grids_back_to_back(torch, v, 2)) for k, v in fields.items()}
    copies = {k: [v] + [v.clone() for _ in range(COLD_COPIES - 1)]
              for k, v in fields.items() if any(c.steps == 1 and bufs[c.name] == k for c in cases)}
    turn = {}
    current = {}
    for c in cases:
        if c.steps > 1:
            a, b = work[bufs[c.name]]
            a.copy_(fields[bufs[c.name]])
            current[c.name] = (a, b)

    def run_case(c):
        """One pass of the case (all its sweeps); iterative cases carry on from the field the previous
        run left (the same arithmetic on the same grid; no copy inside the timed region)."""
        if c.steps == 1:   # a single pass reads a different copy of its input at every launch (cold, as in the default run)
            key = bufs[c.name]
            turn[key] = (turn.get(key, 0) + 1) % len(copies[key])
            run_single(ssam, c, copies[key][turn[key]], work[key][1])
        else:
            a, b = current[c.name]
            res = ssam.ssam_stencil_iterate(a, b, case_coef(c), c.steps, c.boundary)
            current[c.name] = (res, b if res is a else a)

    key0 = bufs[cases[0].name]
    src, (dst, _) = fields[key0], work[key0]
    copy_ms = float(np.median(time_groups(timer, lambda: ssam.ssam_probe_copy(src, dst), 1, 0.05)))
    copy_gbps = 2 * src.numel() * src.element_size() / (copy_ms * 1e-3) / 1e9

    for _ in range(warmup):
        for c in cases:
            run_case(c)
    torch.cuda.synchronize()
    ev = {c.name: [] for c in cases}
    t0 = time.perf_counter()
    for _ in range(steps):
        for c in cases:
            s, e = timer.pair()
            s.record(timer.stream)
            run_case(c)
            e.record(timer.stream)
            ev[c.name].append((s, e))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    kernels, total_pts = [], 0
    for c in cases:
        ms = float(np.median([s.elapsed_time(e) for s, e in ev[c.name]]))
        if c.steps == 1:
            launches, kname = 1, ssam.ssam_describe(c.kind, c.shape, case_coef(c), c.boundary).split()[0]
            names = [kname]
        else:
            launches, kname, names = launches_of(ssam, c)
        kernels.append(kernel_entry(c, kname, ms / launches, launches, traffic, {"launch_names": names}))
        total_pts += c.points * c.steps
    dom = max(kernels, key=lambda k: k["launch_ms"] * k["launches_per_step"])
    tag = "f32" if "f32" in dom["case"] else "f64"
    if dom["bound"] == "hbm":
        roof = {"bound": "hbm", "achieved": dom["hbm_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": dom["hbm_frac"]}
    else:
        roof = {"bound": dom["bound"], "achieved": dom["alu_TFLOPs"], "peak": ALU_PEAK_TFLOPS[tag], "unit": "TFLOP/s", "frac": dom["alu_frac"]}
    roof.update({"traffic": dom["traffic"], "kernel": dom["kernel"], "case": dom["case"]})
    out = {
        "metric": "GStencil/s", "value": total_pts / (wall / steps) / 1e9, "unit": "GStencil/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": wall / steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype_tag(cases[0].dtype) if len({dtype_tag(c.dtype) for c in cases}) == 1 else "f32+f64",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: " + ", ".join(c.name for c in cases), "grid": grid_tag(cases[0].shape),
                   "boundary": cases[0].boundary, "sweeps_per_case": cases[0].steps, "fuse_sweeps": args.fuse_sweeps,
                   "input": f"single-pass cases: rotated among {COLD_COPIES} copies per launch (cold in the memory-side cache); "
                            "iterated cases: two grids back to back"},
        "roofline": roof, "consistency": {"timed_region_s": wall}, "plain_copy_GBps": copy_gbps,
        "copy_bytes_each_way": src.numel() * src.element_size(), "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"], _ = cpu_baseline_and_parity(ssam, torch, cases, {}, args.cpu_seconds)
    print(json.dumps(out))
    return 0


# ---- scan ------------------------------------------------------------------------------------

def bench_scan(ssam, wl, torch, args) -> int:
    """The scan mapping of the model (paper Sec. 3.6; not evaluated there): inclusive prefix sums of
    1 GiB arrays, fp32 then fp64, one call each per step; elements per second, with the roofline of
    the fp32 call (one read and one write per element are the algorithmic bytes)."""
    traffic = measured_traffic()
    steps = args.steps if args.steps is not None else 20
    warmup = args.warmup if args.warmup is not None else 3
    nbytes = 1 << 30
    arrays = {}
    for tag, dt in (("f32", np.float32), ("f64", np.float64)):
        n = nbytes // np.dtype(dt).itemsize
        a = wl.uniform_field_on("cuda", (n,), -1.0, 1.0, 11, dt)
        work = torch.empty(ssam.ssam_scan_workspace_bytes(n, dt), dtype=torch.uint8, device="cuda")
        arrays[tag] = (a, torch.empty_like(a), work)
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        for a, b, work in arrays.values():
            ssam.ssam_scan(a, b, work)
    torch.cuda.synchronize()
    ev = {tag: [] for tag in arrays}
    t0 = time.perf_counter()
    for _ in range(steps):
        for tag, (a, b, work) in arrays.items():
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record(stream)
            ssam.ssam_scan(a, b, work)
            e.record(stream)
            ev[tag].append((s, e))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernels, elems = [], 0
    for tag, (a, b, work) in arrays.items():
        ms = float(np.median([s.elapsed_time(e) for s, e in ev[tag]]))
        gbps = 2 * nbytes / (ms * 1e-3) / 1e9
        kernels.append({"case": f"scan_{tag}_1GiB", "call_ms": ms, "gelem_per_s": a.numel() / ms / 1e6, "hbm_GBps": gbps,
                        "hbm_frac": gbps / HBM_PEAK_GBPS, "traffic": traffic.get(f"scan_chained_{tag}@{a.numel()}"),
                        "redone_after_giving_up": int(work.view(torch.int64)[16])})
        elems += a.numel()
    dom = kernels[0]
    out = {"metric": "Gelem/s", "value": elems / (wall / steps) / 1e9, "unit": "Gelem/s", "n_gpus": 1, "steps": steps,
           "warmup": warmup, "ms_per_step": wall / steps * 1e3, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32+f64", "data": "synthetic",
           "config": {"workload": "scan: inclusive prefix sums of 2^28 fp32 and 2^27 fp64 elements (1 GiB each), out of place"},
           "roofline": {"bound": "hbm", "achieved": dom["hbm_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                        "frac": dom["hbm_frac"], "traffic": dom["traffic"], "kernel": "scan_chained<float>", "case": dom["case"]},
           "kernels": kernels}
    if not args.no_cpu_baseline:
        import oracle
        sample = arrays["f32"][0][: 1 << 26].cpu().numpy()
        reps, t1 = 0, time.perf_counter()
        while time.perf_counter() - t1 < min(args.cpu_seconds, 10.0):
            oracle.scan(sample)
            reps += 1
        dt = time.perf_counter() - t1
        out["cpu_baseline"] = {"value": reps * sample.size / dt / 1e9, "unit": "Gelem/s", "cores": 1, "kind": "oracle",
                               "sample": f"the first 2^26 fp32 elements of the same array, {reps} passes, {dt:.1f} s (the oracle's scan is sequential)"}
    print(json.dumps(out))
    return 0


# ---- tuning sweeps ------------------------------------------------------------------------------

def tune(ssam, wl, torch, args) -> int:
    """Times the selected cases under every combination of the listed tuning overrides; one text line
    per combination.  Iterative cases run min(steps, 24) sweeps per repetition.  A library built with
    other compile-time options can be compared by pointing SSAM_LIB_PATH at it."""
    keys, vals = [], []
    for item in args.tune.split(";"):
        if item:
            k, v = item.split("=")
            keys.append(k)
            vals.append([int(x) for x in v.split(",")])
    timer = Timer(torch)
    workload = "config2" if args.workload == "default" else args.workload
    if workload == "scan":
        for tag, n in ((c.split(":")[0], int(c.split(":")[1])) for c in (args.cases or "f32:268435456").split(",")):
            dt = np.float32 if tag == "f32" else np.float64
            a = wl.uniform_field_on("cuda", (n,), -1.0, 1.0, 11, dt)
            b = torch.empty_like(a)
            work = torch.empty(8 << 20, dtype=torch.uint8, device="cuda")   # above the largest workspace of any schedule
            time_groups(timer, lambda: ssam.ssam_scan(a, b, work), 1, 0.3)
            for combo in itertools.product(*vals):
                for k, v in zip(keys, combo):
                    ssam.ssam_set_tuning(k, v)
                ms = float(np.median(time_groups(timer, lambda: ssam.ssam_scan(a, b, work), 1, args.min_case_seconds / 2)))
                knobs = " ".join(f"{k}={v}" for k, v in zip(keys, combo))
                print(f"scan {tag} n={n} {knobs}  {ms * 1e3:8.1f} us {n / ms / 1e6:7.1f} Gelem/s {2 * a.element_size() * n / ms / 1e6:7.0f} GB/s "
                      f"(workspace {ssam.ssam_scan_workspace_bytes(n, dt)} B)", flush=True)
            for k in keys:
                ssam.ssam_set_tuning(k, -1)
            ms = float(np.median(time_groups(timer, lambda: ssam.ssam_probe_copy(a, b), 1, 0.1)))
            print(f"copy {tag} n={n}  {ms * 1e3:8.1f} us {n / ms / 1e6:7.1f} Gelem/s {2 * a.element_size() * n / ms / 1e6:7.0f} GB/s", flush=True)
        return 0
    cases = wl.all_configs()[workload]
    if args.cases:
        sel = args.cases.split(",")
        cases = [c for c in cases if any(k in c.name for k in sel)]
    for c in cases:
        src = wl.uniform_field_on("cuda", c.shape, c.field_range[0], c.field_range[1], c.field_seed, c.dtype)
        a, b = grids_back_to_back(torch, src, 2)
        a.copy_(src)
        del src
        sweeps = 1 if c.kind == "conv2d" else min(c.steps, 24)
        # --cold: a single-pass case reads a different copy of its input at every launch
        inputs = [a] + [a.clone() for _ in range(COLD_COPIES - 1)] if args.cold and c.kind == "conv2d" else [a]
        turn = [0]

        def run():
            if c.kind == "conv2d":
                turn[0] = (turn[0] + 1) % len(inputs)
                ssam.ssam_conv2d(inputs[turn[0]], c.coef, c.boundary, d_out=b)
            else:
                ssam.ssam_stencil_iterate(a, b, case_coef(c), sweeps, c.boundary)

        time_groups(timer, run, 1, 0.3)      # bring the clocks up before the first figure
        for combo in itertools.product(*vals):
            for k, v in zip(keys, combo):
                ssam.ssam_set_tuning(k, v)
            run()
            ms = float(np.median(time_groups(timer, run, sweeps, args.min_case_seconds / 2, min_groups=5)))
            gpt = c.points / ms / 1e6
            knobs = " ".join(f"{k}={v}" for k, v in zip(keys, combo))
            print(f"{c.name:26s} {knobs}  {ms * 1e3:8.1f} us {gpt:7.1f} GStencil/s {gpt * 2 * np.dtype(c.dtype).itemsize:7.0f} GB/s", flush=True)
        for k in keys:
            ssam.ssam_set_tuning(k, -1)
        del a, b, inputs
        torch.cuda.empty_cache()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="default",
                    choices=["default", "config1", "config2", "config3", "config4", "config5", "filter_sweep", "table3", "conv3d", "scan"])
    ap.add_argument("--cases", default=None, help="comma-separated substrings selecting cases of the workload")
    ap.add_argument("--fuse-sweeps", type=int, default=-1,
                    help="cap on the sweeps ssam_stencil_iterate fuses into one launch (0: none; default: the library's choice)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle legs (CPU baseline and parity)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="oracle time to spend on the CPU baseline")
    ap.add_argument("--min-case-seconds", type=float, default=0.5, help="GPU time every per-kernel figure is measured over")
    ap.add_argument("--headline-only", action="store_true", help="default workload: skip configurations 1, 3, 4, 5")
    ap.add_argument("--variant", type=int, default=-1,
                    help="tuning variant for the whole run (e.g. 5: vector-unit instances of the matrix-core filters)")
    ap.add_argument("--cold", action="store_true", help="--tune: rotate the input of single-pass cases among 4 copies")
    ap.add_argument("--tune", default=None, help='"knob=v1,v2;knob2=..." : time the selected cases under tuning overrides')
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1. "
              "Across GPUs the path would shard by slabs along the slowest axis with a halo exchange between neighbours.", file=sys.stderr)
        return 2

    import torch

    import paper_1907_06154_amd as ssam
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    ssam.lib()
    torch.cuda.set_device(0)

    if args.variant >= 0:
        ssam.ssam_set_tuning("variant", args.variant)
    if args.tune is not None:
        return tune(ssam, wl, torch, args)
    if args.workload == "scan":
        return bench_scan(ssam, wl, torch, args)
    if args.workload == "default":
        return bench_default(ssam, wl, torch, args)
    return bench_config(ssam, wl, torch, args)


if __name__ == "__main__":
    sys.exit(main())
