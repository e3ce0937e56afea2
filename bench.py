#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config2]

A "step" is one pass of the whole hot path over one batch of synthetic input: for the
default workload (benchmark configuration 2) that is one 8192x8192 fp32 2D filter pass for
each of the seven filter shapes; for the iterative configurations it is the full
`steps`-sweep Jacobi run of every stencil of the configuration.  Inputs are generated from
seeds on the host and are resident in HBM before the timed region starts.

Prints ONE JSON line: whole-job GStencil/s (output points x sweeps / second), the roofline
figures of the dominant kernel (live HIP-event timing on the launch stream), every kernel's
own figures under "kernels", and the CPU oracle timed on a bounded sample of the same
workload ("cpu_baseline").
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0                          # MI355X HBM3E, published
ALU_PEAK_TFLOPS = {"f32": 157.3, "f64": 78.6}   # published vector peaks (fp32 figure assumes packed FMA)

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled by the
# same counters' reading for ssam_probe_copy of known size; see profiles/.  Keyed by case name.
MEASURED_TRAFFIC_BYTES = {}


def dtype_tag(dt) -> str:
    return "f32" if np.dtype(dt) == np.float32 else "f64"


def case_coef(case):
    return case.coef if case.kind != "stencil2d" else case.coef[0]


def run_case(ssam, case, bufs):
    """Enqueue one pass of `case` (all its sweeps) on the current stream."""
    a, b = bufs
    if case.kind == "conv2d":
        ssam.ssam_conv2d(a, case.coef, case.boundary, d_out=b)
    elif case.steps == 1 and case.kind == "stencil2d":
        ssam.ssam_stencil2d(a, case_coef(case), case.boundary, d_out=b)
    elif case.steps == 1:
        ssam.ssam_stencil3d(a, case_coef(case), case.boundary, d_out=b)
    else:
        ssam.ssam_stencil_iterate(a, b, case_coef(case), case.steps, case.boundary)


def cpu_baseline(cases, budget_taps: float):
    """Times the oracle, as it stands, on a bounded sample: the leading rows (planes) of each
    case's grid, one sweep each, sized so that the whole sample costs about `budget_taps`
    multiply-adds.  Returns GStencil/s over the sample."""
    import oracle
    from paper_1907_06154_amd import workloads as wl
    pts = 0
    secs = 0.0
    desc = []
    for case in cases:
        shape = list(case.shape)
        inner = int(np.prod(shape[1:]))
        want_pts = budget_taps / len(cases) / max(1, case.taps)
        shape[0] = max(1, min(shape[0], int(want_pts // inner)))
        # the leading block of the row-major field is a prefix of the same counter stream
        sample = wl.uniform_field(tuple(shape), case.field_range[0], case.field_range[1], case.field_seed, case.dtype)
        t0 = time.perf_counter()
        if case.kind == "conv2d":
            oracle.conv2d(sample, case.coef, case.boundary)
        else:
            oracle.stencil(sample, case_coef(case), case.boundary)
        secs += time.perf_counter() - t0
        pts += int(np.prod(shape))
        desc.append("x".join(str(s) for s in shape))
    return {"value": pts / secs / 1e9, "unit": "GStencil/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"one sweep of each of the {len(cases)} cases on the leading block of its grid "
                      f"({', '.join(desc)}; {pts} points, {secs:.1f} s of oracle time)"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="config2", choices=["config1", "config2", "config3", "config4", "config5"])
    ap.add_argument("--cases", default=None, help="comma-separated substrings selecting cases of the workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-taps", type=float, default=24e9, help="oracle sample size in multiply-adds")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1. "
              "DESIGN.md describes how the path would shard.", file=sys.stderr)
        return 2

    import torch

    import paper_1907_06154_amd as ssam
    from paper_1907_06154_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    ssam.lib()
    torch.cuda.set_device(0)

    cases = wl.all_configs()[args.workload]
    if args.cases:
        keys = args.cases.split(",")
        cases = [c for c in cases if any(k in c.name for k in keys)]
    iterative = cases[0].steps > 1
    steps = args.steps if args.steps is not None else (3 if iterative else 20)
    warmup = args.warmup if args.warmup is not None else (1 if iterative else 3)

    # inputs resident in HBM before timing; cases of one workload share grid shape and seed per dtype
    fields = {}
    bufs = {}
    for c in cases:
        key = (dtype_tag(c.dtype), c.shape, c.field_seed)
        if key not in fields:
            host = c.field()
            fields[key] = torch.from_numpy(host).cuda()
        bufs[c.name] = key
    work = {k: (torch.empty_like(v), torch.empty_like(v)) for k, v in fields.items()}

    # Single-pass cases read the resident input and write a work buffer.  Iterative cases
    # ping-pong between the two work buffers and carry on from the field the previous run
    # left (the same arithmetic on the same grid; no copy inside the timed region).
    current = {}
    for c in cases:
        if c.steps > 1:
            a, b = work[bufs[c.name]]
            a.copy_(fields[bufs[c.name]])
            current[c.name] = (a, b)

    def prepare(c):
        if c.steps == 1:
            return fields[bufs[c.name]], work[bufs[c.name]][1]
        return current[c.name]

    def finish(c):
        if c.steps > 1 and c.steps % 2 == 1:
            a, b = current[c.name]
            current[c.name] = (b, a)

    stream = torch.cuda.current_stream()

    # copy ceiling (1 read + 1 write of the same size), for context
    key0 = bufs[cases[0].name]
    src, (dst, _) = fields[key0], work[key0]
    for _ in range(3):
        ssam.ssam_probe_copy(src, dst)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(10):
        ssam.ssam_probe_copy(src, dst)
    e1.record(stream)
    torch.cuda.synchronize()
    copy_gbps = 10 * 2 * src.numel() * src.element_size() / (e0.elapsed_time(e1) * 1e-3) / 1e9

    for _ in range(warmup):
        for c in cases:
            run_case(ssam, c, prepare(c))
            finish(c)
    torch.cuda.synchronize()

    ev = {c.name: [] for c in cases}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for c in cases:
            pair = prepare(c)
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record(stream)
            run_case(ssam, c, pair)
            e.record(stream)
            finish(c)
            ev[c.name].append((s, e))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    kernels = []
    total_pts = 0
    for c in cases:
        ms = float(np.mean([s.elapsed_time(e) for s, e in ev[c.name]]))
        per_launch_ms = ms / c.steps
        esz = np.dtype(c.dtype).itemsize
        alg_bytes = c.points * 2 * esz
        flops = c.points * (2 * c.taps - 1)
        tag = dtype_tag(c.dtype)
        t_hbm = alg_bytes / (HBM_PEAK_GBPS * 1e9)
        t_alu = flops / (ALU_PEAK_TFLOPS[tag] * 1e12)
        gbps = alg_bytes / (per_launch_ms * 1e-3) / 1e9
        tflops = flops / (per_launch_ms * 1e-3) / 1e12
        k = {"case": c.name, "kernel": ssam.ssam_describe(c.kind, c.shape, case_coef(c), c.boundary).split()[0],
             "launch_ms": per_launch_ms, "launches_per_step": c.steps, "gstencil_per_s": c.points / per_launch_ms / 1e6,
             "hbm_GBps": gbps, "hbm_frac": gbps / HBM_PEAK_GBPS, "alu_TFLOPs": tflops,
             "alu_frac": tflops / ALU_PEAK_TFLOPS[tag], "bound": "hbm" if t_hbm >= t_alu else "alu",
             "traffic": MEASURED_TRAFFIC_BYTES.get(c.name)}
        kernels.append(k)
        total_pts += c.points * c.steps

    dom = max(kernels, key=lambda k: k["launch_ms"] * k["launches_per_step"])
    if dom["bound"] == "hbm":
        roof = {"bound": "hbm", "achieved": dom["hbm_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": dom["hbm_frac"], "traffic": dom["traffic"], "kernel": dom["kernel"], "case": dom["case"]}
    else:
        tag = "f32" if "f32" in dom["case"] else "f64"
        roof = {"bound": "alu", "achieved": dom["alu_TFLOPs"], "peak": ALU_PEAK_TFLOPS[tag], "unit": "TFLOP/s",
                "frac": dom["alu_frac"], "traffic": dom["traffic"], "kernel": dom["kernel"], "case": dom["case"]}

    ms_per_step = wall / steps * 1e3
    out = {
        "metric": "GStencil/s", "value": total_pts / (wall / steps) / 1e9, "unit": "GStencil/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype_tag(cases[0].dtype) if len({dtype_tag(c.dtype) for c in cases}) == 1 else "f32+f64",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: " + ", ".join(c.name for c in cases),
                   "grid": "x".join(str(s) for s in cases[0].shape), "boundary": cases[0].boundary,
                   "sweeps_per_case": cases[0].steps},
        "roofline": roof,
        "copy_ceiling_GBps": copy_gbps,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cases, args.cpu_taps)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
