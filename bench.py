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

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000, the
# factors being what the same counters read for ssam_probe_copy of known size); the runs and
# their commands are summarised under profiles/.  Keyed by case name and, for the multi-sweep
# kernels of the iterative 2D cases, by case and kernel instance; offline figures, not re-measured
# by this script.
MEASURED_TRAFFIC_BYTES = {
    "c2_conv3x3_f32": 537671369,
    "c2_conv5x5_f32": 538194718,
    "c2_conv9x9_f32": 570754529,
    "c2_conv15x15_f32": 574873014,
    "c2_conv20x20_f32": 586910020,
    "c2_conv3x11_f32": 575620141,
    "c2_conv11x3_f32": 552730765,
    "c3_2d_box_r1_f64": 1075826419,
    "c3_2d_box_r2_f64": 1076305303,
    "c3_2d_star_r4_f64": 1078286643,
    "c3_2d_box_r1_f64:double_R1_b2_v2p4nt2_fused8": 1109794685,
    "c3_2d_box_r2_f64:double_R2_b2_v2p4nt2_fused4": 1120376530,
    "c3_2d_star_r4_f64:double_R4_b1_v2p4nt2_fused3": 1150265600,
    "c4_3d_star_r1_f64": 2439207291,
    "c4_3d_box_r1_f64": 2347660545,
    "c4_3d_faces_edges_f64": 2313081318,
    "c4_3d_star_r1_f64:double_r111_b1_v2p4f1nt2_fused2": 2305148286,
    "c4_3d_box_r1_f64:double_r111_b3_v2p4f1nt2_fused2": 2526118196,
    "c4_3d_faces_edges_f64:double_r111_b2_v2p4f0nt2_fused2": 2252726714,
    "c5_3d_star_r4_f32": 1252975790,
    "c5_3d_star_r4_f64": 2446461759,
}


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
        return ssam.ssam_stencil_iterate(a, b, case_coef(case), case.steps, case.boundary)
    return b


def cpu_baseline(cases, target_seconds: float):
    """Times the oracle, as it stands, on a bounded sample: the leading rows (planes) of each
    case's grid, one sweep each.  A short calibration run measures the oracle's rate on this
    host, then the sample is sized for about `target_seconds` of oracle time in total.
    Returns GStencil/s over the sample."""
    import oracle
    from paper_1907_06154_amd import workloads as wl

    def run(case, lead):
        shape = (lead,) + tuple(case.shape[1:])
        # the leading block of the row-major field is a prefix of the same counter stream
        sample = wl.uniform_field(shape, case.field_range[0], case.field_range[1], case.field_seed, case.dtype)
        t0 = time.perf_counter()
        if case.kind == "conv2d":
            oracle.conv2d(sample, case.coef, case.boundary)
        else:
            oracle.stencil(sample, case_coef(case), case.boundary)
        return time.perf_counter() - t0, int(np.prod(shape))

    # calibration: about 2e8 multiply-adds on the first case
    c0 = cases[0]
    inner0 = int(np.prod(c0.shape[1:]))
    lead0 = max(1, min(c0.shape[0], int(2e8 / max(1, c0.taps) / inner0)))
    dt, n = run(c0, lead0)
    taps_per_s = n * c0.taps / max(dt, 1e-6)

    pts, secs, desc = 0, 0.0, []
    for case in cases:
        inner = int(np.prod(case.shape[1:]))
        want_pts = target_seconds / len(cases) * taps_per_s / max(1, case.taps)
        lead = max(1, min(case.shape[0], int(want_pts // inner)))
        dt, n = run(case, lead)
        secs += dt
        pts += n
        desc.append("x".join(str(v) for v in (lead,) + tuple(case.shape[1:])))
    # one thread on a reduced extent, for the per-point cost of the oracle itself
    threads = oracle.num_threads()
    oracle.set_num_threads(1)
    dt1, n1 = run(c0, max(1, lead0 // max(1, threads)))
    oracle.set_num_threads(threads)
    return {"value": pts / secs / 1e9, "unit": "GStencil/s", "cores": threads, "kind": "oracle",
            "single_thread_ns_per_point": dt1 / n1 * 1e9, "single_thread_case": c0.name,
            "sample": f"one sweep of each of the {len(cases)} cases on the leading block of its grid "
                      f"({', '.join(desc)}; {pts} points, {secs:.1f} s of oracle time)"}


# HBM bytes one ssam_scan call moves at the benchmark size (one-pass schedule), from the rocprofv3
# FETCH_SIZE / WRITE_SIZE counters scaled by the copy kernel's readings (profiles/scan_1GiB_f32_f64.md)
SCAN_MEASURED_TRAFFIC_BYTES = {"f32": int((1027.0 + 1026.4) * 2 ** 20), "f64": int((1027.0 + 1026.3) * 2 ** 20)}


def bench_scan(ssam, wl, torch, args) -> int:
    """The scan mapping of the model (paper Sec. 3.6; not evaluated there): inclusive prefix sums of
    1 GiB arrays, fp32 then fp64, one call each per step; elements per second, with the roofline of
    the fp32 call (one read and one write per element are the algorithmic bytes)."""
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
        ms = float(np.mean([s.elapsed_time(e) for s, e in ev[tag]]))
        gbps = 2 * nbytes / (ms * 1e-3) / 1e9
        kernels.append({"case": f"scan_{tag}_1GiB", "call_ms": ms, "gelem_per_s": a.numel() / ms / 1e6, "hbm_GBps": gbps,
                        "hbm_frac": gbps / HBM_PEAK_GBPS, "traffic": SCAN_MEASURED_TRAFFIC_BYTES[tag],
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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="config2", choices=["config1", "config2", "config3", "config4", "config5", "filter_sweep", "table3", "scan"])
    ap.add_argument("--cases", default=None, help="comma-separated substrings selecting cases of the workload")
    ap.add_argument("--fuse-sweeps", type=int, default=-1,
                    help="cap on the sweeps ssam_stencil_iterate fuses into one launch (0: none; default: the library's choice)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="oracle time to spend on the CPU baseline")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1. "
              "Across GPUs the path would shard by slabs along the slowest axis with a halo exchange between neighbours.", file=sys.stderr)
        return 2

    import torch

    import paper_1907_06154_amd as ssam
    from paper_1907_06154_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    ssam.lib()
    torch.cuda.set_device(0)
    ssam.ssam_set_tuning("fuse_sweeps", args.fuse_sweeps)

    if args.workload == "scan":
        return bench_scan(ssam, wl, torch, args)

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

    def finish(c, res):
        if c.steps > 1:   # carry on from whichever buffer holds the field now
            a, b = current[c.name]
            current[c.name] = (res, b if res is a else a)

    stream = torch.cuda.current_stream()

    # the plain grid-stride copy (1 read + 1 write of the same size), for context
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
            finish(c, run_case(ssam, c, prepare(c)))
    torch.cuda.synchronize()

    ev = {c.name: [] for c in cases}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for c in cases:
            pair = prepare(c)
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record(stream)
            res = run_case(ssam, c, pair)
            e.record(stream)
            finish(c, res)
            ev[c.name].append((s, e))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    kernels = []
    total_pts = 0
    for c in cases:
        ms = float(np.mean([s.elapsed_time(e) for s, e in ev[c.name]]))
        # a launch is one sweep, or several where ssam_stencil_iterate fuses 2D sweeps: such a
        # launch still reads and writes the grid once, and does the arithmetic of all its sweeps
        kind = c.kind if c.steps == 1 else {"stencil2d": "iterate2d", "stencil3d": "iterate3d"}[c.kind]
        kname = ssam.ssam_describe(kind, c.shape, case_coef(c), c.boundary).split()[0]
        launches, t = 0, 0
        while t < c.steps:   # replay the planner: a "..._fusedS" launch performs S sweeps
            if kind == "iterate2d":
                nm = ssam.ssam_describe(kind, c.shape, case_coef(c), c.boundary, remaining=c.steps - t).split()[0]
            else:   # 3D: pairs of sweeps while two or more remain
                nm = kname if c.steps - t >= 2 else ssam.ssam_describe(c.kind, c.shape, case_coef(c), c.boundary).split()[0]
            t += int(nm.rsplit("_fused", 1)[1]) if "_fused" in nm else 1
            launches += 1
        per_launch_ms = ms / launches
        esz = np.dtype(c.dtype).itemsize
        alg_bytes = c.points * 2 * esz
        flops = c.points * (2 * c.taps - 1) * c.steps / launches
        tag = dtype_tag(c.dtype)
        t_hbm = alg_bytes / (HBM_PEAK_GBPS * 1e9)
        t_alu = flops / (ALU_PEAK_TFLOPS[tag] * 1e12)
        gbps = alg_bytes / (per_launch_ms * 1e-3) / 1e9
        tflops = flops / (per_launch_ms * 1e-3) / 1e12
        k = {"case": c.name, "kernel": kname, "launch_ms": per_launch_ms, "launches_per_step": launches,
             "sweeps_per_launch": c.steps / launches, "gstencil_per_s": c.points * c.steps / ms / 1e6,
             "hbm_GBps": gbps, "hbm_frac": gbps / HBM_PEAK_GBPS, "alu_TFLOPs": tflops,
             "alu_frac": tflops / ALU_PEAK_TFLOPS[tag],
             # arithmetic-bound kernels whose products run on the matrix cores ("...mx") are priced
             # against the dense fp32 MFMA peak, which equals the published fp32 vector peak
             "bound": "hbm" if t_hbm >= t_alu else ("mfma" if kname.split("+")[0].endswith("mx") else "alu"),
             "traffic": MEASURED_TRAFFIC_BYTES.get(c.name + ":" + kname if "_fused" in kname else c.name)}
        kernels.append(k)
        total_pts += c.points * c.steps

    dom = max(kernels, key=lambda k: k["launch_ms"] * k["launches_per_step"])
    if dom["bound"] == "hbm":
        roof = {"bound": "hbm", "achieved": dom["hbm_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": dom["hbm_frac"], "traffic": dom["traffic"], "kernel": dom["kernel"], "case": dom["case"]}
    else:
        tag = "f32" if "f32" in dom["case"] else "f64"
        roof = {"bound": dom["bound"], "achieved": dom["alu_TFLOPs"], "peak": ALU_PEAK_TFLOPS[tag], "unit": "TFLOP/s",
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
                   "sweeps_per_case": cases[0].steps, "fuse_sweeps": args.fuse_sweeps},
        "roofline": roof,
        "plain_copy_GBps": copy_gbps,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cases, args.cpu_seconds)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
