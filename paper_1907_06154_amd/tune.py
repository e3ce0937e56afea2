"""Times benchmark cases under tuning overrides (launch geometry, compiled-instance variants).

    python -m paper_1907_06154_amd.tune <config> <case-substring> "<knob>=v1,v2;<knob2>=..." [reps]

e.g.  python -m paper_1907_06154_amd.tune config2 conv3x3 "rows_per_wave=32,64;valid_lanes=56,62" 20

      python -m paper_1907_06154_amd.tune scan f32:268435456 "scan_segments=8192,32768;scan_order=0,1" 20

(config "scan": the case is <f32|f64>:<elements>; the figure is elements per second and the
algorithmic bytes, one read and one write per element, per second.)

Every combination of the listed knob values (see ssam_set_tuning in include/ssam.h) is timed
with HIP events on the launch stream; iterative cases run min(steps, 24) sweeps per repetition.
A library built with other compile-time options can be compared by pointing SSAM_LIB_PATH at it
(python -m paper_1907_06154_amd.build other.so -DNAME).
"""
from __future__ import annotations

import itertools
import sys

import numpy as np


def main(argv) -> int:
    import torch

    import paper_1907_06154_amd as ssam
    from paper_1907_06154_amd import workloads as wl

    if len(argv) < 3:
        print(__doc__)
        return 2
    cfg, sub, spec = argv[0], argv[1], argv[2]
    reps = int(argv[3]) if len(argv) > 3 else 10
    keys, vals = [], []
    for item in spec.split(";"):
        if item:
            k, v = item.split("=")
            keys.append(k)
            vals.append([int(x) for x in v.split(",")])
    if cfg == "scan":
        return tune_scan(ssam, wl, torch, sub, keys, vals, reps)
    cases = [c for c in wl.all_configs()[cfg] if sub in c.name]
    for c in cases:
        fld = torch.from_numpy(c.field()).cuda()
        a, b = fld.clone(), torch.empty_like(fld)
        coef = c.coef if c.kind != "stencil2d" else c.coef[0]
        sweeps = 1 if c.kind == "conv2d" else min(c.steps, 24)

        def run():
            if c.kind == "conv2d":
                ssam.ssam_conv2d(a, coef, c.boundary, d_out=b)
            else:
                ssam.ssam_stencil_iterate(a, b, coef, sweeps, c.boundary)

        # bring the clocks up before the first figure: a short run after idling reads low
        t_end = torch.cuda.Event(enable_timing=True)
        t_beg = torch.cuda.Event(enable_timing=True)
        t_beg.record()
        while True:
            for _ in range(5):
                run()
            t_end.record()
            torch.cuda.synchronize()
            if t_beg.elapsed_time(t_end) > 300.0:
                break
        for combo in itertools.product(*vals):
            for k, v in zip(keys, combo):
                ssam.ssam_set_tuning(k, v)
            for _ in range(2):
                run()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                run()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps / sweeps
            gpt = c.points / ms / 1e6
            gbs = gpt * 2 * np.dtype(c.dtype).itemsize
            knobs = " ".join(f"{k}={v}" for k, v in zip(keys, combo))
            print(f"{c.name:26s} {knobs}  {ms * 1e3:8.1f} us {gpt:7.1f} GStencil/s {gbs:7.0f} GB/s", flush=True)
        for k in keys:
            ssam.ssam_set_tuning(k, -1)
    return 0


def tune_scan(ssam, wl, torch, case: str, keys, vals, reps: int) -> int:
    tag, n = case.split(":")
    n = int(n)
    dt = torch.float32 if tag == "f32" else torch.float64
    a = wl.uniform_field_on("cuda", (n,), -1.0, 1.0, 11, np.float32 if tag == "f32" else np.float64)
    b = torch.empty_like(a)
    work = torch.empty(8 << 20, dtype=torch.uint8, device="cuda")   # above the largest workspace of any schedule
    esz = a.element_size()

    def run():
        ssam.ssam_scan(a, b, work)

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    while True:
        for _ in range(5):
            run()
        e1.record()
        torch.cuda.synchronize()
        if e0.elapsed_time(e1) > 300.0:
            break
    for combo in itertools.product(*vals):
        for k, v in zip(keys, combo):
            ssam.ssam_set_tuning(k, v)
        for _ in range(2):
            run()
        e0.record()
        for _ in range(reps):
            run()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        knobs = " ".join(f"{k}={v}" for k, v in zip(keys, combo))
        print(f"scan {tag} n={n} {knobs}  {ms * 1e3:8.1f} us {n / ms / 1e6:7.1f} Gelem/s {2 * esz * n / ms / 1e6:7.0f} GB/s "
              f"(workspace {ssam.ssam_scan_workspace_bytes(n, dt)} B)", flush=True)
    for k in keys:
        ssam.ssam_set_tuning(k, -1)
    # the ceiling for one read and one write per element: the plain copy kernel on the same arrays
    for _ in range(2):
        ssam.ssam_probe_copy(a, b)
    e0.record()
    for _ in range(reps):
        ssam.ssam_probe_copy(a, b)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    print(f"copy {tag} n={n}  {ms * 1e3:8.1f} us {n / ms / 1e6:7.1f} Gelem/s {2 * esz * n / ms / 1e6:7.0f} GB/s", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
