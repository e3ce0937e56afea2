"""Turns rocprofv3 output into the short summaries kept under profiles/ (text only), and keeps
profiles/measured_traffic.json, the HBM bytes per launch that bench.py reports as roofline.traffic.

    python -m paper_1907_06154_amd.profiling summarize <prefix> <out.md> --title T --bench-args "..."
    python -m paper_1907_06154_amd.profiling sq <counter dir> [<counter dir> ...] <out.md>
    python -m paper_1907_06154_amd.profiling lds <counter dir> [<counter dir> ...] <out.md>
    python -m paper_1907_06154_amd.profiling resources <out.md>
    python -m paper_1907_06154_amd.profiling catalogue <single.json> <default.json> <out.md>
    python -m paper_1907_06154_amd.profiling sweep <default.json> <variant5.json> <out.md>
    python -m paper_1907_06154_amd.profiling scan <dir> <out.md>

`summarize` expects three rocprofv3 runs of the same bench.py command (the commands are written
into the summary), each with its bench.py output saved beside it:
    <prefix>_trace/  (--kernel-trace --stats)   <prefix>_trace.json
    <prefix>_fetch/  (--pmc FETCH_SIZE)         <prefix>_fetch.json
    <prefix>_write/  (--pmc WRITE_SIZE)         <prefix>_write.json
The counters are scaled by what they read for the plain copy kernel of known size that bench.py
runs first (ssam_probe_copy).  Dispatches are matched to kernel instances by their order: the
counter runs use --steps 1 --warmup 0, so the library's dispatches are exactly the launches
bench.py lists per case ("launch_names").

`resources` compiles every translation unit for gfx950 with -Rpass-analysis=kernel-resource-usage
(no GPU needed) and tabulates registers, LDS, scratch and waves per SIMD of every kernel.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
TRAFFIC = os.path.join(ROOT, "profiles", "measured_traffic.json")


def short(name: str) -> str:
    for prefix in ("void ", "ssam::", "(anonymous namespace)::"):
        if name.startswith(prefix):
            name = name[len(prefix):]
    return name.split("(ssam::")[0].split("(HIP_vector")[0].split("(float")[0].split("(double")[0]


def ours(kernel: str) -> bool:
    """A compute kernel of the library (not its plain copy kernel, not one of torch's)."""
    k = short(kernel)
    return k.startswith(("ssam2d", "ssam3d", "scan_", "generic_kernel"))


def is_copy(kernel: str) -> bool:
    return short(kernel).startswith("copy_kernel")


def one(pattern: str) -> str:
    hits = glob.glob(pattern, recursive=True)
    if not hits:
        raise SystemExit(f"nothing matches {pattern}")
    return hits[0]


def load_traffic() -> dict:
    try:
        return json.load(open(TRAFFIC))
    except (OSError, ValueError):
        return {"comment": "HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE, scaled by the readings of the "
                           "plain copy kernel; keys: <kernel instance>@<grid>; written by paper_1907_06154_amd.profiling",
                "bytes_per_launch": {}, "source": {}}


def counter_dispatches(dirname: str):
    """[(kernel, {counter: value}, duration_us)] in dispatch order."""
    rows = collections.OrderedDict()
    for r in csv.DictReader(open(one(os.path.join(dirname, "**", "*counter_collection.csv")))):
        d = rows.setdefault(int(r["Dispatch_Id"]), {"kernel": short(r["Kernel_Name"]), "c": {},
                                                    "us": (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3})
        d["c"][r["Counter_Name"]] = d["c"].get(r["Counter_Name"], 0.0) + float(r["Counter_Value"])
    return [(d["kernel"], d["c"], d["us"]) for _, d in sorted(rows.items())]


def summarize(prefix: str, out_md: str, title: str, bench_args: str) -> None:
    bench = {k: json.load(open(f"{prefix}_{k}.json")) for k in ("trace", "fetch", "write")}
    out = [f"# rocprofv3 summary: {title}\n"]
    cmd = f"python3 bench.py {bench_args} --no-cpu-baseline"
    out.append(f"Kernel durations:\n\n    rocprofv3 --kernel-trace --stats --output-format csv -d {prefix}_trace -o c -- {cmd} "
               f"--steps {bench['trace']['steps']} --warmup {bench['trace']['warmup']}\n")
    out.append("| kernel | calls | avg us | min us | max us | % of GPU time |\n|---|---|---|---|---|---|")
    for r in csv.DictReader(open(one(os.path.join(prefix + "_trace", "**", "*kernel_stats.csv")))):
        if ours(r["Name"]) or is_copy(r["Name"]):
            out.append(f"| `{short(r['Name'])}` | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | {float(r['MinNs']) / 1e3:.1f} | "
                       f"{float(r['MaxNs']) / 1e3:.1f} | {r['Percentage']} |")
    b = bench["trace"]
    out.append("\nThe same run's bench.py line (HIP events on the launch stream, median over the steps; a launch of a `_fusedS` "
               "instance performs S sweeps, so GStencil/s counts S updates per point per launch while the algorithmic GB/s is "
               "the one read and one write the launch makes):\n")
    out.append("| case | kernel instance (most launches) | launches per step | launch us | GStencil/s | algorithmic GB/s per launch "
               "| fraction of 8 TB/s | TFLOP/s | fraction of published vector peak |\n|---|---|---|---|---|---|---|---|---|")
    for k in b["kernels"]:
        out.append(f"| {k['case']} | `{k['kernel']}` | {k['launches_per_step']} | {k['launch_ms'] * 1e3:.1f} | {k['gstencil_per_s']:.1f} | "
                   f"{k['hbm_GBps']:.0f} | {k['hbm_frac']:.3f} | {k['alu_TFLOPs']:.1f} | {k['alu_frac']:.3f} |")
    out.append(f"\nWhole bench line: value {b['value']:.1f} {b['unit']}, {b['ms_per_step']:.2f} ms per step "
               f"({len(b['kernels'])} cases, timed region {b['consistency']['timed_region_s']:.2f} s).\n")

    out.append("HBM traffic counters (each in a run of its own; per dispatch, mean over the dispatches of an instance):\n")
    for kind, ctr in (("fetch", "FETCH_SIZE"), ("write", "WRITE_SIZE")):
        out.append(f"    rocprofv3 --pmc {ctr} --kernel-trace --output-format csv -d {prefix}_{kind} -o c -- {cmd} --steps 1 --warmup 0")
    out.append("")
    per_inst = {}
    scale = {}
    grid = b["config"]["grid"]
    for kind, ctr in (("fetch", "FETCH_SIZE"), ("write", "WRITE_SIZE")):
        disp = counter_dispatches(f"{prefix}_{kind}")
        names = [n for k in bench[kind]["kernels"] for n in k["launch_names"]]
        mine = [(k, c) for k, c, _ in disp if ours(k)]
        if len(mine) != len(names):
            raise SystemExit(f"{prefix}_{kind}: {len(mine)} library dispatches for {len(names)} launches bench.py lists")
        copies = [c[ctr] for k, c, _ in disp if is_copy(k)]
        copy_bytes = bench[kind]["copy_bytes_each_way"]
        scale[kind] = (copy_bytes / 1024.0) / (sum(copies) / len(copies))
        for inst, (k, c) in zip(names, mine):
            per_inst.setdefault(inst, {"kernel": k, "fetch": [], "write": []})[kind].append(c[ctr])
    out.append(f"The plain copy kernel (`ssam_probe_copy`, {bench['fetch']['copy_bytes_each_way'] / 2 ** 20:.0f} MiB read and written) "
               f"gives the scale factors {scale['fetch']:.3f} (FETCH_SIZE, KiB) and {scale['write']:.3f} (WRITE_SIZE, KiB).\n")
    out.append("| kernel instance | kernel | dispatches | FETCH_SIZE KiB | WRITE_SIZE KiB | scaled read MiB | scaled write MiB | "
               "algorithmic MiB per launch (read+write) | traffic / algorithmic |\n|---|---|---|---|---|---|---|---|---|")
    traffic = load_traffic()
    esz = {"float": 4, "double": 8}
    pts = 1
    for s in grid.split("x"):
        pts *= int(s)
    for inst, v in per_inst.items():
        f = sum(v["fetch"]) / len(v["fetch"])
        w = sum(v["write"]) / len(v["write"])
        alg = 2 * pts * esz[inst.split("_")[0]] / 2 ** 20
        tot = (f * scale["fetch"] + w * scale["write"]) / 1024
        out.append(f"| `{inst}` | `{v['kernel']}` | {len(v['fetch'])} | {f:.0f} | {w:.0f} | {f * scale['fetch'] / 1024:.1f} | "
                   f"{w * scale['write'] / 1024:.1f} | {alg:.0f} | {tot / alg:.3f} |")
        traffic["bytes_per_launch"][f"{inst}@{grid}"] = int(tot * 2 ** 20)
        traffic["source"][f"{inst}@{grid}"] = os.path.relpath(out_md, ROOT)
    open(out_md, "w").write("\n".join(out) + "\n")
    json.dump(traffic, open(TRAFFIC, "w"), indent=1, sort_keys=True)
    print("\n".join(out))


def sweeps_of(kernel: str) -> int:
    if "ssam2d_fused" in kernel:
        return int(re.search(r">, (\d+), \d+>$", kernel).group(1))
    return 2 if "ssam3d_fused" in kernel or "ssam3d_star2" in kernel else 1


def sq(dirs, out_md: str) -> None:
    """VALU utilisation per kernel from one pass of 8 SQ counters per directory."""
    ctrs = "SQ_WAVE_CYCLES SQ_BUSY_CYCLES SQ_INSTS_MFMA SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS SQ_INSTS_VALU SQ_INSTS_LDS SQ_WAIT_ANY"
    out = ["# VALU utilisation of the benchmark kernels (rocprofv3 SQ counters)\n",
           "One MI355X, one counter pass per configuration (8 SQ counters):\n",
           f"    rocprofv3 --pmc {ctrs} --kernel-trace --output-format csv -d <dir> -o c -- python3 bench.py --workload config<N> "
           "--no-cpu-baseline --steps 1 --warmup 0\n",
           "Per dispatch, mean over the dispatches of a kernel.  `VALU instr / point / sweep` = SQ_INSTS_VALU x 64 lanes / (grid "
           "points x sweeps of the launch): what one output costs in lane-instructions, halo lanes and warm-up rows included.  "
           "`VALU busy` = (SQ_ACTIVE_INST_VALU + SQ_INSTS_MFMA) x 4 cycles / (1024 SIMDs x dispatch duration x 2.4 GHz): the "
           "fraction of all VALU issue slots of the chip the kernel used.  `MFMA share` = SQ_INSTS_MFMA / SQ_INSTS_VALU.  "
           "`waiting` = SQ_WAIT_ANY / SQ_WAVE_CYCLES: share of wave-cycles spent waiting on any counter (memory, LDS).  "
           "Durations are those of the counter run (serialised dispatches), a few per cent above the timed runs.\n",
           "| run | kernel | dispatches | duration us | sweeps | VALU instr / point / sweep | VALU busy | MFMA share | "
           "LDS instr / VALU instr | waiting |\n|---|---|---|---|---|---|---|---|---|---|"]
    for d in dirs:
        bench = json.load(open(d.rstrip("/") + ".json"))
        pts = 1
        for s in bench["config"]["grid"].split("x"):
            pts *= int(s)
        agg = collections.OrderedDict()
        for k, c, us in counter_dispatches(d):
            if ours(k):
                agg.setdefault(k, []).append((c, us))
        for k, rows in agg.items():
            m = {name: sum(r[0].get(name, 0.0) for r in rows) / len(rows) for name in ctrs.split()}
            us = sum(r[1] for r in rows) / len(rows)
            sw = sweeps_of(k)
            out.append(f"| {os.path.basename(d.rstrip('/'))} | `{k}` | {len(rows)} | {us:.1f} | {sw} | "
                       f"{m['SQ_INSTS_VALU'] * 64 / pts / sw:.1f} | "
                       f"{(m['SQ_ACTIVE_INST_VALU'] + m['SQ_INSTS_MFMA']) * 4 / (1024 * us * 1e-6 * 2.4e9):.2f} | "
                       f"{m['SQ_INSTS_MFMA'] / max(m['SQ_INSTS_VALU'], 1):.2f} | {m['SQ_INSTS_LDS'] / max(m['SQ_INSTS_VALU'], 1):.3f} | "
                       f"{m['SQ_WAIT_ANY'] / max(m['SQ_WAVE_CYCLES'], 1):.2f} |")
    open(out_md, "w").write("\n".join(out) + "\n")
    print("\n".join(out))


def lds(dirs, out_md: str) -> None:
    """LDS bank conflicts of the kernels that use LDS."""
    ctrs = "SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_LDS_ADDR_CONFLICT SQ_INSTS_LDS SQ_ACTIVE_INST_LDS SQ_WAVE_CYCLES SQ_BUSY_CYCLES SQ_WAIT_INST_LDS"
    out = ["# LDS bank conflicts of the kernels that use LDS (rocprofv3 SQ counters)\n",
           "One MI355X, one counter pass per configuration:\n",
           f"    rocprofv3 --pmc {ctrs} --kernel-trace --output-format csv -d <dir> -o c -- python3 bench.py --workload config<N> "
           "--no-cpu-baseline --steps 1 --warmup 0\n",
           "Per dispatch, mean over the dispatches of a kernel.  `conflict share` = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE: "
           "cycles the LDS spent replaying bank conflicts over the cycles it was busy with indexed accesses.  `LDS busy` = "
           "SQ_LDS_IDX_ACTIVE / (256 CUs x dispatch duration x 2.4 GHz).  Kernels that issue no LDS instruction are left out.\n",
           "| run | kernel | dispatches | duration us | LDS instructions | conflict cycles | LDS active cycles | conflict share | LDS busy |\n"
           "|---|---|---|---|---|---|---|---|---|"]
    for d in dirs:
        agg = collections.OrderedDict()
        for k, c, us in counter_dispatches(d):
            if ours(k):
                agg.setdefault(k, []).append((c, us))
        for k, rows in agg.items():
            m = {name: sum(r[0].get(name, 0.0) for r in rows) / len(rows) for name in ctrs.split()}
            if m["SQ_INSTS_LDS"] == 0:
                continue
            us = sum(r[1] for r in rows) / len(rows)
            out.append(f"| {os.path.basename(d.rstrip('/'))} | `{k}` | {len(rows)} | {us:.1f} | {m['SQ_INSTS_LDS']:.0f} | "
                       f"{m['SQ_LDS_BANK_CONFLICT']:.0f} | {m['SQ_LDS_IDX_ACTIVE']:.0f} | "
                       f"{m['SQ_LDS_BANK_CONFLICT'] / max(m['SQ_LDS_IDX_ACTIVE'], 1):.3f} | "
                       f"{m['SQ_LDS_IDX_ACTIVE'] / (256 * us * 1e-6 * 2.4e9):.2f} |")
    open(out_md, "w").write("\n".join(out) + "\n")
    print("\n".join(out))


def resources(out_md: str, only_default: bool = True) -> None:
    from . import build
    flags = [f for f in build.FLAGS if f not in ("-fPIC",)]
    rows = []
    for src in sorted(glob.glob(os.path.join(build.CSRC, "*.hip"))):
        res = subprocess.run(["hipcc", *flags, "--cuda-device-only", "-c", src, "-o", "/dev/null",
                              "-Rpass-analysis=kernel-resource-usage"], capture_output=True, text=True)
        if res.returncode != 0:
            raise SystemExit(res.stderr)
        cur = None
        for line in res.stderr.splitlines():
            m = re.search(r"remark:\s+(Function Name|VGPRs|AGPRs|TotalSGPRs|ScratchSize \[bytes/lane\]|Occupancy \[waves/SIMD\]|LDS Size \[bytes/block\]): (\S+)", line)
            if not m:
                continue
            if m.group(1) == "Function Name":
                name = subprocess.run(["c++filt", m.group(2)], capture_output=True, text=True).stdout.strip()
                cur = {"file": os.path.basename(src), "src": src, "mangled": m.group(2), "kernel": short(name)}
                rows.append(cur)
            elif cur is not None:
                cur[m.group(1).split(" [")[0]] = m.group(2)
    # A private segment can be reserved without ever being used (slots of scalar-register spills that ended up in
    # vector-register lanes): for the kernels that report one, count the scratch instructions in the assembly.
    for src in sorted({r["src"] for r in rows if r.get("ScratchSize", "0") != "0"}):
        asm = subprocess.run(["hipcc", *flags, "--cuda-device-only", "-S", src, "-o", "-"], capture_output=True, text=True)
        if asm.returncode != 0:
            raise SystemExit(asm.stderr)
        for body in re.split(r"\n\t\.type\t", asm.stdout)[1:]:
            mangled = body.split(",")[0]
            for r in rows:
                if r.get("mangled") == mangled:
                    r["scratch_instructions"] = len(re.findall(r"\bscratch_(?:load|store)", body))
    spilled = [r for r in rows if r.get("ScratchSize", "0") != "0"]
    out = ["# Registers, LDS and scratch of every compiled kernel (gfx950)\n",
           "From the compiler's resource report, no GPU involved:\n",
           "    python -m paper_1907_06154_amd.profiling resources profiles/kernel_resources.md\n",
           "(`hipcc --offload-arch=gfx950 -O3 ... --cuda-device-only -Rpass-analysis=kernel-resource-usage` per translation unit.)  "
           "VGPRs + AGPRs share one file of 512 registers per SIMD lane: waves per SIMD = floor(512 / (VGPRs + AGPRs, rounded up "
           "to 8)), at most 8; a block's LDS also limits the blocks per compute unit (160 KiB).  Kernels for which the compiler "
           "reserves a private segment (bytes per lane; scratch loads and stores in their code): "
           + (", ".join(f"`{r['kernel']}` ({r.get('ScratchSize')}; {r.get('scratch_instructions', '?')})" for r in spilled) or "none")
           + ".  A reserved segment without scratch instructions is never touched: its slots belonged to scalar-register "
           "spills that ended up in vector-register lanes.\n",
           "| translation unit | kernel | VGPRs | AGPRs | SGPRs | LDS bytes / block | scratch bytes / lane | waves / SIMD |\n|---|---|---|---|---|---|---|---|"]
    for r in rows:
        out.append(f"| {r['file']} | `{r['kernel']}` | {r.get('VGPRs', '')} | {r.get('AGPRs', '')} | {r.get('TotalSGPRs', '')} | "
                   f"{r.get('LDS Size', '')} | {r.get('ScratchSize', '')} | {r.get('Occupancy', '')} |")
    open(out_md, "w").write("\n".join(out) + "\n")
    print(f"{len(rows)} kernels -> {out_md}")


def catalogue(single_json: str, default_json: str, out_md: str) -> None:
    """Table 3 catalogue: two bench.py runs of --workload table3 (one sweep per launch / default)."""
    a, b = json.load(open(single_json)), json.load(open(default_json))
    out = ["# bench.py timing: Stencil shapes of Table 3 (paper Sec. 6.3): 2D on 8192^2, 3D on 512^3, fp32 and fp64, zero padding\n",
           "One MI355X, HIP events on the launch stream, medians.  Two runs: one sweep per launch, and the library's default, where "
           "`ssam_stencil_iterate` runs several sweeps per launch for the shapes that have a multi-sweep instance (2D r <= 6; 3D "
           "r = 1: the three fp64 shapes and the fp32 7-point star).  `2d64pt`, an 8x8 box, runs as one pass of a dense 8x8 filter.\n",
           f"    python bench.py --workload table3 --no-cpu-baseline --steps {a['steps']} --fuse-sweeps 0 > {single_json}\n"
           f"    python bench.py --workload table3 --no-cpu-baseline --steps {b['steps']} > {default_json}\n"
           f"    python -m paper_1907_06154_amd.profiling catalogue {single_json} {default_json} {os.path.relpath(out_md, ROOT)}\n",
           f"Whole-step throughput {a['value']:.1f} GStencil/s ({a['ms_per_step']:.2f} ms per step) with single sweeps, "
           f"{b['value']:.1f} GStencil/s ({b['ms_per_step']:.2f} ms) by default; plain grid-stride copy on the first case's buffers "
           f"{b['plain_copy_GBps']:.0f} GB/s.\n",
           "Single-sweep columns: launch time, GStencil/s, algorithmic GB/s (one read + one write per sweep) as a fraction of "
           "8 TB/s, TFLOP/s as a fraction of the published vector peak (157.3 fp32, 78.6 fp64).  Default columns: instance used "
           "for most launches, launches per run, GStencil/s and the gain.\n",
           "| case | single-sweep instance | launch us | GStencil/s | GB/s | of 8 TB/s | TFLOP/s | of peak | bound | default instance "
           "| launches | GStencil/s | gain |\n|---|---|---|---|---|---|---|---|---|---|---|---|---|"]
    kb = {k["case"]: k for k in b["kernels"]}
    for k in a["kernels"]:
        f = kb[k["case"]]
        out.append(f"| {k['case']} | `{k['kernel']}` | {k['launch_ms'] * 1e3:.1f} | {k['gstencil_per_s']:.1f} | {k['hbm_GBps']:.0f} | "
                   f"{k['hbm_frac']:.3f} | {k['alu_TFLOPs']:.1f} | {k['alu_frac']:.3f} | {k['bound']} | `{f['kernel']}` | "
                   f"{f['launches_per_step']} | {f['gstencil_per_s']:.1f} | {f['gstencil_per_s'] / k['gstencil_per_s']:.2f}x |")
    open(out_md, "w").write("\n".join(out) + "\n")
    print("\n".join(out))


def sweep(default_json: str, vector_json: str, out_md: str) -> None:
    """Filter sweep 2x2 .. 20x20: bench.py --workload filter_sweep by default and with --tune-variant 5
    (the vector-unit instances of the filters whose defaults run on the matrix cores)."""
    a, v = json.load(open(default_json)), json.load(open(vector_json))
    out = ["# bench.py timing: Filter sweep 2x2 .. 20x20 (paper Sec. 6.2), 8192x8192 fp32, clamp\n",
           "One MI355X, HIP events on the launch stream, medians per launch; every launch reads a different one of four copies "
           "of the image, so nothing it reads is resident in the memory-side cache (cold, as in `bench.py` without arguments).  "
           "Second run: tuning variant 5, the "
           "vector-unit instances of the filters whose default instances (`...mx`) evaluate their products on the matrix cores "
           "(shapes without such an alternative run their default in both).\n",
           f"    python bench.py --workload filter_sweep --no-cpu-baseline --steps {a['steps']} --warmup {a['warmup']} > {default_json}\n"
           f"    python bench.py --workload filter_sweep --no-cpu-baseline --steps {v['steps']} --warmup {v['warmup']} --variant 5 > {vector_json}\n"
           f"    python -m paper_1907_06154_amd.profiling sweep {default_json} {vector_json} {os.path.relpath(out_md, ROOT)}\n",
           f"Whole-step throughput {a['value']:.1f} GStencil/s, {a['ms_per_step']:.2f} ms per step (variant 5: {v['value']:.1f}, "
           f"{v['ms_per_step']:.2f} ms); plain grid-stride copy on the same buffers {a['plain_copy_GBps']:.0f} GB/s.\n",
           "Fractions: algorithmic GB/s of 8 TB/s; TFLOP/s of 157.3 (the published fp32 vector peak, which assumes packed FMA and "
           "equals the fp32 matrix peak; the non-packed vector rate reachable here is 78.6).\n",
           "| case | kernel instance | launch us | GStencil/s | algorithmic GB/s | of 8 TB/s | TFLOP/s | of 157.3 | bound | "
           "vector-unit instance | launch us | GStencil/s | of 78.6 TFLOP/s |\n|---|---|---|---|---|---|---|---|---|---|---|---|---|"]
    kv = {k["case"]: k for k in v["kernels"]}
    for k in a["kernels"]:
        u = kv[k["case"]]
        out.append(f"| {k['case']} | `{k['kernel']}` | {k['launch_ms'] * 1e3:.1f} | {k['gstencil_per_s']:.1f} | {k['hbm_GBps']:.0f} | "
                   f"{k['hbm_frac']:.3f} | {k['alu_TFLOPs']:.1f} | {k['alu_frac']:.3f} | {k['bound']} | `{u['kernel']}` | "
                   f"{u['launch_ms'] * 1e3:.1f} | {u['gstencil_per_s']:.1f} | {u['alu_TFLOPs'] / 78.6:.3f} |")
    open(out_md, "w").write("\n".join(out) + "\n")
    print("\n".join(out))


def scan_summary(prefix: str, out_md: str) -> None:
    """The scan: <prefix>/<tag>_{trace,fetch,write}/ (rocprofv3 output) and <prefix>/<tag>_trace.txt (what the traced
    bench.py --tune run printed), tag = f32, f64; both schedules of the 1 GiB arrays in every run."""
    out = ["# rocprofv3 summary: inclusive scan (ssam_scan), 1 GiB arrays: 2^28 fp32 and 2^27 fp64 elements, both schedules\n",
           "Both schedules are timed by the same command (`scan_chained=0`: three launches, `scan_chained=1`: one pass, the "
           "default at this size), followed by the plain copy kernel on the same arrays.\n"]
    traffic = load_traffic()
    for tag, n, tname in (("f32", 1 << 28, "float"), ("f64", 1 << 27, "double")):
        cmd = f'python3 bench.py --workload scan --cases {tag}:{n} --tune "scan_chained=0,1"'
        out.append(f"## {tag}, n = {n}\n\nKernel durations:\n")
        out.append(f"    rocprofv3 --kernel-trace --stats --output-format csv -d {prefix}/{tag}_trace -o c -- {cmd}\n")
        out.append("From the kernel trace of that run; `scan_one_group` is the one-workgroup fallback enqueued behind every "
                   "one-pass call; it returns at once unless a wave gave up (never in these runs):\n")
        out.append("| kernel | dispatches | avg us | min us | max us |\n|---|---|---|---|---|")
        for r in csv.DictReader(open(one(os.path.join(prefix, tag + "_trace", "**", "*kernel_stats.csv")))):
            if ours(r["Name"]) or is_copy(r["Name"]):
                out.append(f"| `{short(r['Name'])}` | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | "
                           f"{float(r['MinNs']) / 1e3:.1f} | {float(r['MaxNs']) / 1e3:.1f} |")
        out.append("\nThe same run's HIP-event timing per call (all launches of the call; algorithmic bytes = one read + one "
                   "write per element):\n\n```")
        out += [l.rstrip() for l in open(os.path.join(prefix, tag + "_trace.txt")) if l.startswith(("scan ", "copy "))]
        out.append("```\n\nHBM traffic counters (each in a run of its own; KiB per dispatch, mean over dispatches):\n")
        per = {}
        copy = {}
        for kind, ctr in (("fetch", "FETCH_SIZE"), ("write", "WRITE_SIZE")):
            out.append(f"    rocprofv3 --pmc {ctr} --kernel-trace --output-format csv -d {prefix}/{tag}_{kind} -o c -- {cmd}")
            for k, c, _ in counter_dispatches(os.path.join(prefix, f"{tag}_{kind}")):
                if is_copy(k):
                    copy.setdefault(kind, []).append(c[ctr])
                elif k.startswith("scan_"):
                    per.setdefault(k, {"fetch": [], "write": []})[kind].append(c[ctr])
        array_kib = (1 << 30) / 1024.0
        scale = {kind: array_kib / (sum(v) / len(v)) for kind, v in copy.items()}
        out.append(f"\nThe plain copy kernel (`ssam_probe_copy`, 1024 MiB read and written) reads FETCH_SIZE = "
                   f"{sum(copy['fetch']) / len(copy['fetch']):.0f} KiB and WRITE_SIZE = {sum(copy['write']) / len(copy['write']):.0f} "
                   f"KiB: scale factors {scale['fetch']:.3f} (fetch) and {scale['write']:.3f} (write).\n")
        out.append("| kernel | dispatches | FETCH_SIZE KiB | WRITE_SIZE KiB | scaled read MiB | scaled write MiB | "
                   "read+write / array size |\n|---|---|---|---|---|---|---|")
        for k, v in per.items():
            f = sum(v["fetch"]) / max(1, len(v["fetch"]))
            w = sum(v["write"]) / max(1, len(v["write"]))
            tot = (f * scale["fetch"] + w * scale["write"]) / 1024
            out.append(f"| `{k}` | {len(v['fetch'])} | {f:.0f} | {w:.0f} | {f * scale['fetch'] / 1024:.1f} | "
                       f"{w * scale['write'] / 1024:.1f} | {tot / 1024:.3f} |")
            if k.startswith("scan_chained"):
                key = f"scan_chained_{tag}@{n}"
                traffic["bytes_per_launch"][key] = int(tot * 2 ** 20)
                traffic["source"][key] = os.path.relpath(out_md, ROOT)
        out.append("")
    open(out_md, "w").write("\n".join(out) + "\n")
    json.dump(traffic, open(TRAFFIC, "w"), indent=1, sort_keys=True)
    print("\n".join(out))


def main(argv) -> int:
    if len(argv) >= 3 and argv[0] == "summarize":
        title = argv[argv.index("--title") + 1]
        bargs = argv[argv.index("--bench-args") + 1]
        summarize(argv[1], argv[2], title, bargs)
    elif len(argv) >= 3 and argv[0] == "sq":
        sq(argv[1:-1], argv[-1])
    elif len(argv) >= 3 and argv[0] == "lds":
        lds(argv[1:-1], argv[-1])
    elif len(argv) == 4 and argv[0] == "catalogue":
        catalogue(argv[1], argv[2], argv[3])
    elif len(argv) == 4 and argv[0] == "sweep":
        sweep(argv[1], argv[2], argv[3])
    elif len(argv) == 3 and argv[0] == "scan":
        scan_summary(argv[1], argv[2])
    elif len(argv) == 2 and argv[0] == "resources":
        resources(argv[1])
    else:
        print(__doc__)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
