"""Prints the gfx950 latency table (the counterpart of Table 2 of the paper's performance model).

    python -m paper_1907_06154_amd.latency [chain]

For every primitive: shader-clock ticks per operation of one dependent chain in one wave
(latency), the same with 8 independent chains per wave, with 4 such waves (one per SIMD: shared
units such as the LDS show up), and with 16 waves (4 per SIMD) of 8 chains each, where the block's
span divided by 4 waves x 8 chains is the issue cost per operation on one SIMD.  The nanosecond column of the first measurement gives the clock the part ran at.
"""
from __future__ import annotations

import sys


def table(chain: int = 1 << 15):
    import torch

    import paper_1907_06154_amd as ssam
    from paper_1907_06154_amd.binding import PROBE_OPS, PROBE_SCRATCH_BYTES

    scratch = torch.empty(PROBE_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
    rows = []
    for op in PROBE_OPS:
        ssam.ssam_probe_latency(op, 1, 1, chain, scratch)   # warm-up launch (code upload, clocks)
        lat, ns = ssam.ssam_probe_latency(op, 1, 1, chain, scratch)
        ilp8, _ = ssam.ssam_probe_latency(op, 8, 1, chain, scratch)
        full, _ = ssam.ssam_probe_latency(op, 8, 16, chain, scratch)
        one, _ = ssam.ssam_probe_latency(op, 8, 4, chain, scratch)
        rows.append({"op": op, "latency_cycles": lat, "latency_ns": ns, "clock_GHz": lat / ns if ns > 0 else float("nan"),
                     "cycles_per_op_ilp8": ilp8 / 8, "cu_4waves": one / 8, "simd_issue_cycles_per_op": full / 32})
    return rows


def main(argv) -> int:
    chain = int(argv[0]) if argv else 1 << 15
    rows = table(chain)
    print("| operation | latency, cycles (1 wave, 1 chain) | ns | implied clock GHz | cycles per op, 8 chains in 1 wave | "
          "same, 4 waves (1 per SIMD) | cycles per op and SIMD, 16 waves x 8 chains |")
    print("|---|---|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['op']} | {r['latency_cycles']:.1f} | {r['latency_ns']:.2f} | {r['clock_GHz']:.2f} | "
              f"{r['cycles_per_op_ilp8']:.2f} | {r['cu_4waves']:.2f} | {r['simd_issue_cycles_per_op']:.2f} |")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
