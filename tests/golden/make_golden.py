"""Writes tests/golden/oracle_lock.txt: oracle outputs on small seeded cases, as hex floats.

Calls only oracle/ and the seeded input generators.  The file locks the (generator, oracle)
pair against silent drift; it is not a pin (the pins are in tests/test_oracle_pins.py).

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import workloads as wl  # noqa: E402


def cases():
    c1 = wl.config1(8)[0]
    yield "config1_8x8_5pt_f32_zero", oracle.stencil(c1.field(), c1.coef[0], "zero")
    img = wl.uniform_field((6, 7), 0.0, 1.0, 3, np.float32)
    yield "conv3x11_6x7_f32_clamp", oracle.conv2d(img, wl.seeded_filter(3, 11, 9, np.float32), "clamp")
    f3 = wl.uniform_field((4, 5, 6), -1.0, 1.0, 6, np.float64)
    yield "faces_edges_4x5x6_f64_zero_3sweeps", oracle.iterate(f3, wl.seeded_coefficients(wl.mask_faces_edges(), 62, np.float64), 3)
    yield "star_r4_4x5x6_f64_clamp", oracle.stencil(f3, wl.seeded_symmetric_star(4, 3, 70, np.float64), "clamp")
    filt3 = wl.uniform_field((2, 3, 4), -1.0, 1.0, 71, np.float64)      # even and odd extents, anchor off the centre
    yield "conv3d_4x3x2_anchor_3_0_1_4x5x6_f64_zero", oracle.conv3d(f3, filt3, "zero", anchor=(3, 0, 1))
    yield "scan_37_f32", oracle.scan(wl.uniform_field((37,), -1.0, 1.0, 72, np.float32))


def render():
    lines = []
    for name, arr in cases():
        lines.append(f"{name} {arr.dtype.name} " + "x".join(str(s) for s in arr.shape))
        lines.append(" ".join(float(v).hex() for v in arr.ravel()))
    return "\n".join(lines) + "\n"


if __name__ == "__main__":
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_lock.txt"), "w") as f:
        f.write(render())
