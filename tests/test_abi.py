"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol the
public header declares, validates its arguments before any GPU call, and plans tile
geometry as the design states.  Every call that is given made-up pointers fails validation
before anything is launched, so the file is safe to run on a machine with a GPU as well (where
the one call that passes validation gets real device memory)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1907_06154_amd as ssam
import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_A, FAKE_B = 0x10000000, 0x50000000      # never dereferenced: every call that gets them fails validation first


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(ssam.binding.LIB_PATH):
        from paper_1907_06154_amd import build
        build.build()
    return ssam.lib()


def declared_symbols():
    import glob
    names = set()
    for header in glob.glob(os.path.join(ROOT, "include", "*.h")):
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names |= set(re.findall(r"\b(ssam_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(L):
    names = declared_symbols()
    assert {"ssam_conv2d", "ssam_conv3d", "ssam_stencil2d", "ssam_stencil3d", "ssam_stencil_iterate", "ssam_scan",
            "ssam_scan_static", "ssam_set_tuning", "ssam_probe_copy"} <= set(names)
    for n in names:
        assert hasattr(L, n), f"{n} declared under include/ but not exported"


def test_status_strings(L):
    seen = {ssam.status_string(i) for i in range(7)}
    assert len(seen) == 7 and ssam.status_string(0) == "ok" and ssam.status_string(99) == "unknown status"


def conv(L, d_in=FAKE_A, d_out=FAKE_B, W=64, H=64, filt=None, M=3, N=3, ax=-1, ay=-1, boundary=1, dtype=0):
    f = np.ones((max(N, 1), max(M, 1)), dtype=np.float32) if filt is None else filt
    fp = None if filt is False else f.ctypes.data
    return L.ssam_conv2d(d_in, d_out, W, H, fp, M, N, ax, ay, boundary, dtype, None)


def test_conv2d_validation(L):
    assert conv(L, d_in=None) == 1 and conv(L, d_out=None) == 1 and conv(L, filt=False) == 1
    assert conv(L, W=0) == 2 and conv(L, H=-3) == 2 and conv(L, W=65536, H=65536) == 2
    assert conv(L, M=0) == 3 and conv(L, N=33) == 3 and conv(L, ax=3) == 3 and conv(L, ay=-2) == 3
    assert conv(L, boundary=2) == 4 and conv(L, dtype=7) == 4
    assert conv(L, d_out=FAKE_A) == 5 and conv(L, d_out=FAKE_A + 64 * 64 * 4 - 4) == 5
    # an output that starts right behind the input is no alias.  That call passes validation, so it launches:
    # with a GPU present it gets real memory (without one the launch fails, which is all this line needs)
    import torch
    if torch.cuda.is_available():
        both = torch.zeros(2 * 64 * 64, dtype=torch.float32, device="cuda")
        assert conv(L, d_in=both.data_ptr(), d_out=both.data_ptr() + 64 * 64 * 4) == 0
        torch.cuda.synchronize()
    else:
        assert conv(L, d_out=FAKE_A + 64 * 64 * 4) != 5


def test_conv3d_validation_and_plan(L):
    f = np.ones((3, 3, 3), dtype=np.float32)

    def call(d_in=FAKE_A, d_out=FAKE_B, W=32, H=32, D=32, filt=f, M=3, N=3, K=3, ax=-1, ay=-1, az=-1, boundary=1, dtype=0):
        return L.ssam_conv3d(d_in, d_out, W, H, D, None if filt is None else filt.ctypes.data, M, N, K, ax, ay, az,
                             boundary, dtype, None)

    assert call(d_in=None) == 1 and call(d_out=None) == 1 and call(filt=None) == 1
    assert call(W=0) == 2 and call(D=-1) == 2 and call(W=2048, H=2048, D=1024) == 2
    assert call(M=0) == 3 and call(K=18) == 3 and call(ax=3) == 3 and call(az=-2) == 3
    assert call(boundary=3) == 4 and call(dtype=2) == 4
    assert call(d_out=FAKE_A) == 5 and call(d_out=FAKE_A + 32 * 32 * 32 * 4 - 4) == 5
    # the plan: compiled cubes, embedding within a waste limit, the direct kernel for the rest
    for shape, prefix in (((3, 3, 3), "float_r111_b3"), ((5, 5, 5), "float_r222_b3"), ((7, 7, 7), "float_r333_b3")):
        assert ssam.ssam_describe("conv3d", (64, 64, 64), np.ones(shape, dtype=np.float32), "clamp").split()[0].startswith(prefix)
    assert ssam.ssam_describe("conv3d", (64, 64, 64), np.ones((2, 2, 2)), "zero").split()[0] == "double_r111_b3_p4w8star_ring3nt2+embedded"
    for shape in ((9, 9, 9), (17, 17, 17), (6, 1, 1), (8, 8, 2)):
        assert ssam.ssam_describe("conv3d", (64, 64, 64), np.ones(shape), "zero").split()[0] == "generic_direct"


def test_stencil_validation(L):
    c = np.ones(27, dtype=np.float64)
    cp = c.ctypes.data
    assert L.ssam_stencil2d(None, FAKE_B, 8, 8, cp, 1, 1, 0, 1, None) == 1
    assert L.ssam_stencil2d(FAKE_A, FAKE_B, 8, 0, cp, 1, 1, 0, 1, None) == 2
    assert L.ssam_stencil2d(FAKE_A, FAKE_B, 8, 8, cp, -1, 1, 0, 1, None) == 3
    assert L.ssam_stencil2d(FAKE_A, FAKE_B, 8, 8, cp, 9, 1, 0, 1, None) == 3
    assert L.ssam_stencil2d(FAKE_A, FAKE_B, 8, 8, cp, 1, 1, 5, 1, None) == 4
    assert L.ssam_stencil3d(FAKE_A, FAKE_A, 8, 8, 8, cp, 1, 1, 1, 0, 1, None) == 5
    assert L.ssam_stencil3d(FAKE_A, FAKE_B, 8, 8, -1, cp, 1, 1, 1, 0, 1, None) == 2
    assert L.ssam_stencil3d(FAKE_A, FAKE_B, 2048, 2048, 2048, cp, 1, 1, 1, 0, 1, None) == 2
    res = ctypes.c_void_p(0)
    assert L.ssam_stencil_iterate(FAKE_A, FAKE_B, 8, 8, 8, cp, 1, 1, 1, 0, 1, -1, None, ctypes.byref(res)) == 3
    assert L.ssam_stencil_iterate(FAKE_A, FAKE_A + 8, 8, 8, 8, cp, 1, 1, 1, 0, 1, 3, None, ctypes.byref(res)) == 5
    # zero steps: nothing to launch, the field stays in d_a
    assert L.ssam_stencil_iterate(FAKE_A, FAKE_B, 8, 8, 8, cp, 1, 1, 1, 0, 1, 0, None, ctypes.byref(res)) == 0
    assert res.value == FAKE_A


def test_tuning_names(L):
    assert L.ssam_set_tuning(b"rows_per_wave", 16) == 0 and L.ssam_set_tuning(b"rows_per_wave", -1) == 0
    assert L.ssam_set_tuning(b"no_such_knob", 1) == 4 and L.ssam_set_tuning(None, 1) == 1


def test_scan_plan_and_validation(L):
    """Workspace sizing and argument checks of ssam_scan; every call here fails validation (or is
    empty) before anything is launched."""
    vp = ctypes.c_void_p
    ws = L.ssam_scan_workspace_bytes
    assert ws(0, 0) == 0 and ws(-5, 0) == 0 and ws(1000, 9) == 0
    assert ws(32768, 0) == 0 and ws(16384, 1) == 0              # up to 128 KiB: one workgroup, no workspace
    assert ws(32769, 0) == 8 * 33 and ws(16385, 1) == 8 * 33    # beyond: segments of 4 wave-rounds
    assert L.ssam_set_tuning(b"scan_one_group", 0) == 0
    assert ws(1024, 0) == 0 and ws(512, 1) == 0                 # one segment: no workspace
    assert ws(1025, 0) == 16 and ws(513, 1) == 16               # two segments
    assert L.ssam_set_tuning(b"scan_one_group", -1) == 0
    # arrays of 128 MiB and more, up to 64^3 register-resident segments of 16 KiB: the one-pass schedule
    # (ticket and flag, 64 padded + 4096 + one per segment published sums of 8 bytes); the three
    # launches use at most 4096 segments
    one_pass = lambda segs: 8 * (32 + 16 * 64 + 4096 + segs)
    assert ws((1 << 25) - 1, 0) == 8 * 4096 and ws(1 << 25, 0) == one_pass(1 << 13)
    assert ws(1 << 28, 0) == one_pass(1 << 16) and ws(1 << 28, 1) == one_pass(1 << 17)
    assert ws(1 << 30, 0) == one_pass(1 << 18) and 8 * 4000 < ws((1 << 30) + 1, 0) <= 8 * 4096
    assert ws(1 << 40, 1) == 8 * 4096 and ws((1 << 40) + 1, 1) == 0
    assert L.ssam_set_tuning(b"scan_chained", 0) == 0 and ws(1 << 28, 0) == 8 * 4096
    assert L.ssam_set_tuning(b"scan_chained", 1) == 0 and ws(5000, 0) == one_pass(2)
    assert L.ssam_set_tuning(b"scan_chained", -1) == 0 and L.ssam_set_tuning(b"scan_spin_limit", -1) == 0
    n = 1 << 20
    assert L.ssam_scan(vp(FAKE_A), vp(FAKE_B), 0, 0, None, 0, None) == 0          # empty: no-op
    assert L.ssam_scan(None, None, 0, 1, None, 0, None) == 0
    assert L.ssam_scan(vp(FAKE_A), vp(FAKE_B), n, 2, vp(0x90000000), 1 << 18, None) == 4
    assert L.ssam_scan(vp(FAKE_A), vp(FAKE_B), -1, 0, vp(0x90000000), 1 << 18, None) == 2
    assert L.ssam_scan(None, vp(FAKE_B), n, 0, vp(0x90000000), 1 << 18, None) == 1
    assert L.ssam_scan(vp(FAKE_A), None, n, 0, vp(0x90000000), 1 << 18, None) == 1
    assert L.ssam_scan(vp(FAKE_A + 2), vp(FAKE_B), n, 0, vp(0x90000000), 1 << 18, None) == 2
    assert L.ssam_scan(vp(FAKE_A), vp(FAKE_A + 4096), n, 0, vp(0x90000000), 1 << 18, None) == 5
    assert L.ssam_scan(vp(FAKE_A), vp(FAKE_B), n, 0, None, 0, None) == 1
    assert L.ssam_scan(vp(FAKE_A), vp(FAKE_B), n, 0, vp(0x90000000), ws(n, 0) - 1, None) == 2
    assert L.ssam_scan(vp(FAKE_A), vp(FAKE_B), n, 0, vp(0x90000004), 1 << 18, None) == 2
    assert L.ssam_scan(vp(FAKE_A), vp(FAKE_B), n, 0, vp(FAKE_B + 64), 1 << 18, None) == 5


def parse(desc):
    name, *kv = desc.split()
    out = {}
    for item in kv:
        k, v = item.split("=")
        out[k] = sum(int(t) for t in v.split("+")) if k == "halo_lanes" else int(v)
    return name, out


def test_dense_fp32_filters_from_7x7_on_use_the_matrix_cores(L):
    """The default instance of a dense fp32 square filter evaluates its column products on the matrix
    cores ("...mx") from 7x7 on; variant 5 is the vector-unit instance of the same shape; smaller
    filters and fp64 have the vector-unit kernels only."""
    for m in range(2, 21):
        f = wl.seeded_filter(m, m, 1, np.float32)
        name, g = parse(ssam.ssam_describe("conv2d", (2048, 2048), f, "clamp"))
        assert name.startswith("float_M%dN%d_b2" % (m, m)) and name.endswith("mx") == (m >= 7), name
        if m >= 7:
            assert g["P"] == 4 and g["V"] == 4
            ssam.ssam_set_tuning("variant", 5)
            other, _ = parse(ssam.ssam_describe("conv2d", (2048, 2048), f, "clamp"))
            ssam.ssam_set_tuning("variant", -1)
            assert other.startswith("float_M%dN%d_b2" % (m, m)) and not other.endswith("mx"), other
    c = wl.seeded_coefficients(wl.mask_box(4, 4), 3, np.float64)[0]
    name, _ = parse(ssam.ssam_describe("stencil2d", (2048, 2048), c, "zero"))
    assert name.startswith("double_M9N9_b2") and not name.endswith("mx")


def test_overlapped_blocking_geometry(L):
    """Tile plan re-derived from Sec. 4.5 / 4.7 for 64 lanes of V columns: a wave caches 64*V
    columns, stores valid_lanes*V of them (valid_lanes <= 64 - halo lanes), and the strips cover W."""
    for (M, N) in wl.CONV_SHAPES:
        f = wl.seeded_filter(M, N, 1, np.float32)
        name, g = parse(ssam.ssam_describe("conv2d", (8192, 8192), f, "clamp"))
        assert name.startswith("float_M%dN%d_b2" % (M, N))
        V = g["V"]
        hl, hr = -(-(M // 2) // V), -(-(M - 1 - M // 2) // V)
        assert V == 4 and g["halo_lanes"] == hl + hr
        assert g["valid_lanes"] <= 64 - hl - hr
        assert g["strips_x"] * g["valid_lanes"] * V >= 8192 > (g["strips_x"] - 1) * g["valid_lanes"] * V
        assert g["rows_per_wave"] % g["P"] == 0 and g["tiles_y"] * g["rows_per_wave"] >= 8192
        assert g["tiles"] == g["strips_x"] * g["tiles_y"] and g["blocks"] * 4 >= g["tiles"]
        assert g["blocks"] % 8 == 0


def test_shape_classification(L):
    cases = {
        "c1_2d5pt_f32": "float_M3N3_b1", "c3_2d_box_r1_f64": "double_M3N3_b2", "c3_2d_box_r2_f64": "double_M5N5_b2",
        "c3_2d_star_r4_f64": "double_M9N9_b1", "c4_3d_star_r1_f64": "double_r111_b1",
        "c4_3d_box_r1_f64": "double_r111_b3", "c4_3d_faces_edges_f64": "double_r111_b2",
        "c5_3d_star_r4_f32": "float_r444_b1", "c5_3d_star_r4_f64": "double_r444_b1",
    }
    allc = {c.name: c for cs in wl.all_configs().values() for c in cs}
    for nm, prefix in cases.items():
        c = allc[nm]
        coef = c.coef if c.kind == "stencil3d" else c.coef[0]
        name, g = parse(ssam.ssam_describe(c.kind, c.shape, coef, c.boundary))
        assert name.startswith(prefix), (nm, name)
    # a shape without a compiled instance runs inside the smallest compiled square box that holds it ...
    name, g = parse(ssam.ssam_describe("conv2d", (100, 100), np.ones((4, 7), dtype=np.float32), "zero"))
    assert name == "float_M7N7_b2_v4p4f1nt2mx+embedded" and g["halo_lanes"] == 2   # the matrix-core instance is the 7x7 default
    name, _ = parse(ssam.ssam_describe("conv2d", (100, 100), np.ones((1, 6), dtype=np.float32), "zero"))
    assert name.startswith("float_M6N6_b2") and name.endswith("+embedded")
    # ... one-dimensional filters of odd length have instances of their own ...
    name, g = parse(ssam.ssam_describe("conv2d", (100, 100), np.ones((7, 1), dtype=np.float32), "zero"))
    assert name.startswith("float_M1N7_b2") and g["halo_lanes"] == 0
    # ... and what no box holds (wider than 20, or embedding switched off) falls to the direct kernel
    name, _ = parse(ssam.ssam_describe("conv2d", (100, 100), np.ones((4, 23), dtype=np.float32), "zero"))
    assert name == "generic_direct"
    ssam.ssam_set_tuning("embed_waste", 0)
    try:
        name, _ = parse(ssam.ssam_describe("conv2d", (100, 100), np.ones((4, 7), dtype=np.float32), "zero"))
        assert name == "generic_direct"
    finally:
        ssam.ssam_set_tuning("embed_waste", -1)
    # every shape up to the advertised limits is accepted: the direct kernel takes a tap list of any
    # length (several launches), so neither a dense 17^3 box nor a 32x32 filter is refused
    for box in (np.ones((9, 9, 9), dtype=np.float64), np.ones((17, 17, 17), dtype=np.float64), np.ones((17, 17, 17), dtype=np.float32)):
        name, _ = parse(ssam.ssam_describe("stencil3d", (32, 32, 32), box, "zero"))
        assert name == "generic_direct"
    star = np.zeros((17, 17, 17)); star[8, 8, :] = 1; star[8, :, 8] = 1; star[:, 8, 8] = 1
    name, _ = parse(ssam.ssam_describe("stencil3d", (32, 32, 32), star, "zero"))
    assert name == "generic_direct"
    for dt in (np.float32, np.float64):
        for shape in ((32, 32), (30, 30), (22, 22), (32, 1), (1, 32)):
            name, _ = parse(ssam.ssam_describe("conv2d", (100, 100), np.ones(shape, dtype=dt), "clamp"))
            assert name == "generic_direct" or name.endswith("+embedded") or "_M" in name, name


def test_extreme_extents_plan_or_refuse(L):
    """Extents near the limits: the planner's arithmetic must not wrap.  Every extent up to
    SSAM_MAX_EXTENT (2^30) with W*H*D <= 2^31-1 either gets a plan with positive counts that
    covers the grid, or SSAM_ERR_DIM; anything above is SSAM_ERR_DIM."""
    big = 1 << 30
    f = np.ones((3, 3), dtype=np.float32)
    for W, H in ((1, big), (big, 1), (2, big - 1), (big - 1, 2), (3, 715827882)):
        name, g = parse(ssam.ssam_describe("conv2d", (H, W), f, "clamp"))
        assert g["valid_lanes"] > 0 and g["strips_x"] > 0 and g["tiles_y"] > 0 and g["blocks"] > 0, (W, H, g)
        assert g["strips_x"] * g["valid_lanes"] * g["V"] >= W and g["tiles_y"] * g["rows_per_wave"] >= H
        assert g["tiles"] == g["strips_x"] * g["tiles_y"] and g["blocks"] * 4 >= g["tiles"] and g["blocks"] < (1 << 22)
    buf = ctypes.create_string_buffer(512)
    for W, H, D in ((2147483647, 1, 1), (1, 2147483647, 1), (1, 1, 2147483647), (big + 1, 1, 1)):
        c3 = np.ones(27, dtype=np.float64)
        assert L.ssam_describe(2, W, H, D, c3.ctypes.data, 1, 1, 1, 0, 1, buf, 512) == 2, (W, H, D)
        if D == 1:   # (with D > 1 the 2D call would see a valid 1x1 grid and launch on these made-up pointers)
            assert L.ssam_conv2d(FAKE_A, FAKE_B, W, H, f.ctypes.data, 3, 3, -1, -1, 1, 0, None) == 2
    # 3D plans of extreme aspect ratio: a plan with positive counts, or SSAM_ERR_DIM -- never a wrapped one
    c3 = np.ones((3, 3, 3), dtype=np.float64)
    for shape in ((2, big, 1), (big, 1, 2), (1, 2, big), (2, 1, big)):
        try:
            name, g = parse(ssam.ssam_describe("stencil3d", shape, c3, "zero"))
        except ssam.SsamError as e:
            assert e.status == 2
            continue
        assert g["blocks"] > 0 and g["tiles"] > 0 and g["strips_x"] > 0 and g["tiles_y"] > 0 and g["tiles_z"] > 0, (shape, g)


def test_fused_sweep_plan(L):
    """2D sweeps with zero padding run several to a launch; the overlap grows with the depth S on
    every side (S*r incomplete columns); shapes without a fused instance keep
    single sweeps; the planner never runs more sweeps than remain."""
    import re
    for c in wl.config3():
        coef = c.coef[0]
        r = coef.shape[0] // 2
        one, g1 = parse(ssam.ssam_describe("stencil2d", c.shape, coef, "zero"))
        assert "_fused" not in one
        for remaining in (0, 2, 3, 4):
            many, g = parse(ssam.ssam_describe("iterate2d", c.shape, coef, "zero", remaining=remaining))
            S = int(re.search(r"_fused(\d+)$", many).group(1))
            assert 2 <= S and (remaining == 0 or S <= remaining)
            assert g["halo_lanes"] == 2 * -(-S * r // g["V"])   # S*r incomplete columns per side
            assert g["valid_lanes"] <= 64 - g["halo_lanes"]
            assert g["strips_x"] * g["valid_lanes"] * g["V"] >= c.shape[1]
            assert g["rows_per_wave"] % g["P"] == 0
        assert parse(ssam.ssam_describe("iterate2d", c.shape, coef, "zero", remaining=1))[0] == one
        assert parse(ssam.ssam_describe("iterate2d", c.shape, coef, "clamp"))[0] == \
            parse(ssam.ssam_describe("iterate2d", c.shape, coef, "zero"))[0]   # both boundary rules fuse in 2D
    coef = wl.config3()[0].coef[0]
    for cap, ok in ((0, lambda n: "_fused" not in n), (1, lambda n: "_fused" not in n), (2, lambda n: n.endswith("_fused2"))):
        ssam.ssam_set_tuning("fuse_sweeps", cap)
        try:
            assert ok(parse(ssam.ssam_describe("iterate2d", (512, 512), coef, "zero"))[0])
        finally:
            ssam.ssam_set_tuning("fuse_sweeps", -1)
    wide = np.ones((15, 15))   # radius 7: no fused instance
    assert parse(ssam.ssam_describe("iterate2d", (512, 512), wide, "zero"))[0] == "generic_direct"


def test_block_cooperative_3d_plans(L):
    """The block-cooperative 3D kernels: every lane stores, one block per compute unit on 512^3, and z-chunks that
    would start a multiple of 128 MiB apart are made four planes longer (the last one shorter)."""
    for dtype, r, planes in ((np.float64, 1, 132), (np.float64, 4, 260), (np.float32, 1, 64), (np.float32, 4, 132)):
        coef = wl.seeded_coefficients(wl.mask_star(r, r, r), 1, dtype)
        name, g = parse(ssam.ssam_describe("stencil3d", (512, 512, 512), coef, "zero"))
        assert "star_ring" in name and g["halo_lanes"] == 0 and g["valid_lanes"] == 64
        assert g["planes_per_wave"] == planes and g["tiles"] == 256
        assert g["tiles_z"] == -(-512 // planes)
    # a chunk spacing that is no multiple of 128 MiB stays as it is
    coef = wl.seeded_coefficients(wl.mask_star(1, 1, 1), 1, np.float64)
    assert parse(ssam.ssam_describe("stencil3d", (256, 256, 256), coef, "zero"))[1]["planes_per_wave"] == 16


def test_fp64_arithmetic_bound_filters_take_short_balanced_tiles(L):
    for r in (4, 5):
        coef = wl.seeded_coefficients(wl.mask_box(r, r), 1, np.float64)
        coef = coef[0] if coef.ndim == 3 else coef
        name, g = parse(ssam.ssam_describe("stencil2d", (8192, 8192), coef, "zero"))
        assert name.startswith("double_M") and g["rows_per_wave"] <= 64
    # the fp32 ones keep the tallest balanced tiles
    name, g = parse(ssam.ssam_describe("conv2d", (8192, 8192), np.ones((20, 20), np.float32), "clamp"))
    assert name.endswith("mx") and g["rows_per_wave"] >= 64


def test_fused_sweep_plan_3d(L):
    """Radius-1 3D stencils with zero padding run two sweeps per launch when marching along z (one wave per
    tile: two incomplete columns per side; the 7-point star: block-cooperative, no incomplete lanes); radius 4
    and the y march keep single sweeps."""
    for c in wl.config4():
        one, g1 = parse(ssam.ssam_describe("stencil3d", c.shape, c.coef, "zero"))
        two, g2 = parse(ssam.ssam_describe("iterate3d", c.shape, c.coef, "zero"))
        assert two.endswith("_fused2") and "_fused" not in one
        if "star" in c.name:   # block-cooperative: every lane stores, the widening columns are recomputed per lane
            assert g2["halo_lanes"] == 0 and g2["valid_lanes"] == 64 and "star_ring" in two
        else:
            assert g2["halo_lanes"] == 2 * -(-2 * 1 // g2["V"]) and g2["valid_lanes"] <= 64 - g2["halo_lanes"]
        assert g2["tiles"] == g2["strips_x"] * g2["tiles_y"] * g2["tiles_z"]
        # under the clamp rule only the 7-point star fuses (the others spill registers and lose)
        assert parse(ssam.ssam_describe("iterate3d", c.shape, c.coef, "clamp"))[0] == (two if "star" in c.name else one)
        ssam.ssam_set_tuning("march_axis", 1)
        try:
            assert "_fused" not in ssam.ssam_describe("iterate3d", c.shape, c.coef, "zero")
        finally:
            ssam.ssam_set_tuning("march_axis", -1)
    for c in wl.config5():
        assert "_fused" not in ssam.ssam_describe("iterate3d", c.shape, c.coef, "zero")
