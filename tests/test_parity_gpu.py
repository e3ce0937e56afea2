"""GPU parity: the HIP path, called through the C ABI (ctypes binding), against the CPU oracle,
element by element on the same seeded inputs.  Sizes here are small enough for the oracle to
finish in seconds yet span several wave tiles, ragged tails and the unaligned slow path.
Tolerance (stated by the acceptance target): max |gpu - oracle| / (sum|w| * max|in|) <= 1e-5
for fp32, <= 1e-12 for fp64."""
import numpy as np
import pytest

import oracle
import workloads as wl
from parity_util import assert_parity

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def ssam():
    import paper_1907_06154_amd as s
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    s.lib()   # raises if the HIP library is missing: there is no fallback
    yield s
    for name in ("rows_per_wave", "valid_lanes", "planes_per_wave", "xcd_remap", "force_generic", "variant", "march_axis",
                 "fuse_sweeps", "embed_waste"):
        s.ssam_set_tuning(name, -1)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


SHAPES_2D = [(70, 300), (37, 259), (5, 7), (1, 1), (64, 1024), (129, 520), (3, 2050)]


@pytest.mark.parametrize("MN", sorted(set(wl.CONV_SHAPES + [(m, m) for m in range(2, 21)] + [(4, 6), (1, 5), (5, 1), (21, 21)])))
@pytest.mark.parametrize("boundary", ["clamp", "zero"])
def test_conv2d_f32(ssam, MN, boundary):
    M, N = MN
    filt = wl.seeded_filter(M, N, 300 + 32 * M + N, np.float32)
    for k, (H, W) in enumerate(SHAPES_2D):
        img = wl.uniform_field((H, W), 0.0, 1.0, 310 + k, np.float32)
        print(f"conv2d f32 {M}x{N} {boundary} grid {H}x{W}", flush=True)
        got = host(ssam.ssam_conv2d(dev(img), filt, boundary))
        want = oracle.conv2d(img, filt, boundary)
        assert_parity(got, want, filt, 1.0, f"conv {M}x{N} {boundary} {H}x{W}")


@pytest.mark.parametrize("m", [7, 8, 9, 12, 14, 15, 17, 20])
def test_matrix_core_and_vector_unit_instances_agree_with_the_oracle(ssam, m):
    """Dense fp32 filters from 7x7 on run on the matrix cores by default and on the vector unit as
    variant 5: both against the oracle, on grids with ragged strips and short tiles."""
    filt = wl.seeded_filter(m, m, 700 + m, np.float32)
    for k, (H, W) in enumerate([(131, 517), (64, 1024), (9, 260)]):
        img = wl.uniform_field((H, W), -1.0, 1.0, 720 + k, np.float32)
        for boundary in ("clamp", "zero"):
            want = oracle.conv2d(img, filt, boundary)
            for variant in (-1, 5):
                ssam.ssam_set_tuning("variant", variant)
                name = ssam.ssam_describe("conv2d", (H, W), filt, boundary).split()[0]
                assert name.endswith("mx") == (variant == -1), name
                print(f"conv {m}x{m} {boundary} {H}x{W} {name}", flush=True)
                got = host(ssam.ssam_conv2d(dev(img), filt, boundary))
                assert_parity(got, want, filt, 1.0, f"{name} {boundary} {H}x{W}")
    ssam.ssam_set_tuning("variant", -1)


@pytest.mark.parametrize("MN", [(5, 7), (7, 5), (1, 4), (4, 1), (1, 15), (15, 1), (1, 20), (20, 1), (2, 16), (7, 13), (13, 1)])
def test_odd_filter_shapes_and_anchors_f32(ssam, MN):
    """Filters without an instance of their own shape -- non-square, one-dimensional, anchored off the
    centre -- run embedded in a compiled square box (or on a 1D instance); same tolerance."""
    M, N = MN
    filt = wl.seeded_filter(M, N, 500 + 32 * M + N, np.float32)
    anchors = [None, (0, 0), (M - 1, N - 1), (M // 3, (2 * N) // 3)]
    for k, (H, W) in enumerate([(70, 300), (37, 259), (3, 2050), (1, 1000), (1000, 1)]):
        img = wl.uniform_field((H, W), 0.0, 1.0, 510 + k, np.float32)
        for anchor in anchors:
            for boundary in ("clamp", "zero"):
                print(f"odd filter {M}x{N} anchor {anchor} {boundary} grid {H}x{W}", flush=True)
                got = host(ssam.ssam_conv2d(dev(img), filt, boundary, anchor))
                assert_parity(got, oracle.conv2d(img, filt, boundary, anchor), filt, 1.0, f"odd {M}x{N} {anchor} {boundary}")
    name = ssam.ssam_describe("conv2d", (70, 300), filt, "clamp").split()[0]
    assert name != "generic_direct"


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_anisotropic_stencils_are_embedded(ssam, dtype):
    for rx, ry in ((3, 1), (1, 2), (0, 2), (4, 0)):
        coef = wl.seeded_coefficients(wl.mask_box(rx, ry), 520 + rx, dtype)[0]
        fld = wl.uniform_field((70, 300), -1.0, 1.0, 521, dtype)
        assert ssam.ssam_describe("stencil2d", (70, 300), coef, "zero").split()[0] != "generic_direct"
        for boundary in ("clamp", "zero"):
            print(f"anisotropic {np.dtype(dtype).name} rx{rx} ry{ry} {boundary}", flush=True)
            got = host(ssam.ssam_stencil2d(dev(fld), coef, boundary))
            assert_parity(got, oracle.stencil(fld, coef, boundary), coef, 1.0, f"aniso {rx} {ry} {boundary}")
        res = ssam.ssam_stencil_iterate(dev(fld), torch.empty_like(dev(fld)), coef, 3, "zero")
        assert_parity(host(res), oracle.iterate(fld, coef, 3, "zero"), coef, 1.0, f"aniso iterate {rx} {ry}")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_3d_shapes_without_instance_are_embedded(ssam, dtype):
    """Unequal radii and radii between the compiled ones run zero-padded inside a compiled star or box."""
    masks = [wl.mask_box(2, 1, 1), wl.mask_star(4, 2, 2), wl.mask_star(3, 3, 3), wl.mask_box(1, 1, 0), wl.mask_star(1, 0, 2)]
    fld = wl.uniform_field((23, 30, 150), -1.0, 1.0, 531, dtype)
    for k, mask in enumerate(masks):
        coef = wl.seeded_coefficients(mask, 532 + k, dtype)
        name = ssam.ssam_describe("stencil3d", fld.shape, coef, "zero").split()[0]
        assert name.endswith("+embedded"), name
        for boundary in ("clamp", "zero"):
            print(f"embedded 3d {np.dtype(dtype).name} {coef.shape} {boundary} {name}", flush=True)
            got = host(ssam.ssam_stencil3d(dev(fld), coef, boundary))
            assert_parity(got, oracle.stencil(fld, coef, boundary), coef, 1.0, f"embedded3d {coef.shape} {boundary}")
        res = ssam.ssam_stencil_iterate(dev(fld), torch.empty_like(dev(fld)), coef, 3, "zero")
        assert_parity(host(res), oracle.iterate(fld, coef, 3, "zero"), coef, 1.0, f"embedded3d iterate {coef.shape}")


@pytest.mark.parametrize("MN", [(3, 3), (5, 5), (9, 9), (4, 3)])
def test_conv2d_f64_and_anchors(ssam, MN):
    M, N = MN
    filt = wl.seeded_filter(M, N, 400 + 32 * M + N, np.float64)
    img = wl.uniform_field((70, 300), -1.0, 1.0, 401, np.float64)
    for anchor in (None, (0, 0), (M - 1, N - 1)):
        for boundary in ("clamp", "zero"):
            print(f"conv2d f64 {M}x{N} anchor {anchor} {boundary}", flush=True)
            got = host(ssam.ssam_conv2d(dev(img), filt, boundary, anchor))
            want = oracle.conv2d(img, filt, boundary, anchor)
            assert_parity(got, want, filt, 1.0, f"conv f64 {M}x{N} {anchor} {boundary}")


STENCILS_2D = [("star", 1), ("star", 2), ("star", 3), ("star", 4), ("star", 5), ("star", 6), ("star", 7),
               ("box", 1), ("box", 2), ("box", 3), ("box", 4), ("box", 5), ("star_wide", 0), ("sparse", 2)]


def stencil2d_coef(kind, r, dtype, seed):
    if kind == "star":
        mask = wl.mask_star(r, r)
    elif kind == "box":
        mask = wl.mask_box(r, r)
    elif kind == "star_wide":           # different radii per axis: no compiled instance
        mask = wl.mask_star(5, 2)
    else:                               # arbitrary zero pattern inside a box
        mask = wl.mask_box(r, r)
        mask[0, 0, 1] = mask[0, 2, 3] = mask[0, 4, 4] = False
    return wl.seeded_coefficients(mask, seed, dtype, -1.0, 1.0, normalise=False)[0]


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("kind,r", STENCILS_2D)
@pytest.mark.parametrize("boundary", ["zero", "clamp"])
def test_stencil2d(ssam, dtype, kind, r, boundary):
    coef = stencil2d_coef(kind, r, dtype, 500 + r)
    for k, (H, W) in enumerate(SHAPES_2D):
        fld = wl.uniform_field((H, W), -1.0, 1.0, 510 + k, dtype)
        print(f"stencil2d {np.dtype(dtype).name} {kind} r{r} {boundary} grid {H}x{W}", flush=True)
        got = host(ssam.ssam_stencil2d(dev(fld), coef, boundary))
        want = oracle.stencil(fld, coef, boundary)
        assert_parity(got, want, coef, 1.0, f"stencil2d {kind} r{r} {boundary} {H}x{W}")


SHAPES_3D = [(9, 10, 130), (70, 6, 30), (3, 3, 3), (1, 5, 5), (20, 13, 259), (12, 11, 140), (6, 5, 516)]
STENCILS_3D = [("star", 1), ("box", 1), ("faces_edges", 1), ("star", 4), ("star", 2), ("box", 2), ("star", 3),
               ("box_aniso", 0)]


def stencil3d_coef(kind, r, dtype, seed):
    if kind == "star":
        mask = wl.mask_star(r, r, r)
    elif kind == "box":
        mask = wl.mask_box(r, r, r)
    elif kind == "faces_edges":
        mask = wl.mask_faces_edges()
    else:
        mask = wl.mask_box(2, 1, 1)     # no compiled instance: direct kernel
    return wl.seeded_coefficients(mask, seed, dtype, -1.0, 1.0, normalise=False)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("kind,r", STENCILS_3D)
@pytest.mark.parametrize("boundary", ["zero", "clamp"])
def test_stencil3d(ssam, dtype, kind, r, boundary):
    coef = stencil3d_coef(kind, r, dtype, 600 + r)
    for k, shape in enumerate(SHAPES_3D):
        fld = wl.uniform_field(shape, -1.0, 1.0, 610 + k, dtype)
        print(f"stencil3d {np.dtype(dtype).name} {kind} r{r} {boundary} grid {shape}", flush=True)
        got = host(ssam.ssam_stencil3d(dev(fld), coef, boundary))
        want = oracle.stencil(fld, coef, boundary)
        assert_parity(got, want, coef, 1.0, f"stencil3d {kind} r{r} {boundary} {shape}")


@pytest.mark.parametrize("tuning", [
    {"rows_per_wave": 8}, {"valid_lanes": 17}, {"xcd_remap": 0}, {"planes_per_wave": 5},
    {"rows_per_wave": 16, "valid_lanes": 40, "planes_per_wave": 3, "xcd_remap": 0}, {"force_generic": 1},
    {"variant": 1}, {"variant": 2}, {"variant": 4}, {"variant": 5}, {"variant": 10},
    {"variant": 4, "planes_per_wave": 5, "valid_lanes": 24}, {"variant": 2, "planes_per_wave": 2, "xcd_remap": 0},
    {"march_axis": 1}, {"march_axis": 1, "variant": 1}, {"march_axis": 1, "variant": 4, "planes_per_wave": 6},
    {"march_axis": 1, "variant": 2},
])
def test_tile_geometry_overrides_do_not_change_results(ssam, tuning):
    try:
        for k, v in tuning.items():
            ssam.ssam_set_tuning(k, v)
        print(f"tuning {tuning}", flush=True)
        img = wl.uniform_field((129, 520), 0.0, 1.0, 701, np.float32)
        filt = wl.seeded_filter(5, 5, 702, np.float32)
        assert_parity(host(ssam.ssam_conv2d(dev(img), filt, "clamp")), oracle.conv2d(img, filt, "clamp"), filt, 1.0)
        fld = wl.uniform_field((70, 300), -1.0, 1.0, 703, np.float64)
        c2 = stencil2d_coef("star", 4, np.float64, 704)
        assert_parity(host(ssam.ssam_stencil2d(dev(fld), c2, "zero")), oracle.stencil(fld, c2, "zero"), c2, 1.0)
        for dt in (np.float64, np.float32):
            for shape in ((20, 13, 259), (9, 37, 260)):
                f3 = wl.uniform_field(shape, -1.0, 1.0, 705, dt)
                for kind, r in (("box", 1), ("star", 1), ("star", 4)):
                    c3 = stencil3d_coef(kind, r, dt, 706)
                    for bnd in ("clamp", "zero"):
                        assert_parity(host(ssam.ssam_stencil3d(dev(f3), c3, bnd)), oracle.stencil(f3, c3, bnd), c3, 1.0,
                                      f"{tuning} {kind} r{r} {bnd} {shape}")
    finally:
        for k in tuning:
            ssam.ssam_set_tuning(k, -1)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_table3_2d64pt(ssam, dtype):
    """The one Table 3 shape no radius describes, an 8x8 box: a dense 8x8 filter with the default anchor
    (4, 4), on an instance of its own in both precisions."""
    case = next(c for c in wl.table3(dtypes=(dtype,)) if "2d64pt" in c.name)
    assert case.coef.shape == (8, 8) and abs(float(case.coef.sum()) - 1.0) < 1e-5
    for k, (H, W) in enumerate(SHAPES_2D):
        img = wl.uniform_field((H, W), -1.0, 1.0, 690 + k, dtype)
        name = ssam.ssam_describe("conv2d", img.shape, case.coef, case.boundary).split()[0]
        assert "_M8N8_" in name and "embedded" not in name, name
        for bnd in ("zero", "clamp"):
            print(f"2d64pt {np.dtype(dtype).name} {bnd} grid {H}x{W} {name}", flush=True)
            got = host(ssam.ssam_conv2d(dev(img), case.coef, bnd))
            assert_parity(got, oracle.conv2d(img, case.coef, bnd), case.coef, 1.0, f"2d64pt {bnd} {H}x{W}")


CONV3D_CASES = [((3, 3, 3), None), ((5, 5, 5), None), ((7, 7, 7), None), ((2, 2, 2), None), ((4, 3, 2), None),
                ((3, 3, 3), (0, 0, 0)), ((4, 4, 4), (3, 1, 2)), ((5, 2, 3), (4, 0, 1)), ((1, 1, 6), None), ((9, 9, 9), None),
                ((17, 2, 1), (16, 1, 0)), ((6, 6, 6), None)]


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("boundary", ["clamp", "zero"])
def test_conv3d(ssam, dtype, boundary):
    """3D filters of odd and even extents, centred and off-centre anchors: the cubes that are compiled
    instances, those embedded in one, and those left to the direct kernel; rows that are and are not a
    multiple of 16 bytes."""
    for k, ((M, N, K), anchor) in enumerate(CONV3D_CASES):
        filt = wl.uniform_field((K, N, M), -1.0, 1.0, 660 + k, dtype)
        for shape in ((19, 23, 132), (9, 10, 67), (3, 2, 4)):
            vol = wl.uniform_field(shape, 0.0, 1.0, 670 + k, dtype)
            name = ssam.ssam_describe("conv3d", shape, filt, boundary).split()[0]
            print(f"conv3d {np.dtype(dtype).name} {M}x{N}x{K} anchor {anchor} {boundary} grid {shape} {name}", flush=True)
            got = host(ssam.ssam_conv3d(dev(vol), filt, boundary, anchor))
            want = oracle.conv3d(vol, filt, boundary, anchor)
            assert_parity(got, want, filt, 1.0, f"conv3d {M}x{N}x{K} {anchor} {boundary} {shape}")
    # a zero in the filter is a tap like any other: same result as the stencil with that box (finite inputs)
    box = wl.seeded_coefficients(wl.mask_star(1, 1, 1), 680, dtype)
    vol = wl.uniform_field((12, 20, 136), -1.0, 1.0, 681, dtype)
    assert_parity(host(ssam.ssam_conv3d(dev(vol), box, boundary)), oracle.conv3d(vol, box, boundary), box, 1.0, "zeros are taps")
    assert ssam.ssam_describe("conv3d", vol.shape, box, boundary).split()[0].startswith(("float_r111_b3", "double_r111_b3"))


STAR_SHAPES = [(33, 70, 260), (75, 9, 512), (10, 40, 4), (5, 3, 8), (13, 37, 132), (21, 66, 1028)]


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("kind,r", [("star", 1), ("star", 2), ("star", 4), ("box", 1), ("faces_edges", 1)])
@pytest.mark.parametrize("tuning", [{}, {"variant": 10}, {"planes_per_wave": 5}, {"planes_per_wave": 8, "xcd_remap": 0},
                                    {"march_axis": 1}, {"planes_per_wave": 1}, {"planes_per_wave": 2, "variant": 10},
                                    {"march_axis": 1, "variant": 10, "planes_per_wave": 9}])
def test_block_cooperative_star_kernel(ssam, dtype, kind, r, tuning):
    """3D stencils on the block-cooperative kernel without halo lanes (rows that are a multiple of 16
    bytes): stars, the 19-point and the 27-point shape; both compiled tile shapes, short z-chunks, both
    march axes, both boundary rules, on grids with partial strips, partial blocks in y, fewer planes than
    the radius and several strips."""
    coef = wl.seeded_symmetric_star(r, 3, 640, dtype) if kind == "star" else stencil3d_coef(kind, r, dtype, 640)
    try:
        for k, v in tuning.items():
            ssam.ssam_set_tuning(k, v)
        for k, shape in enumerate(STAR_SHAPES):
            fld = wl.uniform_field(shape, -1.0, 1.0, 641 + k, dtype)
            name = ssam.ssam_describe("stencil3d", shape, coef, "zero").split()[0]
            assert "star_ring" in name, (name, tuning)
            for bnd in ("zero", "clamp"):
                print(f"star kernel {np.dtype(dtype).name} r{r} {tuning} {bnd} grid {shape} {name}", flush=True)
                got = host(ssam.ssam_stencil3d(dev(fld), coef, bnd))
                assert_parity(got, oracle.stencil(fld, coef, bnd), coef, 1.0, f"r{r} {tuning} {bnd} {shape}")
        # unsymmetric coefficients: every tap multiplies its own neighbour
        c2 = stencil3d_coef(kind, r, dtype, 650)
        fld = wl.uniform_field((19, 41, 264), -1.0, 1.0, 651, dtype)
        for bnd in ("zero", "clamp"):
            got = host(ssam.ssam_stencil3d(dev(fld), c2, bnd))
            assert_parity(got, oracle.stencil(fld, c2, bnd), c2, 1.0, f"r{r} {tuning} {bnd} unsymmetric")
        # rows that are not a multiple of 16 bytes take the fallback instance
        odd = wl.uniform_field((9, 12, 131), -1.0, 1.0, 652, dtype)
        assert "halo_lanes=0+0" not in ssam.ssam_describe("stencil3d", odd.shape, coef, "zero")   # a tile plan with halo lanes
        got = host(ssam.ssam_stencil3d(dev(odd), coef, "zero"))
        assert_parity(got, oracle.stencil(odd, coef, "zero"), coef, 1.0, f"r{r} {tuning} fallback")
    finally:
        for k in tuning:
            ssam.ssam_set_tuning(k, -1)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_iterate_matches_oracle_and_ping_pongs(ssam, dtype):
    cases = [((70, 300), wl.seeded_coefficients(wl.mask_box(2, 2), 801, dtype)[0]),
             ((70, 300), wl.seeded_coefficients(wl.mask_star(4, 4), 802, dtype)[0]),
             ((20, 13, 140), wl.seeded_coefficients(wl.mask_star(1, 1, 1), 803, dtype)),
             ((20, 13, 140), wl.seeded_symmetric_star(4, 3, 804, dtype))]
    for shape, coef in cases:
        fld = wl.uniform_field(shape, -1.0, 1.0, 810, dtype)
        for steps in (0, 1, 2, 7):
            print(f"iterate {np.dtype(dtype).name} {shape} steps {steps}", flush=True)
            a, b = dev(fld), torch.full(shape, float("nan"), dtype=torch.from_numpy(fld).dtype, device="cuda")
            res = ssam.ssam_stencil_iterate(a, b, coef, steps, "zero")
            assert res.data_ptr() in (a.data_ptr(), b.data_ptr()) and (steps or res.data_ptr() == a.data_ptr())
            want = oracle.iterate(fld, coef, steps, "zero")
            if steps == 0:
                assert np.array_equal(host(res), fld)
            else:
                assert_parity(host(res), want, coef, 1.0, f"iterate {shape} {steps}")


FUSED_SHAPES = [(1, 1), (3, 5), (9, 130), (33, 224), (70, 300), (131, 449), (150, 1000), (260, 96)]


def planned_launches(ssam, shape, coef, steps, boundary):
    """Launches ssam_stencil_iterate issues for `steps` 2D sweeps, from the planning query."""
    import re
    t = n = 0
    while t < steps:
        name = ssam.ssam_describe("iterate2d", shape, coef, boundary, remaining=steps - t).split()[0]
        m = re.search(r"_fused(\d+)$", name)
        t += int(m.group(1)) if m else 1
        n += 1
    assert t == steps
    return n


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("kind,r", [("box", 1), ("star", 1), ("box", 2), ("star", 2), ("star", 3), ("star", 4), ("star", 5), ("star", 6)])
def test_fused_sweeps_match_oracle(ssam, dtype, kind, r):
    """Several 2D sweeps run as one launch (zero padding): every step count and fusion depth, grids
    smaller than a tile, ragged tails, rows that are not vector-aligned; and fusion switched off."""
    mask = wl.mask_box(r, r) if kind == "box" else wl.mask_star(r, r)
    coef = wl.seeded_coefficients(mask, 820 + r, dtype)[0]
    assert "_fused" in ssam.ssam_describe("iterate2d", (4096, 4096), coef, "zero")
    assert "_fused" in ssam.ssam_describe("iterate2d", (4096, 4096), coef, "clamp")
    for shape in FUSED_SHAPES:
        fld = wl.uniform_field(shape, -1.0, 1.0, 830 + shape[0], dtype)
        for boundary in ("zero", "clamp"):
            for steps in (2, 3, 4, 5, 6, 7, 9):
                want = oracle.iterate(fld, coef, steps, boundary)
                for fuse in (-1, 0, 2, 3):
                    print(f"fused {np.dtype(dtype).name} {kind} r{r} {shape} {boundary} steps {steps} fuse {fuse}", flush=True)
                    ssam.ssam_set_tuning("fuse_sweeps", fuse)
                    try:
                        launches = planned_launches(ssam, shape, coef, steps, boundary)
                        a, b = dev(fld), torch.full(shape, float("nan"), dtype=torch.from_numpy(fld).dtype, device="cuda")
                        res = ssam.ssam_stencil_iterate(a, b, coef, steps, boundary)
                    finally:
                        ssam.ssam_set_tuning("fuse_sweeps", -1)
                    # (grids this small run a remaining pair of sweeps as two launches unless a cap asks for pairs)
                    assert launches == steps if fuse == 0 else launches <= steps
                    if fuse != 0 and (fuse in (2, 3) or (steps >= 3 and r <= 4)):
                        assert launches < steps
                    assert res.data_ptr() == (a if launches % 2 == 0 else b).data_ptr()
                    assert_parity(host(res), want, coef, 1.0, f"fused {kind} r{r} {shape} {boundary} steps {steps} fuse {fuse}")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_fused_sweeps_tile_overrides_and_clamp(ssam, dtype):
    coef = wl.seeded_coefficients(wl.mask_box(2, 2), 841, dtype)[0]
    fld = wl.uniform_field((300, 1200), -1.0, 1.0, 842, dtype)
    want = oracle.iterate(fld, coef, 4, "zero")
    for tuning in ({"rows_per_wave": 8}, {"rows_per_wave": 40, "valid_lanes": 17}, {"xcd_remap": 0}, {"variant": 1},
                   {"fuse_sweeps": 2, "variant": 1}, {"fuse_sweeps": 3, "rows_per_wave": 4}):
        print(f"fused overrides {np.dtype(dtype).name} {tuning}", flush=True)
        for k, v in tuning.items():
            ssam.ssam_set_tuning(k, v)
        try:
            a = dev(fld)
            res = ssam.ssam_stencil_iterate(a, torch.empty_like(a), coef, 4, "zero")
            assert_parity(host(res), want, coef, 1.0, f"fused {tuning}")
        finally:
            for k in tuning:
                ssam.ssam_set_tuning(k, -1)
    want = oracle.iterate(fld, coef, 4, "clamp")
    for tuning in ({}, {"rows_per_wave": 8}, {"rows_per_wave": 40, "valid_lanes": 17}, {"fuse_sweeps": 2, "variant": 1}):
        for k, v in tuning.items():
            ssam.ssam_set_tuning(k, v)
        try:
            a = dev(fld)
            res = ssam.ssam_stencil_iterate(a, torch.empty_like(a), coef, 4, "clamp")
            assert_parity(host(res), want, coef, 1.0, f"fused clamp {tuning}")
        finally:
            for k in tuning:
                ssam.ssam_set_tuning(k, -1)


FUSED_SHAPES_3D = [(1, 1, 1), (3, 5, 7), (1, 1, 4), (2, 3, 8), (9, 33, 130), (20, 13, 140), (70, 10, 224), (17, 40, 300), (5, 70, 520)]


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("kind", ["star", "faces_edges", "box"])
def test_fused_sweeps_3d_match_oracle(ssam, dtype, kind):
    """Radius-1 3D stencils run two sweeps per launch (zero padding, march along z): odd and even step
    counts, grids smaller than a tile, ragged tails, unaligned rows, every compiled variant."""
    mask = {"star": wl.mask_star(1, 1, 1), "box": wl.mask_box(1, 1, 1), "faces_edges": wl.mask_faces_edges()}[kind]
    coef = wl.seeded_coefficients(mask, 850, dtype)
    # no two-sweep instance where it measured no faster than single sweeps: in fp32 only the 7-point star has one
    has_fused = kind == "star" or dtype == np.float64
    assert ssam.ssam_describe("iterate3d", (512, 512, 512), coef, "zero").split()[0].endswith("_fused2") == has_fused
    # ... and under the clamp rule only the 7-point star has one
    assert ssam.ssam_describe("iterate3d", (512, 512, 512), coef, "clamp").split()[0].endswith("_fused2") == (kind == "star")
    assert "_fused" not in ssam.ssam_describe("iterate3d", (64, 64, 64), coef, "zero")   # too small to pay
    for shape in FUSED_SHAPES_3D:
        fld = wl.uniform_field(shape, -1.0, 1.0, 860 + shape[0], dtype)
        for boundary in ("zero", "clamp"):
            for steps in (2, 3, 4, 5):
                want = oracle.iterate(fld, coef, steps, boundary)
                # fuse_sweeps = 2 asks for pairs whatever the grid size; the default leaves grids this small unfused
                for tuning in ({"fuse_sweeps": 2}, {}, {"fuse_sweeps": 0}, {"fuse_sweeps": 2, "variant": 1},
                               {"fuse_sweeps": 2, "planes_per_wave": 3}, {"fuse_sweeps": 2, "planes_per_wave": 1},
                               {"fuse_sweeps": 2, "valid_lanes": 9, "planes_per_wave": 5}, {"fuse_sweeps": 2, "march_axis": 1}):
                    print(f"fused3d {np.dtype(dtype).name} {kind} {shape} {boundary} steps {steps} {tuning}", flush=True)
                    for k, v in tuning.items():
                        ssam.ssam_set_tuning(k, v)
                    try:
                        fused = "_fused2" in ssam.ssam_describe("iterate3d", shape, coef, boundary)
                        a_, b_ = dev(fld), torch.full(shape, float("nan"), dtype=torch.from_numpy(fld).dtype, device="cuda")
                        res = ssam.ssam_stencil_iterate(a_, b_, coef, steps, boundary)
                    finally:
                        for k in tuning:
                            ssam.ssam_set_tuning(k, -1)
                    assert fused == (has_fused and (boundary == "zero" or kind == "star") and
                                     tuning.get("fuse_sweeps") == 2 and tuning.get("march_axis") != 1)
                    launches = steps // 2 + steps % 2 if fused else steps
                    assert res.data_ptr() == (a_ if launches % 2 == 0 else b_).data_ptr()
                    assert_parity(host(res), want, coef, 1.0, f"fused3d {kind} {shape} {boundary} steps {steps} {tuning}")


def test_results_are_bitwise_reproducible(ssam):
    img = dev(wl.uniform_field((257, 1031), 0.0, 1.0, 901, np.float32))
    filt = wl.seeded_filter(9, 9, 902, np.float32)
    first = host(ssam.ssam_conv2d(img, filt, "clamp"))
    for _ in range(3):
        assert np.array_equal(host(ssam.ssam_conv2d(img, filt, "clamp")), first)
    f3 = dev(wl.uniform_field((40, 21, 300), -1.0, 1.0, 903, np.float64))
    c3 = stencil3d_coef("star", 4, np.float64, 904)
    first3 = host(ssam.ssam_stencil3d(f3, c3, "zero"))
    assert np.array_equal(host(ssam.ssam_stencil3d(f3, c3, "zero")), first3)


def test_output_outside_grid_untouched_and_input_preserved(ssam):
    """The kernels must write exactly W*H elements and never modify the input."""
    H, W = 37, 259
    img = wl.uniform_field((H, W), 0.0, 1.0, 911, np.float32)
    filt = wl.seeded_filter(5, 5, 912, np.float32)
    big = torch.full((H + 2, W), -7.0, dtype=torch.float32, device="cuda")
    d_in = dev(img)
    out_view = big[1:H + 1]
    ssam.ssam_conv2d(d_in, filt, "clamp", d_out=out_view)
    res = host(big)
    assert np.all(res[0] == -7.0) and np.all(res[-1] == -7.0)
    assert_parity(res[1:H + 1], oracle.conv2d(img, filt, "clamp"), filt, 1.0)
    assert np.array_equal(host(d_in), img)


def test_config1_full(ssam):
    """Benchmark configuration 1 at its full size: 512x512 fp32 five-point star, zero padding, one sweep."""
    case = wl.config1()[0]
    fld = case.field()
    got = host(ssam.ssam_stencil2d(dev(fld), case.coef[0], case.boundary))
    want = oracle.stencil(fld, case.coef[0], case.boundary)
    assert_parity(got, want, case.coef, 1.0, case.name)


def test_errors_are_reported_not_launched(ssam):
    img = dev(np.zeros((8, 8), dtype=np.float32))
    filt = np.ones((3, 3), dtype=np.float32)
    with pytest.raises(ssam.SsamError) as e:
        ssam.ssam_conv2d(img, filt, "clamp", d_out=img)
    assert e.value.status == 5
    with pytest.raises(ssam.SsamError) as e:
        ssam.ssam_conv2d(img, np.ones((40, 3), dtype=np.float32), "clamp")
    assert e.value.status == 3
    with pytest.raises(ssam.SsamError) as e:
        ssam.ssam_stencil_iterate(img, torch.empty_like(img), filt, -1)
    assert e.value.status == 3


def test_latency_probe_orders_the_primitives(ssam):
    """The micro-benchmarks behind the latency table: every figure is positive and finite, a longer
    chain gives the same per-operation cost, and the orderings the kernel design rests on hold --
    a DPP lane shift costs about one VALU operation and far less than the same shift through the
    LDS crossbar or an LDS read (Sec. 5.1 of the paper puts the warp shuffle at the cost of a
    shared-memory read; here it is not)."""
    from paper_1907_06154_amd.binding import PROBE_OPS
    scratch = torch.empty(2 << 20, dtype=torch.uint8, device="cuda")
    lat = {}
    for op in PROBE_OPS:
        print(f"latency probe {op}", flush=True)
        ssam.ssam_probe_latency(op, 1, 1, 4096, scratch)
        c1, ns1 = ssam.ssam_probe_latency(op, 1, 1, 8192, scratch)
        c2, _ = ssam.ssam_probe_latency(op, 1, 1, 32768, scratch)
        assert np.isfinite(c1) and np.isfinite(ns1) and c1 > 0.5 and ns1 > 0.1 and c1 < 5000
        assert abs(c1 - c2) <= 0.15 * c2 + 1.0, (op, c1, c2)
        lat[op] = c2
        many, _ = ssam.ssam_probe_latency(op, 8, 4, 8192, scratch)
        assert many / 8 <= lat[op] * 1.1 + 1.0     # independent chains overlap
    assert lat["dpp_wave_shr"] < 3 * lat["fma_f32"]
    assert lat["dpp_wave_shr"] < 0.5 * lat["ds_bpermute"]
    assert lat["dpp_wave_shr"] < 0.5 * lat["lds_read"]
    assert lat["lds_read"] < lat["load_l2"]
    assert lat["load_l1"] <= lat["load_l2"] * 1.05
    assert lat["shift_f64"] < 3 * lat["dpp_wave_shr"] + 4
    with pytest.raises(ssam.SsamError):
        ssam.ssam_probe_latency("fma_f32", 3, 1, 4096, scratch)
    with pytest.raises(ssam.SsamError):
        ssam.ssam_probe_latency("fma_f32", 1, 1, 4096, scratch[:1024])


def test_direct_kernel_on_tall_and_deep_grids(ssam):
    """The one-point-per-thread kernel numbers its blocks in one grid dimension, so extents beyond the
    65535-block limit of the other two dimensions work (a filter too wide for any compiled box)."""
    filt = wl.seeded_filter(23, 1, 601, np.float32)
    img = wl.uniform_field((300000, 5), 0.0, 1.0, 602, np.float32)
    assert ssam.ssam_describe("conv2d", img.shape, filt, "clamp").split()[0] == "generic_direct"
    got = host(ssam.ssam_conv2d(dev(img), filt, "clamp"))
    assert_parity(got, oracle.conv2d(img, filt, "clamp"), filt, 1.0, "tall grid, direct kernel")
    coef = wl.seeded_coefficients(wl.mask_star(5, 5, 5), 603, np.float64)
    fld = wl.uniform_field((70000, 3, 4), -1.0, 1.0, 604, np.float64)
    assert ssam.ssam_describe("stencil3d", fld.shape, coef, "zero").split()[0] == "generic_direct"
    got = host(ssam.ssam_stencil3d(dev(fld), coef, "zero"))
    assert_parity(got, oracle.stencil(fld, coef, "zero"), coef, 1.0, "deep grid, direct kernel")


def test_direct_kernel_takes_every_shape_up_to_the_limits(ssam):
    """Shapes whose tap list exceeds one argument block run as several launches, every later one
    adding its part to the output: the largest filter and the largest dense boxes the header
    advertises, both precisions, both boundary rules."""
    for dt in (np.float32, np.float64):
        img = wl.uniform_field((45, 150), 0.0, 1.0, 611, dt)
        for (M, N) in ((32, 32), (30, 31), (22, 22), (32, 1)):
            filt = wl.seeded_filter(M, N, 612 + M, dt)
            for bnd in ("clamp", "zero"):
                print(f"direct conv2d {np.dtype(dt).name} {M}x{N} {bnd}", flush=True)
                got = host(ssam.ssam_conv2d(dev(img), filt, bnd))
                assert_parity(got, oracle.conv2d(img, filt, bnd), filt, 1.0, f"direct {M}x{N} {bnd}")
        fld = wl.uniform_field((11, 9, 70), -1.0, 1.0, 613, dt)
        for r in ((4, 4, 4), (8, 8, 8), (8, 3, 5)):
            coef = wl.seeded_coefficients(wl.mask_box(*r), 614, dt)
            for bnd in ("zero", "clamp"):
                print(f"direct stencil3d {np.dtype(dt).name} box r{r} {bnd}", flush=True)
                assert ssam.ssam_describe("stencil3d", fld.shape, coef, bnd).split()[0] == "generic_direct"
                got = host(ssam.ssam_stencil3d(dev(fld), coef, bnd))
                assert_parity(got, oracle.stencil(fld, coef, bnd), coef, 1.0, f"direct box r{r} {bnd}")
        # nothing but zeros: no tap at all, the output is zero everywhere (not left unwritten)
        none = np.zeros((17, 17, 17), dtype=dt)
        out = torch.full(fld.shape, float("nan"), dtype=torch.from_numpy(fld).dtype, device="cuda")
        got = host(ssam.ssam_stencil3d(dev(fld), none, "zero", d_out=out))
        assert np.array_equal(got, np.zeros_like(fld))


@pytest.mark.parametrize("shape,mask", [((200, 512), wl.mask_star(1, 1)), ((40, 64, 128), wl.mask_star(1, 1, 1)),
                                        ((33, 40, 130), wl.mask_star(4, 4, 4))])
def test_iterate_can_be_captured_in_a_hip_graph(ssam, shape, mask):
    """The entry points only enqueue kernels on the caller's stream (no allocation, no memset, no
    synchronisation), so a launch-bound time loop can be captured once and replayed.  Every replay
    is checked against the eager result, with eager work and synchronisations in between."""
    dtype = np.float32
    coef = wl.seeded_coefficients(mask, 610, dtype)
    coef = coef[0] if len(shape) == 2 else coef
    steps = 12
    fld = wl.uniform_field(shape, -1.0, 1.0, 611, dtype)
    want = oracle.iterate(fld, coef, steps, "zero")
    a0 = dev(fld)
    a, b = a0.clone(), torch.empty_like(a0)
    eager = host(ssam.ssam_stencil_iterate(a, b, coef, steps, "zero")).copy()     # also the warm-up launch
    assert_parity(eager, want, coef, 1.0, "eager")
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    a.copy_(a0)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        res = ssam.ssam_stencil_iterate(a, b, coef, steps, "zero")
    for replay in range(4):
        print(f"graph replay {replay} {shape}", flush=True)
        a.copy_(a0)
        b.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = host(res)
        assert np.array_equal(got, eager), f"replay {replay} differs from the eager run"
        # unrelated eager work between replays
        assert_parity(host(ssam.ssam_stencil_iterate(a0.clone(), torch.empty_like(a0), coef, 3, "zero")),
                      oracle.iterate(fld, coef, 3, "zero"), coef, 1.0, "eager between replays")


def test_concurrent_host_threads_on_their_own_streams(ssam):
    """Calls from several host threads, each on its own stream, give the results of serial calls
    (the dispatcher keeps no per-call state; tuning globals are not touched here)."""
    import threading
    jobs = []
    for k, (M, dt) in enumerate([(3, np.float32), (9, np.float32), (5, np.float64), (20, np.float32)]):
        filt = wl.seeded_filter(M, M, 700 + k, dt)
        img = wl.uniform_field((300, 1000), 0.0, 1.0, 710 + k, dt)
        jobs.append((filt, img, oracle.conv2d(img, filt, "clamp")))
    coef = wl.seeded_coefficients(wl.mask_star(1, 1, 1), 720, np.float64)
    fld = wl.uniform_field((40, 50, 200), -1.0, 1.0, 721, np.float64)
    want3 = oracle.iterate(fld, coef, 5, "zero")
    results, errors = {}, []

    def conv_worker(idx):
        try:
            filt, img, _ = jobs[idx]
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                d = dev(img)
                for _ in range(20):
                    out = ssam.ssam_conv2d(d, filt, "clamp", stream=stream)
                stream.synchronize()
                results[idx] = out.cpu().numpy()
        except Exception as e:   # surfaced in the main thread
            errors.append(e)

    def stencil_worker():
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                a = dev(fld)
                for _ in range(10):
                    res = ssam.ssam_stencil_iterate(a.clone(), torch.empty_like(a), coef, 5, "zero", stream=stream)
                stream.synchronize()
                results["s"] = res.cpu().numpy()
        except Exception as e:
            errors.append(e)

    threads = [threading.Thread(target=conv_worker, args=(i,)) for i in range(len(jobs))] + [threading.Thread(target=stencil_worker)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for idx, (filt, _, want) in enumerate(jobs):
        assert_parity(results[idx], want, filt, 1.0, f"thread {idx}")
    assert_parity(results["s"], want3, coef, 1.0, "stencil thread")
