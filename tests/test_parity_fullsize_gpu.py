"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The oracle cannot sweep an 8192x8192 or 512^3 grid 100 times in seconds, so the HIP result of
the whole run is compared on sampled windows: each window is evaluated by the oracle on a crop
grown by the dependency reach (radius x sweeps) and clipped to the grid, which gives the exact
values inside the window (see parity_util.expanded_window).  Windows sit on grid corners and
edges, across wave-tile seams and in the interior.  Same tolerance as the small cases."""
import numpy as np
import pytest

import oracle
import workloads as wl
from parity_util import assert_parity, oracle_window

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def ssam():
    import paper_1907_06154_amd as s
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    s.lib()
    return s


_FIELDS = {}


def field_of(case):
    """Full-size seeded field, generated once per (shape, seed) in float64 and cast."""
    key = (case.shape, case.field_seed, case.field_range)
    if key not in _FIELDS:
        _FIELDS.clear()          # keep at most one full-size field on the host
        _FIELDS[key] = wl.uniform_field(case.shape, case.field_range[0], case.field_range[1], case.field_seed,
                                        np.float64)
    return _FIELDS[key].astype(case.dtype, copy=False)


def run_gpu(ssam, case):
    fld = field_of(case)
    a = torch.from_numpy(np.ascontiguousarray(fld)).cuda()
    b = torch.empty_like(a)
    if case.kind == "conv2d":
        res = ssam.ssam_conv2d(a, case.coef, case.boundary, d_out=b)
    elif case.kind == "conv3d":
        res = ssam.ssam_conv3d(a, case.coef, case.boundary, d_out=b)
    else:
        coef = case.coef if case.kind == "stencil3d" else case.coef[0]
        res = ssam.ssam_stencil_iterate(a, b, coef, case.steps, case.boundary)
    torch.cuda.synchronize()
    return res


def windows_2d(n, h, w):
    """Corners, edges, tile seams (x = 244 and 248 are strip seams for fp32 / fp64, y = 32, 64 row-tile seams)."""
    return [((0, 0), (h, w)), ((0, n - w), (h, n)), ((n - h, 0), (n, w)), ((n - h, n - w), (n, n)),
            ((20, 200), (20 + h, 200 + w)), ((n // 2 - 7, n // 2 - 33), (n // 2 - 7 + h, n // 2 - 33 + w)),
            ((n - h, 3000), (n, 3000 + w))]


def windows_3d(n, s):
    m = n // 2
    return [((0, 0, 0), (s, s, s)), ((n - s, n - s, n - s), (n, n, n)), ((0, n - s, 96), (s, n, 96 + s)),
            ((60, 2, 100), (60 + s, 2 + s, 100 + s)), ((m - 3, m - 5, m - 9), (m - 3 + s, m - 5 + s, m - 9 + s))]


def check(ssam, case, windows):
    res = run_gpu(ssam, case)
    in_max = max(abs(case.field_range[0]), abs(case.field_range[1]))
    worst = 0.0
    for lo, hi in windows:
        print(f"{case.name}: window {lo}..{hi}", flush=True)
        sl = tuple(slice(l, h) for l, h in zip(lo, hi))
        got = res[sl].cpu().numpy()
        want = oracle_window(case, lo, hi)
        worst = max(worst, assert_parity(got, want, case.coef, in_max, f"{case.name} {lo}"))
    print(f"{case.name}: worst normalised error {worst:.2e}", flush=True)


@pytest.mark.parametrize("case", wl.config2(), ids=lambda c: c.name)
def test_config2_full_size(ssam, case):
    check(ssam, case, windows_2d(8192, 48, 320))


@pytest.mark.parametrize("name", ["c2_conv3x3_f32", "c2_conv9x9_f32", "c2_conv20x20_f32", "c2_conv11x3_f32"])
def test_config2_full_grid(ssam, name):
    """Every one of the 67 M outputs of a configuration-2 pass against the oracle's full field (one
    bandwidth-bound filter, the two matrix-core ones at either end of their range, and the wide one);
    the oracle needs a few seconds per filter on the GPU machine's host cores."""
    case = next(c for c in wl.config2() if c.name == name)
    res = run_gpu(ssam, case).cpu().numpy()
    print(f"{name}: oracle on the full {case.shape} grid", flush=True)
    want = oracle.conv2d(field_of(case), case.coef, case.boundary)
    err = assert_parity(res, want, case.coef, 1.0, f"{name} full grid")
    print(f"{name}: worst normalised error over {res.size} points {err:.2e}", flush=True)


@pytest.mark.parametrize("case", wl.config3(), ids=lambda c: c.name)
def test_config3_full_size_100_sweeps(ssam, case):
    wins = windows_2d(8192, 24, 40)
    check(ssam, case, [wins[0], wins[3], wins[4], wins[5]])


@pytest.mark.parametrize("case", wl.config4(), ids=lambda c: c.name)
def test_config4_full_size_10_sweeps(ssam, case):
    check(ssam, case, windows_3d(512, 24))


@pytest.mark.parametrize("case", wl.config5(), ids=lambda c: c.name)
def test_config5_full_size_20_sweeps(ssam, case):
    wins = windows_3d(512, 12)
    check(ssam, case, [wins[0], wins[1], wins[3], wins[4]])


@pytest.mark.parametrize("case", wl.conv3d_filters(), ids=lambda c: c.name)
def test_conv3d_full_size(ssam, case):
    """The 512^3 dense 3D filters that bench.py --workload conv3d times: cubes with an instance of their own,
    an even cube and a flat box that run inside a larger cube."""
    check(ssam, case, windows_3d(512, 20))


def test_full_size_run_is_deterministic(ssam):
    case = wl.config4()[1]
    first = run_gpu(ssam, case).clone()
    second = run_gpu(ssam, case)
    assert torch.equal(first, second)
