"""GPU parity at the largest grids the C ABI accepts (just under 2^31 elements): index arithmetic
beyond 32 bits, tile counts two orders of magnitude above the benchmark sizes.

The field is generated on the device by the bit-identical torch version of the seeded generator;
the oracle evaluates sampled windows (grid corners, the far end of the address range, tile seams,
the interior) on crops regenerated from the same counters.  Same tolerance as everywhere else."""
import numpy as np
import pytest

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


def corners_and_middle(shape, win):
    """Windows at every low/high corner combination of the two outermost axes plus the middle."""
    out = []
    nd = len(shape)
    for mask in range(4):
        lo = []
        for ax in range(nd):
            high = (mask >> ax) & 1 if ax < 2 else (mask & 1)
            lo.append(shape[ax] - win[ax] if high else 0)
        out.append(tuple(lo))
    out.append(tuple(s // 2 - w // 2 for s, w in zip(shape, win)))
    out.append(tuple(min(s - w, s // 3 + 5) for s, w in zip(shape, win)))
    return [(lo, tuple(l + w for l, w in zip(lo, win))) for lo in dict.fromkeys(out)]


CASES = [
    wl.Case("max_conv5x5_f32", "conv2d", np.float32, (65535, 32768), (0.0, 1.0), 41,
            wl.seeded_filter(5, 5, 42, np.float32), "clamp", 1, "2^31 - 2^15 elements"),
    wl.Case("max_2d_star_r1_f32_fused", "stencil2d", np.float32, (46340, 46340), (-1.0, 1.0), 43,
            wl.seeded_coefficients(wl.mask_star(1, 1), 44, np.float32), "zero", 4, "four sweeps in one launch"),
    wl.Case("max_2d_box_r1_f32_unaligned", "stencil2d", np.float32, (46341, 46339), (-1.0, 1.0), 45,
            wl.seeded_coefficients(wl.mask_box(1, 1), 46, np.float32), "clamp", 1, "odd row length: element path"),
    wl.Case("max_3d_star_r1_f32_fused", "stencil3d", np.float32, (1290, 1290, 1288), (-1.0, 1.0), 47,
            wl.seeded_coefficients(wl.mask_star(1, 1, 1), 48, np.float32), "zero", 2, "two sweeps in one launch"),
    wl.Case("max_3d_box_r1_f32", "stencil3d", np.float32, (1290, 1290, 1288), (-1.0, 1.0), 47,
            wl.seeded_coefficients(wl.mask_box(1, 1, 1), 49, np.float32), "clamp", 1, "single sweep"),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: c.name)
def test_largest_grids(ssam, case):
    assert case.points < 2 ** 31 and case.points > 2 ** 31 - 2 ** 24
    print(f"{case.name}: generating {case.points} points on the device", flush=True)
    a = wl.uniform_field_on("cuda", case.shape, case.field_range[0], case.field_range[1], case.field_seed, case.dtype)
    b = torch.empty_like(a)
    # the device generator is the host generator: spot-check the last row of the grid
    last = tuple(s - 1 for s in case.shape[:-1])
    want_row = case.window(last + (0,), (1,) * (len(case.shape) - 1) + (case.shape[-1],)).ravel()
    assert np.array_equal(a[last].cpu().numpy(), want_row)
    print(f"{case.name}: launching", flush=True)
    if case.kind == "conv2d":
        res = ssam.ssam_conv2d(a, case.coef, case.boundary, d_out=b)
    else:
        coef = case.coef if case.kind == "stencil3d" else case.coef[0]
        res = ssam.ssam_stencil_iterate(a, b, coef, case.steps, case.boundary)
    torch.cuda.synchronize()
    win = (24, 300) if len(case.shape) == 2 else (10, 12, 200)
    in_max = max(abs(case.field_range[0]), abs(case.field_range[1]))
    for lo, hi in corners_and_middle(case.shape, win):
        print(f"{case.name}: window {lo}..{hi}", flush=True)
        sl = tuple(slice(l, h) for l, h in zip(lo, hi))
        got = res[sl].cpu().numpy()
        assert_parity(got, oracle_window(case, lo, hi), case.coef, in_max, f"{case.name} {lo}")
    del a, b, res
    torch.cuda.empty_cache()
