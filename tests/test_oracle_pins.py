"""Pins for the CPU oracle: every check here compares oracle/ against something other than
itself (exact rational arithmetic written a different way, closed forms, hand-worked values
from the equations of Sec. 2.1 / 2.2, scipy.ndimage and torch routines, identities).
None of these tests needs a GPU."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as wl

DTYPES = [np.float32, np.float64]


# ---------------------------------------------------------------------------------------
# Independent evaluators (tap-list driven, exact rationals) -- not the oracle's loop nest.
# ---------------------------------------------------------------------------------------

def _fetch(field, coords, boundary):
    """field indexed [z][y][x]; coords (x, y, z) possibly outside."""
    D, H, W = field.shape
    x, y, z = coords
    if boundary == "clamp":
        x = min(max(x, 0), W - 1)
        y = min(max(y, 0), H - 1)
        z = min(max(z, 0), D - 1)
    elif not (0 <= x < W and 0 <= y < H and 0 <= z < D):
        return Fraction(0)
    return Fraction(float(field[z, y, x]))


def exact_taps(field3, taps, boundary):
    """taps: list of (dx, dy, dz, coef).  Returns an object array of Fractions."""
    D, H, W = field3.shape
    out = np.empty((D, H, W), dtype=object)
    for z in range(D):
        for y in range(H):
            for x in range(W):
                acc = Fraction(0)
                for dx, dy, dz, c in taps:
                    acc += Fraction(float(c)) * _fetch(field3, (x + dx, y + dy, z + dz), boundary)
                out[z, y, x] = acc
    return out


def round_to(exact, dtype):
    f = np.vectorize(lambda q: float(q), otypes=[np.float64])(exact)
    return f.astype(dtype)


def assert_within_ulp(got, exact, dtype, ulps=1.0):
    want = round_to(exact, dtype)
    tol = ulps * np.spacing(np.abs(want).astype(dtype)).astype(np.float64)
    tol = np.maximum(tol, np.finfo(dtype).tiny)
    assert got.dtype == np.dtype(dtype)
    assert np.all(np.abs(got.astype(np.float64) - want.astype(np.float64)) <= tol)


def filter_taps(filt, ax, ay):
    N, M = filt.shape
    return [(m - ax, n - ay, 0, filt[n, m]) for n in range(N) for m in range(M)]


def box_taps(coef3):
    nz, ny, nx = coef3.shape
    rz, ry, rx = nz // 2, ny // 2, nx // 2
    return [(i - rx, j - ry, k - rz, coef3[k, j, i])
            for k in range(nz) for j in range(ny) for i in range(nx) if coef3[k, j, i] != 0]


def rng_field(shape, seed, dtype, lo=-1.0, hi=1.0):
    return wl.uniform_field(shape, lo, hi, seed, dtype)


# ---------------------------------------------------------------------------------------
# 1. Exact brute force on tiny grids (grids smaller than the filter, even sizes, M != N,
#    explicit anchors, both boundary rules, both precisions).
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("boundary", ["zero", "clamp"])
@pytest.mark.parametrize("W,H,M,N,anchor", [
    (7, 5, 3, 3, None), (7, 5, 2, 2, None), (6, 4, 4, 3, None), (5, 6, 3, 11, None), (9, 3, 11, 3, None),
    (4, 3, 6, 5, None), (7, 5, 3, 2, (0, 0)), (7, 5, 4, 3, (3, 2)), (1, 1, 3, 3, None), (8, 1, 3, 1, None),
])
def test_conv2d_exact_bruteforce(dtype, boundary, W, H, M, N, anchor):
    img = rng_field((H, W), 11, dtype)
    filt = wl.seeded_filter(M, N, 12, dtype)
    ax, ay = (M // 2, N // 2) if anchor is None else anchor
    got = oracle.conv2d(img, filt, boundary, anchor)
    exact = exact_taps(img[None], filter_taps(filt, ax, ay), boundary)[0]
    assert_within_ulp(got, exact, dtype)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("boundary", ["zero", "clamp"])
@pytest.mark.parametrize("shape,mask", [
    ((5, 7), wl.mask_star(1, 1)[0]), ((5, 7), wl.mask_box(2, 1)[0]), ((3, 4), wl.mask_star(4, 4)[0]),
    ((6, 5), wl.mask_star(1, 2)[0]),
    ((4, 3, 5), wl.mask_star(1, 1, 1)), ((4, 3, 5), wl.mask_box(1, 1, 1)), ((3, 4, 4), wl.mask_faces_edges()),
    ((2, 3, 9), wl.mask_star(4, 1, 2)), ((5, 2, 3), wl.mask_box(1, 2, 1)),
])
def test_stencil_exact_bruteforce(dtype, boundary, shape, mask):
    fld = rng_field(shape, 21, dtype)
    mask3 = mask if mask.ndim == 3 else mask[None]
    coef3 = wl.seeded_coefficients(mask3, 22, dtype, -1.0, 1.0, normalise=False)
    coef = coef3 if len(shape) == 3 else coef3[0]
    got = oracle.stencil(fld, coef, boundary)
    f3 = fld if fld.ndim == 3 else fld[None]
    exact = exact_taps(f3, box_taps(coef3), boundary)
    exact = exact if fld.ndim == 3 else exact[0]
    assert_within_ulp(got, exact, dtype)


# ---------------------------------------------------------------------------------------
# 2. Hand-worked values straight from the equations.
# ---------------------------------------------------------------------------------------

def test_five_point_equation_by_hand():
    """Sec. 2.2: s'(x,y) = s(x-1,y)West + s(x,y-1)North + s(x,y)Current + s(x,y+1)South + s(x+1,y)East."""
    s = np.array([[1, 2, 3], [4, 5, 6], [7, 8, 9]], dtype=np.float64)   # s[y][x]
    West, North, Current, South, East = 1.0, 2.0, 3.0, 4.0, 5.0
    coef = np.array([[0, North, 0], [West, Current, East], [0, South, 0]], dtype=np.float64)
    out = oracle.stencil(s, coef, "zero")
    # centre (x=1,y=1): 4*1 + 2*2 + 5*3 + 8*4 + 6*5
    assert out[1, 1] == 85.0
    # corner (x=0,y=0), zero padding: 0*1 + 0*2 + 1*3 + 4*4 + 2*5
    assert out[0, 0] == 29.0
    # edge (x=2,y=1): 5*1 + 3*2 + 6*3 + 9*4 + 0*5
    assert out[1, 2] == 65.0
    outc = oracle.stencil(s, coef, "clamp")
    # corner with clamp: west->s(0,0)=1, north->1 : 1*1 + 1*2 + 1*3 + 4*4 + 2*5
    assert outc[0, 0] == 32.0
    assert outc[1, 1] == 85.0


def test_seven_point_above_below_by_hand():
    """Sec. 2.2 last paragraph: Above multiplies s(x,y,z-1), Below s(x,y,z+1)."""
    s = np.arange(27, dtype=np.float64).reshape(3, 3, 3)                # s[z][y][x]
    coef = np.zeros((3, 3, 3))
    coef[0, 1, 1] = 10.0     # Above: dz = -1
    coef[2, 1, 1] = 100.0    # Below: dz = +1
    coef[1, 1, 1] = 1.0
    out = oracle.stencil(s, coef, "zero")
    assert out[1, 1, 1] == 13.0 + 10.0 * 4.0 + 100.0 * 22.0
    assert out[0, 1, 1] == 4.0 + 100.0 * 13.0            # nothing above the first plane
    assert out[2, 0, 2] == 20.0 + 10.0 * 11.0


def test_one_dimensional_example():
    """Sec. 3.5: three-tap 1D filter, b_i = a_{i-1} f_0 + a_i f_1 + a_{i+1} f_2."""
    a = np.array([[3, 1, 4, 1, 5, 9, 2, 6]], dtype=np.float32)
    f = np.array([[2, 3, 5]], dtype=np.float32)
    b = oracle.conv2d(a, f, "zero")
    want = [3 * 3 + 1 * 5, 3 * 2 + 1 * 3 + 4 * 5, 1 * 2 + 4 * 3 + 1 * 5, 4 * 2 + 1 * 3 + 5 * 5,
            1 * 2 + 5 * 3 + 9 * 5, 5 * 2 + 9 * 3 + 2 * 5, 9 * 2 + 2 * 3 + 6 * 5, 2 * 2 + 6 * 3]
    assert b[0].tolist() == [float(v) for v in want]


def test_true_convolution_is_correlation_with_flipped_filter():
    """Sec. 2.1's canonical form (f*w)(x,y) = sum_{s,t} f(x-s, y-t) w(s,t), evaluated literally,
    equals the oracle (which does not flip, like Listing 1) called with the filter flipped."""
    dtype = np.float64
    H, W, M, N = 6, 7, 3, 5
    img = np.round(rng_field((H, W), 31, dtype) * 16)        # small integers: exact arithmetic
    w = np.round(wl.seeded_filter(M, N, 32, dtype) * 8)
    a, c = -(M // 2), -(N // 2)                               # s in [a, a+M), t in [c, c+N)
    literal = np.zeros((H, W))
    for y in range(H):
        for x in range(W):
            acc = 0.0
            for t in range(c, c + N):
                for s in range(a, a + M):
                    xs, yt = x - s, y - t
                    if 0 <= xs < W and 0 <= yt < H:
                        acc += img[yt, xs] * w[t - c, s - a]
            literal[y, x] = acc
    got = oracle.conv2d(img, np.ascontiguousarray(w[::-1, ::-1]), "zero", anchor=(M - 1 - M // 2, N - 1 - N // 2))
    assert np.array_equal(got, literal)


# ---------------------------------------------------------------------------------------
# 3. Delta, constant and linear inputs.
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", DTYPES)
def test_delta_reproduces_filter_point_reflected(dtype):
    M, N, W, H = 5, 4, 16, 13
    ax, ay = M // 2, N // 2
    filt = wl.seeded_filter(M, N, 41, dtype)
    x0, y0 = 8, 6
    img = np.zeros((H, W), dtype=dtype)
    img[y0, x0] = 1
    out = oracle.conv2d(img, filt, "zero")
    want = np.zeros_like(img)
    for n in range(N):
        for m in range(M):
            want[y0 + ay - n, x0 + ax - m] = filt[n, m]
    assert np.array_equal(out, want)


def test_delta_at_corner_zero_cuts_and_clamp_sums():
    dtype = np.float64
    filt = (np.arange(9, dtype=dtype).reshape(3, 3) + 1)          # w[n][m] = 3n+m+1
    img = np.zeros((5, 6), dtype=dtype)
    img[0, 0] = 1
    z = oracle.conv2d(img, filt, "zero")
    # out[y][x] = w[n][m] with x+m-1 == 0, y+n-1 == 0 -> m = 1-x, n = 1-y
    assert z[0, 0] == filt[1, 1] and z[0, 1] == filt[1, 0] and z[1, 0] == filt[0, 1] and z[1, 1] == filt[0, 0]
    assert np.count_nonzero(z) == 4
    c = oracle.conv2d(img, filt, "clamp")
    # at (0,0) every tap with x+m-1 <= 0 and y+n-1 <= 0 clamps onto the delta: m in {0,1}, n in {0,1}
    assert c[0, 0] == filt[0, 0] + filt[0, 1] + filt[1, 0] + filt[1, 1]
    assert c[0, 1] == filt[0, 0] + filt[1, 0]      # x=1: only m=0 reaches column 0; n in {0,1}
    assert c[1, 0] == filt[0, 0] + filt[0, 1]
    assert c[1, 1] == filt[0, 0]


@pytest.mark.parametrize("dtype", DTYPES)
def test_constant_field_sums_weights(dtype):
    """Dyadic constants and weights make every sum exact.  Zero padding: a point near the edge
    gets the sum of the taps that still fall inside, which exposes anchor and orientation."""
    M, N, W, H = 4, 3, 9, 8
    ax, ay = M // 2, N // 2
    filt = (np.round(wl.seeded_filter(M, N, 51, np.float64) * 64) / 64).astype(dtype)
    c0 = dtype(0.375)
    img = np.full((H, W), c0, dtype=dtype)
    clamp = oracle.conv2d(img, filt, "clamp")
    assert np.all(clamp == dtype(c0 * filt.astype(np.float64).sum()))
    zero = oracle.conv2d(img, filt, "zero")
    for y in range(H):
        for x in range(W):
            inside = sum(float(filt[n, m]) for n in range(N) for m in range(M)
                         if 0 <= x + m - ax < W and 0 <= y + n - ay < H)
            assert zero[y, x] == dtype(float(c0) * inside)


@pytest.mark.parametrize("dims", [2, 3])
def test_linear_field_preserved_by_symmetric_unit_sum_stencil(dims):
    dtype = np.float64
    r = 2
    coef = wl.seeded_symmetric_star(r, dims, 61, dtype)
    n = 12
    if dims == 2:
        yy, xx = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
        fld = (0.5 * xx - 0.25 * yy + 3).astype(dtype)
        out = oracle.stencil(fld, coef[0], "zero")
        sl = (slice(r, n - r),) * 2
    else:
        zz, yy, xx = np.meshgrid(np.arange(n), np.arange(n), np.arange(n), indexing="ij")
        fld = (0.5 * xx - 0.25 * yy + 2.0 * zz + 3).astype(dtype)
        out = oracle.stencil(fld, coef, "zero")
        sl = (slice(r, n - r),) * 3
    assert np.allclose(out[sl], fld[sl], rtol=0, atol=1e-13)
    assert not np.allclose(out, fld, rtol=0, atol=1e-3)      # the zero-padded rim does change


# ---------------------------------------------------------------------------------------
# 4. Library routines as special cases.
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("boundary,mode", [("zero", "constant"), ("clamp", "nearest")])
@pytest.mark.parametrize("M,N", [(3, 3), (5, 5), (2, 2), (4, 6), (3, 11), (11, 3), (20, 20)])
def test_conv2d_matches_scipy_correlate(boundary, mode, M, N):
    from scipy import ndimage
    img = rng_field((37, 45), 71, np.float64)
    filt = wl.seeded_filter(M, N, 72, np.float64)
    got = oracle.conv2d(img, filt, boundary)
    want = ndimage.correlate(img, filt, mode=mode, cval=0.0, origin=0)
    assert np.allclose(got, want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("boundary,mode", [("zero", "constant"), ("clamp", "nearest")])
def test_stencil3d_matches_scipy_correlate(boundary, mode):
    from scipy import ndimage
    fld = rng_field((9, 11, 13), 73, np.float64)
    for mask in (wl.mask_star(1, 1, 1), wl.mask_box(1, 1, 1), wl.mask_faces_edges(), wl.mask_star(4, 4, 4),
                 wl.mask_box(2, 1, 0)):
        coef = wl.seeded_coefficients(mask, 74, np.float64, -1.0, 1.0, normalise=False)
        got = oracle.stencil(fld, coef, boundary)
        want = ndimage.correlate(fld, coef, mode=mode, cval=0.0, origin=0)
        assert np.allclose(got, want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("boundary,pad_mode", [("zero", "constant"), ("clamp", "replicate")])
@pytest.mark.parametrize("anchor", [None, (0, 0), (3, 1)])
def test_conv2d_matches_torch_conv2d(boundary, pad_mode, anchor):
    import torch
    import torch.nn.functional as F
    M, N = 4, 3
    ax, ay = (M // 2, N // 2) if anchor is None else anchor
    img = rng_field((19, 23), 75, np.float32)
    filt = wl.seeded_filter(M, N, 76, np.float32)
    got = oracle.conv2d(img, filt, boundary, anchor)
    t = torch.from_numpy(img.astype(np.float64))[None, None]
    t = F.pad(t, (ax, M - 1 - ax, ay, N - 1 - ay), mode=pad_mode)
    want = F.conv2d(t, torch.from_numpy(filt.astype(np.float64))[None, None])[0, 0].numpy()
    assert np.allclose(got, want, rtol=0, atol=2e-6)


# ---------------------------------------------------------------------------------------
# 3D filter (Sec. 2.1 with a z index): brute force, delta, library routines, reductions.
# ---------------------------------------------------------------------------------------

def filter_taps3(filt, ax, ay, az):
    K, N, M = filt.shape
    return [(m - ax, n - ay, k - az, filt[k, n, m]) for k in range(K) for n in range(N) for m in range(M)]


def seeded_filter3(M, N, K, seed, dtype):
    return wl.uniform_field((K, N, M), -1.0, 1.0, seed, dtype)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("boundary", ["zero", "clamp"])
@pytest.mark.parametrize("W,H,D,M,N,K,anchor", [
    (6, 5, 4, 3, 3, 3, None), (5, 4, 3, 2, 2, 2, None), (4, 5, 3, 4, 3, 2, None), (3, 2, 2, 5, 3, 4, None),
    (5, 4, 3, 3, 2, 2, (0, 0, 0)), (5, 4, 3, 4, 3, 2, (3, 2, 1)), (1, 1, 1, 3, 3, 3, None), (6, 1, 1, 3, 1, 1, None),
    (4, 3, 5, 1, 1, 4, (0, 0, 3)),
])
def test_conv3d_exact_bruteforce(dtype, boundary, W, H, D, M, N, K, anchor):
    vol = rng_field((D, H, W), 171, dtype)
    filt = seeded_filter3(M, N, K, 172, dtype)
    ax, ay, az = (M // 2, N // 2, K // 2) if anchor is None else anchor
    got = oracle.conv3d(vol, filt, boundary, anchor)
    exact = exact_taps(vol, filter_taps3(filt, ax, ay, az), boundary)
    assert_within_ulp(got, exact, dtype)


@pytest.mark.parametrize("dtype", DTYPES)
def test_conv3d_delta_reproduces_filter_point_reflected(dtype):
    """A unit impulse at p0 puts w[k][n][m] at p0 + anchor - (m, n, k): the filter reflected through the
    anchor, on every axis -- an axis mixed up with another, or a sign error, moves entries."""
    M, N, K, W, H, D = 4, 3, 5, 11, 9, 12
    ax, ay, az = 1, 2, 3
    filt = seeded_filter3(M, N, K, 173, dtype)
    x0, y0, z0 = 5, 4, 6
    vol = np.zeros((D, H, W), dtype=dtype)
    vol[z0, y0, x0] = 1
    out = oracle.conv3d(vol, filt, "zero", (ax, ay, az))
    want = np.zeros_like(vol)
    for k in range(K):
        for n in range(N):
            for m in range(M):
                want[z0 + az - k, y0 + ay - n, x0 + ax - m] = filt[k, n, m]
    assert np.array_equal(out, want)


@pytest.mark.parametrize("boundary,mode", [("zero", "constant"), ("clamp", "nearest")])
@pytest.mark.parametrize("MNK,anchor", [((3, 3, 3), None), ((2, 2, 2), None), ((4, 3, 2), None), ((5, 2, 3), (0, 1, 2)),
                                        ((3, 5, 4), (2, 0, 3)), ((7, 7, 7), None), ((1, 1, 6), None)])
def test_conv3d_matches_scipy_correlate_with_origin(boundary, mode, MNK, anchor):
    """scipy centres an even or odd filter at size // 2 and moves it with `origin` (axis order z, y, x):
    the filter element on the output point is size // 2 + origin."""
    from scipy import ndimage
    M, N, K = MNK
    ax, ay, az = (M // 2, N // 2, K // 2) if anchor is None else anchor
    vol = rng_field((10, 12, 13), 174, np.float64)
    filt = seeded_filter3(M, N, K, 175, np.float64)
    got = oracle.conv3d(vol, filt, boundary, anchor)
    want = ndimage.correlate(vol, filt, mode=mode, cval=0.0, origin=(az - K // 2, ay - N // 2, ax - M // 2))
    assert np.allclose(got, want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("boundary,pad_mode", [("zero", "constant"), ("clamp", "replicate")])
@pytest.mark.parametrize("anchor", [None, (0, 0, 0), (3, 1, 1)])
def test_conv3d_matches_torch_conv3d(boundary, pad_mode, anchor):
    import torch
    import torch.nn.functional as F
    M, N, K = 4, 3, 2
    ax, ay, az = (M // 2, N // 2, K // 2) if anchor is None else anchor
    vol = rng_field((7, 9, 11), 176, np.float32)
    filt = seeded_filter3(M, N, K, 177, np.float32)
    got = oracle.conv3d(vol, filt, boundary, anchor)
    t = torch.from_numpy(vol.astype(np.float64))[None, None]
    t = F.pad(t, (ax, M - 1 - ax, ay, N - 1 - ay, az, K - 1 - az), mode=pad_mode)
    want = F.conv3d(t, torch.from_numpy(filt.astype(np.float64))[None, None])[0, 0].numpy()
    assert np.allclose(got, want, rtol=0, atol=2e-6)


def test_conv3d_reduces_to_conv2d_and_to_the_stencil():
    """One filter plane (K = 1) on every z-plane separately is the 2D filter; an odd box without zero
    entries, anchored at its centre, is the 3D stencil with that coefficient box."""
    vol = rng_field((5, 8, 9), 178, np.float64)
    f2 = wl.seeded_filter(4, 3, 179, np.float64)
    got = oracle.conv3d(vol, f2[None], "clamp", (1, 2, 0))
    for z in range(vol.shape[0]):
        assert np.array_equal(got[z], oracle.conv2d(vol[z], f2, "clamp", (1, 2)))
    box = wl.seeded_coefficients(wl.mask_box(1, 2, 1), 180, np.float64, 0.5, 1.0, normalise=False)
    assert np.all(box != 0)
    for bnd in ("zero", "clamp"):
        assert np.array_equal(oracle.conv3d(vol, box, bnd), oracle.stencil(vol, box, bnd))


def test_conv3d_constant_field_enumerates_partial_sums():
    """Constant input, zero padding: the output at a corner is the sum of the filter entries whose tap
    stays inside the grid; every anchor / orientation mistake changes which entries those are.  Dyadic
    values, so the sums are exact."""
    M, N, K = 3, 2, 4
    filt = (np.arange(M * N * K, dtype=np.float64).reshape(K, N, M) - 7.0) / 8.0
    vol = np.full((6, 5, 7), 0.5)
    for anchor in [(1, 1, 2), (0, 0, 0), (2, 1, 3)]:
        ax, ay, az = anchor
        out = oracle.conv3d(vol, filt, "zero", anchor)
        for (x, y, z) in [(0, 0, 0), (6, 4, 5), (0, 4, 2), (3, 2, 3)]:
            want = 0.0
            for k in range(K):
                for n in range(N):
                    for m in range(M):
                        if 0 <= x + m - ax < 7 and 0 <= y + n - ay < 5 and 0 <= z + k - az < 6:
                            want += filt[k, n, m] * 0.5
            assert out[z, y, x] == want
        assert np.array_equal(oracle.conv3d(vol, filt, "clamp", anchor), np.full_like(vol, 0.5 * filt.sum()))


def test_stencil3d_matches_torch_conv3d():
    import torch
    import torch.nn.functional as F
    fld = rng_field((6, 7, 8), 77, np.float64)
    coef = wl.seeded_coefficients(wl.mask_box(2, 1, 1), 78, np.float64, -1.0, 1.0, normalise=False)
    got = oracle.stencil(fld, coef, "zero")
    want = F.conv3d(torch.from_numpy(fld)[None, None], torch.from_numpy(coef)[None, None],
                    padding=(1, 1, 2))[0, 0].numpy()
    assert np.allclose(got, want, rtol=0, atol=1e-12)


def test_separable_filter_equals_row_then_column_pass():
    dtype = np.float64
    u = wl.uniform_at(np.arange(5), -1, 1, 81, dtype)       # vertical factor (N=5)
    v = wl.uniform_at(np.arange(7), -1, 1, 82, dtype)       # horizontal factor (M=7)
    img = rng_field((21, 26), 83, dtype)
    full = oracle.conv2d(img, np.outer(u, v), "zero")
    rows = oracle.conv2d(img, v[None, :], "zero")
    both = oracle.conv2d(rows, u[:, None], "zero")
    assert np.allclose(full, both, rtol=0, atol=1e-13)


# ---------------------------------------------------------------------------------------
# 5. Iteration (Jacobi, two buffers).
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", DTYPES)
def test_iterate_identities(dtype):
    fld = rng_field((14, 17), 91, dtype)
    coef = wl.seeded_coefficients(wl.mask_box(2, 2), 92, dtype)[0]
    assert np.array_equal(oracle.iterate(fld, coef, 0), fld)
    assert np.array_equal(oracle.iterate(fld, coef, 1), oracle.stencil(fld, coef, "zero"))
    five = oracle.iterate(fld, coef, 5)
    assert np.array_equal(oracle.iterate(oracle.iterate(fld, coef, 2), coef, 3), five)
    # explicit repeated single sweeps, odd and even step counts (buffer parity)
    cur = fld
    for _ in range(4):
        cur = oracle.stencil(cur, coef, "zero")
    assert np.array_equal(oracle.iterate(fld, coef, 4), cur)


def test_iterate_is_a_max_norm_contraction_and_linear():
    dtype = np.float64
    coef = wl.seeded_coefficients(wl.mask_star(1, 1, 1), 93, dtype)        # w >= 0, sum 1
    u = rng_field((6, 7, 8), 94, dtype)
    v = rng_field((6, 7, 8), 95, dtype)
    prev = np.abs(u).max()
    for t in range(1, 5):
        cur = np.abs(oracle.iterate(u, coef, t)).max()
        assert cur <= prev + 1e-15
        prev = cur
    lhs = oracle.iterate(2.0 * u - 0.5 * v, coef, 3)
    rhs = 2.0 * oracle.iterate(u, coef, 3) - 0.5 * oracle.iterate(v, coef, 3)
    assert np.allclose(lhs, rhs, rtol=0, atol=1e-14)


def test_iterate_3d_matches_repeated_scipy():
    from scipy import ndimage
    fld = rng_field((7, 8, 9), 96, np.float64)
    coef = wl.seeded_coefficients(wl.mask_faces_edges(), 97, np.float64)
    want = fld
    for _ in range(3):
        want = ndimage.correlate(want, coef, mode="constant", cval=0.0)
    assert np.allclose(oracle.iterate(fld, coef, 3), want, rtol=0, atol=1e-13)


def test_zero_coefficient_means_no_tap():
    """An exactly-zero coefficient is skipped, so a non-finite neighbour under it does not leak."""
    fld = np.ones((5, 5), dtype=np.float64)
    fld[2, 1] = np.inf
    coef = np.array([[0, 1, 0], [0, 1, 1], [0, 1, 0]], dtype=np.float64)    # no West tap
    out = oracle.stencil(fld, coef, "zero")
    assert out[2, 2] == 4.0
    assert np.isinf(out[2, 1])


# ---------------------------------------------------------------------------------------
# 6. The windowed evaluation used by the full-size GPU parity tests equals the full-grid oracle.
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("kind", ["conv2d", "stencil2d", "stencil3d"])
def test_windowed_oracle_equals_full_grid_oracle(kind):
    from parity_util import oracle_window
    if kind == "conv2d":
        case = wl.Case("w_conv", "conv2d", np.float32, (40, 50), (0.0, 1.0), 3, wl.seeded_filter(5, 4, 9, np.float32),
                       "clamp", 1)
        full = oracle.conv2d(case.field(), case.coef, "clamp")
        wins = [((0, 0), (6, 7)), ((34, 43), (40, 50)), ((15, 20), (22, 31)), ((0, 30), (3, 50))]
    elif kind == "stencil2d":
        case = wl.Case("w_s2", "stencil2d", np.float64, (40, 50), (-1.0, 1.0), 5,
                       wl.seeded_coefficients(wl.mask_star(2, 2), 8, np.float64), "zero", 4)
        full = oracle.iterate(case.field(), case.coef[0], 4, "zero")
        wins = [((0, 0), (6, 7)), ((34, 43), (40, 50)), ((15, 20), (22, 31))]
    else:
        case = wl.Case("w_s3", "stencil3d", np.float64, (14, 15, 16), (-1.0, 1.0), 6,
                       wl.seeded_coefficients(wl.mask_box(1, 1, 1), 7, np.float64), "zero", 3)
        full = oracle.iterate(case.field(), case.coef, 3, "zero")
        wins = [((0, 0, 0), (4, 4, 4)), ((10, 11, 12), (14, 15, 16)), ((5, 5, 5), (9, 8, 10))]
    for lo, hi in wins:
        sl = tuple(slice(l, h) for l, h in zip(lo, hi))
        assert np.array_equal(oracle_window(case, lo, hi), full[sl])


# ---- scan (Sec. 3.6) ---------------------------------------------------------------------

@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_scan_matches_exact_rational_prefix_sums(dtype):
    """Prefix sums of short arrays against exact rational arithmetic, rounded once to the type."""
    from fractions import Fraction
    rng = np.random.default_rng(7)
    for n in (1, 2, 3, 17, 50):
        a = rng.uniform(-1.0, 1.0, n).astype(dtype)
        got = oracle.scan(a)
        run = Fraction(0)
        for i in range(n):
            run += Fraction(float(a[i]))
            want = dtype(float(run)) if dtype == np.float64 else np.float32(float(run))
            assert abs(float(got[i]) - float(want)) <= (0.0 if dtype == np.float32 else 2.3e-16 * max(1.0, abs(float(want)))), (n, i)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_scan_closed_forms_and_edges(dtype):
    assert oracle.scan(np.zeros(0, dtype=dtype)).shape == (0,)
    assert np.array_equal(oracle.scan(np.array([2.5], dtype=dtype)), np.array([2.5], dtype=dtype))
    n = 4000
    assert np.array_equal(oracle.scan(np.ones(n, dtype=dtype)), np.arange(1, n + 1).astype(dtype))
    ramp = np.arange(1, n + 1).astype(dtype)                      # 1 + 2 + ... + i = i (i + 1) / 2, exact here
    assert np.array_equal(oracle.scan(ramp), (np.arange(1, n + 1) * np.arange(2, n + 2) // 2).astype(dtype))
    alt = np.where(np.arange(n) % 2 == 0, 1.0, -1.0).astype(dtype)
    assert np.array_equal(oracle.scan(alt), (np.arange(n) % 2 == 0).astype(dtype))
    # a sign error or an exclusive scan would break this one: last prefix is the total, first is a_0
    a = wl.uniform_field((1000,), -1.0, 1.0, 77, dtype)
    got = oracle.scan(a)
    assert got[0] == a[0]
    assert abs(float(got[-1]) - math.fsum(float(v) for v in a)) <= (1e-5 if dtype == np.float32 else 1e-13)
    # differences of consecutive prefixes give the input back (to rounding)
    back = np.diff(np.concatenate([[0.0], got.astype(np.float64)]))
    assert np.max(np.abs(back - a.astype(np.float64))) <= (1e-5 if dtype == np.float32 else 1e-13)


def test_scan_fp32_is_sequential_double_accumulation():
    a = wl.uniform_field((100000,), 0.0, 1.0, 78, np.float32)
    assert np.array_equal(oracle.scan(a), np.cumsum(a.astype(np.float64)).astype(np.float32))
