"""Seeded synthetic inputs for the structured-grid workloads of the paper's evaluation.

This module only *generates data*: grids, filters and stencil coefficient boxes with the
sizes, precisions and shapes of the paper's experiments (Sec. 6.2: 8192x8192 images and
filters from 2x2 to 20x20; Sec. 6.3 / Table 3: 2D stencils on 8192^2 and 3D stencils on
512^3, single and double precision).  It holds none of the method's arithmetic, and it is
the one module that both the HIP path's tests/bench and the CPU oracle's tests read, so
that both sides see identical bits.

Random numbers are a counter-based hash: element i of stream `seed` is
splitmix64(seed * 2**40 + i); the top 53 bits give u in [0, 1), mapped affinely to
[lo, hi) in float64 and then cast to the working type.  Any element can therefore be
regenerated on its own (the full-size parity tests rely on that for cropped windows).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Iterable, List, Optional, Tuple

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_MUL1 = np.uint64(0xBF58476D1CE4E5B9)
_MUL2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def splitmix64(x: np.ndarray) -> np.ndarray:
    """The splitmix64 output function applied elementwise to uint64 counters."""
    with np.errstate(over="ignore"):
        z = x.astype(np.uint64) + _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _MUL1
        z = (z ^ (z >> np.uint64(27))) * _MUL2
        z = z ^ (z >> np.uint64(31))
    return z


def _unit_from_counters(counters: np.ndarray) -> np.ndarray:
    bits = splitmix64(counters) >> np.uint64(11)
    return bits.astype(np.float64) * (1.0 / 9007199254740992.0)


def uniform_at(flat_index: np.ndarray, lo: float, hi: float, seed: int, dtype) -> np.ndarray:
    """Values of stream `seed` at arbitrary flat indices (any shape), cast to `dtype`."""
    idx = np.asarray(flat_index, dtype=np.uint64)
    with np.errstate(over="ignore"):
        counters = idx + (np.uint64(seed) << np.uint64(40))
    u = _unit_from_counters(counters)
    return (lo + (hi - lo) * u).astype(dtype)


def uniform_field(shape: Tuple[int, ...], lo: float, hi: float, seed: int, dtype) -> np.ndarray:
    """Dense row-major field (x fastest) of i.i.d. uniform[lo, hi) values from `seed`."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=dtype)
    for start in range(0, n, _CHUNK):
        stop = min(n, start + _CHUNK)
        out[start:stop] = uniform_at(np.arange(start, stop, dtype=np.uint64), lo, hi, seed, dtype)
    return out.reshape(shape)


def uniform_field_on(device, shape: Tuple[int, ...], lo: float, hi: float, seed: int, dtype):
    """uniform_field(...) computed on a torch device: the same counters, the same integer hash in
    two's-complement int64 arithmetic and the same float64 mapping, so the bits are identical.  For
    grids too large to generate on the host in reasonable time.  Returns a torch tensor."""
    import torch
    n = int(np.prod(shape))
    tdt = {np.dtype(np.float32): torch.float32, np.dtype(np.float64): torch.float64}[np.dtype(dtype)]
    out = torch.empty(n, dtype=tdt, device=device)

    def i64(v: int) -> int:   # the uint64 constant as the int64 with the same bits
        return v - (1 << 64) if v >= (1 << 63) else v

    def lsr(z, k: int):       # logical shift right of int64 bit patterns
        return (z >> k) & ((1 << (64 - k)) - 1)

    chunk = 1 << 26
    for start in range(0, n, chunk):
        stop = min(n, start + chunk)
        z = torch.arange(start, stop, dtype=torch.int64, device=device) + i64(((seed << 40) + int(_GOLDEN)) % (1 << 64))
        z = (z ^ lsr(z, 30)) * i64(int(_MUL1))
        z = (z ^ lsr(z, 27)) * i64(int(_MUL2))
        z = z ^ lsr(z, 31)
        u = lsr(z, 11).to(torch.float64) * (1.0 / 9007199254740992.0)
        u = u * (hi - lo)      # two rounded operations, as in uniform_at (no fused multiply-add)
        u = u + lo
        out[start:stop] = u.to(tdt)
    return out.reshape(shape)


def uniform_window(full_shape: Tuple[int, ...], lo_corner: Tuple[int, ...], win_shape: Tuple[int, ...],
                   lo: float, hi: float, seed: int, dtype) -> np.ndarray:
    """The sub-block [lo_corner, lo_corner + win_shape) of uniform_field(full_shape, ...)."""
    grids = np.meshgrid(*[np.arange(c, c + s, dtype=np.uint64) for c, s in zip(lo_corner, win_shape)],
                        indexing="ij")
    flat = np.zeros(win_shape, dtype=np.uint64)
    for axis, g in enumerate(grids):
        flat = flat * np.uint64(full_shape[axis]) + g
    return uniform_at(flat, lo, hi, seed, dtype)


# ----------------------------------------------------------------------------------------
# Stencil shapes: a stencil is a dense coefficient box of (2rz+1) x (2ry+1) x (2rx+1)
# values indexed [dz+rz][dy+ry][dx+rx]; an exact zero means "no tap at that offset".
# ----------------------------------------------------------------------------------------

def mask_box(rx: int, ry: int, rz: int = 0) -> np.ndarray:
    return np.ones((2 * rz + 1, 2 * ry + 1, 2 * rx + 1), dtype=bool)


def mask_star(rx: int, ry: int, rz: int = 0) -> np.ndarray:
    """Taps on the coordinate axes only (the 5-point / 7-point diffusion shapes of Sec. 2.2)."""
    m = np.zeros((2 * rz + 1, 2 * ry + 1, 2 * rx + 1), dtype=bool)
    m[rz, ry, :] = True
    m[rz, :, rx] = True
    m[:, ry, rx] = True
    return m


def mask_faces_edges() -> np.ndarray:
    """19-point shape: the 3x3x3 box without its 8 corners (Table 3's "poisson" tap count)."""
    m = np.ones((3, 3, 3), dtype=bool)
    for dz in (0, 2):
        for dy in (0, 2):
            for dx in (0, 2):
                m[dz, dy, dx] = False
    return m


def seeded_coefficients(mask: np.ndarray, seed: int, dtype, lo: float = 0.0, hi: float = 1.0,
                        normalise: bool = True) -> np.ndarray:
    """One uniform[lo, hi) value per tap of `mask` (box index order), optionally scaled to sum 1.

    A tap that draws exactly 0 would vanish from the shape, so draws are nudged off zero.
    """
    u = uniform_at(np.arange(mask.size, dtype=np.uint64), lo, hi, seed, np.float64).reshape(mask.shape)
    u = np.where(u == 0.0, 0.5 * (lo + hi) if (lo + hi) != 0 else 0.5, u)
    c = np.where(mask, u, 0.0)
    if normalise:
        c = c / c.sum()
    c = c.astype(dtype)
    assert np.all((c != 0) == mask), "a tap rounded to zero"
    return c


def seeded_symmetric_star(r: int, dims: int, seed: int, dtype) -> np.ndarray:
    """Star of radius r whose coefficient depends on (axis, |distance|) only, scaled to sum 1."""
    rz = r if dims == 3 else 0
    vals = uniform_at(np.arange(1 + dims * r, dtype=np.uint64), 0.0, 1.0, seed, np.float64)
    vals = np.where(vals == 0.0, 0.5, vals)
    c = np.zeros((2 * rz + 1, 2 * r + 1, 2 * r + 1), dtype=np.float64)
    c[rz, r, r] = vals[0]
    for d in range(1, r + 1):
        c[rz, r, r - d] = c[rz, r, r + d] = vals[1 + (d - 1)]
        c[rz, r - d, r] = c[rz, r + d, r] = vals[1 + r + (d - 1)]
        if dims == 3:
            c[rz - d, r, r] = c[rz + d, r, r] = vals[1 + 2 * r + (d - 1)]
    c = c / c.sum()
    return c.astype(dtype)


def seeded_filter(M: int, N: int, seed: int, dtype, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    """Dense filter of width M and height N, stored [n][m] (row n, column m)."""
    return uniform_at(np.arange(M * N, dtype=np.uint64), lo, hi, seed, dtype).reshape(N, M)


# ----------------------------------------------------------------------------------------
# Workload catalogue: the five benchmark configurations.
# ----------------------------------------------------------------------------------------

@dataclass
class Case:
    """One (grid, coefficients, boundary, steps) problem instance."""
    name: str
    kind: str                 # "conv2d" | "conv3d" | "stencil2d" | "stencil3d"
    dtype: type
    shape: Tuple[int, ...]    # (H, W) or (D, H, W)
    field_range: Tuple[float, float]
    field_seed: int
    coef: np.ndarray          # conv2d: [N][M]; conv3d: [K][N][M]; stencils: [2rz+1][2ry+1][2rx+1]
    boundary: str             # "zero" | "clamp"
    steps: int
    paper_analogue: str = ""

    @property
    def points(self) -> int:
        return int(np.prod(self.shape))

    @property
    def taps(self) -> int:
        return int(np.count_nonzero(self.coef))

    def field(self) -> np.ndarray:
        return uniform_field(self.shape, self.field_range[0], self.field_range[1], self.field_seed, self.dtype)

    def window(self, lo_corner, win_shape) -> np.ndarray:
        return uniform_window(self.shape, lo_corner, win_shape, self.field_range[0], self.field_range[1],
                              self.field_seed, self.dtype)


CONV_SHAPES = [(3, 3), (5, 5), (9, 9), (15, 15), (20, 20), (3, 11), (11, 3)]   # (M width, N height)


def config1(n: int = 512) -> List[Case]:
    c = seeded_coefficients(mask_star(1, 1), 2, np.float32, 0.0, 0.25, normalise=False)
    return [Case("c1_2d5pt_f32", "stencil2d", np.float32, (n, n), (-1.0, 1.0), 1, c, "zero", 1,
                 "Listing 2 / Table 3 2d5pt")]


def config2(n: int = 8192, shapes: Optional[Iterable[Tuple[int, int]]] = None) -> List[Case]:
    out = []
    for (M, N) in (list(shapes) if shapes is not None else CONV_SHAPES):
        k = CONV_SHAPES.index((M, N)) if (M, N) in CONV_SHAPES else 100 + 32 * M + N
        f = seeded_filter(M, N, 4 + k, np.float32)
        out.append(Case(f"c2_conv{M}x{N}_f32", "conv2d", np.float32, (n, n), (0.0, 1.0), 3, f, "clamp", 1,
                        "Fig. 4 filter sweep on 8192^2"))
    return out


def config3(n: int = 8192, steps: int = 100) -> List[Case]:
    specs = [("box_r1", mask_box(1, 1), "3x3 box"), ("box_r2", mask_box(2, 2), "Table 3 2d25pt"),
             ("star_r4", mask_star(4, 4), "Table 3 2d17pt")]
    return [Case(f"c3_2d_{nm}_f64", "stencil2d", np.float64, (n, n), (-1.0, 1.0), 5,
                 seeded_coefficients(m, 50 + i, np.float64), "zero", steps, pa)
            for i, (nm, m, pa) in enumerate(specs)]


def config4(n: int = 512, steps: int = 10) -> List[Case]:
    specs = [("star_r1", mask_star(1, 1, 1), "Table 3 3d7pt"), ("box_r1", mask_box(1, 1, 1), "Table 3 3d27pt"),
             ("faces_edges", mask_faces_edges(), "Table 3 poisson (19 taps)")]
    return [Case(f"c4_3d_{nm}_f64", "stencil3d", np.float64, (n, n, n), (-1.0, 1.0), 6,
                 seeded_coefficients(m, 60 + i, np.float64), "zero", steps, pa)
            for i, (nm, m, pa) in enumerate(specs)]


def config5(n: int = 512, steps: int = 20) -> List[Case]:
    return [Case(f"c5_3d_star_r4_{'f32' if dt == np.float32 else 'f64'}", "stencil3d", dt, (n, n, n),
                 (-1.0, 1.0), 7, seeded_symmetric_star(4, 3, 70, dt), "zero", steps,
                 "high-order star, register-pressure case")
            for dt in (np.float32, np.float64)]


def filter_sweep(n: int = 8192) -> List[Case]:
    """The paper's full filter sweep (Sec. 6.2): square filters 2x2 .. 20x20 on an n x n fp32 image."""
    out = []
    for m in range(2, 21):
        f = seeded_filter(m, m, 200 + m, np.float32)
        out.append(Case(f"fs_conv{m}x{m}_f32", "conv2d", np.float32, (n, n), (0.0, 1.0), 3, f, "clamp", 1,
                        "Fig. 4 filter sweep on 8192^2"))
    return out


def table3(n2: int = 8192, n3: int = 512, steps: int = 10, dtypes=(np.float32, np.float64)) -> List[Case]:
    """The stencil shapes of Table 3: 2D stars of order 1..6, 2D boxes of order 2, 4, 5, 3D stars of order
    1, 2, 3D boxes of order 1, 2 and the 19-point shape, in both precisions, `steps` sweeps with seeded
    coefficients of sum 1; and `2d64pt`, the one shape no radius describes: an 8x8 box, run as one pass of
    a dense 8x8 filter (anchor (4, 4), zero padding) with coefficients of sum 1."""
    specs2 = [("2d5pt", mask_star(1, 1)), ("2d9pt", mask_star(2, 2)), ("2d13pt", mask_star(3, 3)),
              ("2d17pt", mask_star(4, 4)), ("2d21pt", mask_star(5, 5)), ("2ds25pt", mask_star(6, 6)),
              ("2d25pt", mask_box(2, 2)), ("2d81pt", mask_box(4, 4)), ("2d121pt", mask_box(5, 5))]
    specs3 = [("3d7pt", mask_star(1, 1, 1)), ("3d13pt", mask_star(2, 2, 2)), ("3d27pt", mask_box(1, 1, 1)),
              ("3d125pt", mask_box(2, 2, 2)), ("poisson", mask_faces_edges())]
    out = []
    for dt in dtypes:
        tag = "f32" if dt == np.float32 else "f64"
        for i, (nm, m) in enumerate(specs2):
            out.append(Case(f"t3_{nm}_{tag}", "stencil2d", dt, (n2, n2), (-1.0, 1.0), 5,
                            seeded_coefficients(m, 300 + i, dt), "zero", steps, f"Table 3 {nm}"))
        f64pt = seeded_filter(8, 8, 340, np.float64, 0.0, 1.0)
        out.append(Case(f"t3_2d64pt_{tag}", "conv2d", dt, (n2, n2), (-1.0, 1.0), 5, (f64pt / f64pt.sum()).astype(dt),
                        "zero", 1, "Table 3 2d64pt"))
        for i, (nm, m) in enumerate(specs3):
            out.append(Case(f"t3_{nm}_{tag}", "stencil3d", dt, (n3, n3, n3), (-1.0, 1.0), 6,
                            seeded_coefficients(m, 320 + i, dt), "zero", steps, f"Table 3 {nm}"))
    return out


def conv3d_filters(n: int = 512) -> List[Case]:
    """Dense 3D filters (the mapping the paper names as its next one, Sec. 6 opening paragraph and Sec. 8) on an
    n^3 volume, clamp, one pass: the cubes 3^3, 5^3 and 7^3 in fp32, 3^3 in fp64, and two shapes that are not
    cubes of odd extent (4x4x4, centre anchor 2; 5x3x2 = M x N x K), which run inside the smallest cube that holds them."""
    out = []
    for i, (M, N, K, dt) in enumerate([(3, 3, 3, np.float32), (5, 5, 5, np.float32), (7, 7, 7, np.float32),
                                       (4, 4, 4, np.float32), (5, 3, 2, np.float32), (3, 3, 3, np.float64)]):
        tag = "f32" if dt == np.float32 else "f64"
        filt = uniform_field((K, N, M), -1.0, 1.0, 400 + i, dt)
        out.append(Case(f"c3d_conv{M}x{N}x{K}_{tag}", "conv3d", dt, (n, n, n), (0.0, 1.0), 8, filt, "clamp", 1,
                        "3D convolution (Sec. 8, future work)"))
    return out


def all_configs() -> Dict[str, List[Case]]:
    return {"config1": config1(), "config2": config2(), "config3": config3(),
            "config4": config4(), "config5": config5(), "filter_sweep": filter_sweep(), "table3": table3(),
            "conv3d": conv3d_filters()}
