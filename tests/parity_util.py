"""Helpers shared by the GPU parity tests: error metric and windowed oracle evaluation."""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np

TOL = {np.dtype(np.float32): 1e-5, np.dtype(np.float64): 1e-12}


def normalised_error(got: np.ndarray, want: np.ndarray, coef: np.ndarray, in_max: float) -> float:
    """max |got - want| / (sum|w| * max|in|): the metric the acceptance tolerance is stated in."""
    scale = float(np.abs(coef.astype(np.float64)).sum()) * float(in_max)
    if scale == 0.0:
        scale = 1.0
    return float(np.max(np.abs(got.astype(np.float64) - want.astype(np.float64)))) / scale


def assert_parity(got: np.ndarray, want: np.ndarray, coef: np.ndarray, in_max: float, what: str = "") -> float:
    assert got.shape == want.shape and got.dtype == want.dtype, (what, got.shape, want.shape, got.dtype, want.dtype)
    assert np.all(np.isfinite(got)), f"{what}: non-finite GPU output"
    err = normalised_error(got, want, coef, in_max)
    tol = TOL[np.dtype(got.dtype)]
    assert err <= tol, f"{what}: normalised error {err:.3e} > {tol:.0e}"
    return err


def expanded_window(full_shape: Sequence[int], lo: Sequence[int], hi: Sequence[int],
                    reach_lo: Sequence[int], reach_hi: Sequence[int]) -> Tuple[Tuple[int, ...], Tuple[int, ...]]:
    """Window [lo, hi) grown by the dependency reach on each side and clipped to the grid.

    Evaluating the oracle on the grown crop, with the true boundary rule at the crop's edges,
    gives the true values inside [lo, hi): where the crop was clipped its edge *is* the grid's
    edge, and elsewhere the crop edge lies at least `reach` away, so the wrong values its
    artificial boundary produces cannot arrive."""
    elo = tuple(max(0, l - r) for l, r in zip(lo, reach_lo))
    ehi = tuple(min(n, h + r) for n, h, r in zip(full_shape, hi, reach_hi))
    return elo, ehi


def reach_of(case):
    """Per-axis dependency reach (low side, high side) of the whole run, slowest axis first."""
    if case.kind == "conv2d":
        N, M = case.coef.shape
        ax, ay = M // 2, N // 2
        return (ay, ax), (N - 1 - ay, M - 1 - ax)
    if case.kind == "conv3d":
        lo = tuple(s // 2 for s in case.coef.shape)                 # centre anchor per axis
        return lo, tuple(s - 1 - a for s, a in zip(case.coef.shape, lo))
    r = [s // 2 * case.steps for s in case.coef.shape]
    if case.kind == "stencil2d":
        r = r[1:]
    return tuple(r), tuple(r)


def oracle_window(case, lo, hi):
    rlo, rhi = reach_of(case)
    elo, ehi = expanded_window(case.shape, lo, hi, rlo, rhi)
    crop = case.window(elo, tuple(h - l for l, h in zip(elo, ehi)))
    import oracle
    if case.kind == "conv2d":
        full = oracle.conv2d(crop, case.coef, case.boundary)
    elif case.kind == "conv3d":
        full = oracle.conv3d(crop, case.coef, case.boundary)
    else:
        coef = case.coef if case.kind == "stencil3d" else case.coef[0]
        full = oracle.iterate(crop, coef, case.steps, case.boundary)
    sl = tuple(slice(l - e, h - e) for l, h, e in zip(lo, hi, elo))
    return full[sl]


