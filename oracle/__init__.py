"""numpy-facing wrapper around the plain-C CPU oracle (ssam_oracle.c).

TEST INFRASTRUCTURE ONLY.  Importable from tests/, from the smoke check and from the
benchmark's cpu_baseline leg; the GPU library and its Python binding never import this.
All arithmetic lives in the C file; this module only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ssam_oracle.c")
_LIB = os.environ.get("SSAM_ORACLE_LIB") or os.path.join(_HERE, "libssam_oracle.so")   # override: a sanitizer build
_lib: Optional[ctypes.CDLL] = None

BOUNDARY = {"zero": 0, "clamp": 1}


def build(force: bool = True, sanitize: Optional[str] = None) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp).  Returns the library path.
    sanitize: path of a second library to build with -fsanitize=address,undefined instead; run the CPU
    tests against it with SSAM_ORACLE_LIB=<path> and gcc's libasan.so / libubsan.so in LD_PRELOAD."""
    if sanitize:
        cmd = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-fsanitize=address,undefined",
               "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", sanitize, _SRC]
        subprocess.run(cmd, check=True, cwd=_HERE)
        return sanitize
    if force or not os.path.exists(_LIB):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build(force=True)
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _suffix(dtype) -> str:
    dt = np.dtype(dtype)
    if dt == np.float32:
        return "f32"
    if dt == np.float64:
        return "f64"
    raise TypeError(f"oracle supports float32/float64, got {dt}")


def _ptr(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def conv2d(image: np.ndarray, filt: np.ndarray, boundary: str = "clamp",
           anchor: Optional[Tuple[int, int]] = None) -> np.ndarray:
    """image [H][W]; filt [N][M]; anchor (ax, ay), default (M//2, N//2)."""
    image = np.ascontiguousarray(image)
    filt = np.ascontiguousarray(filt, dtype=image.dtype)
    H, W = image.shape
    N, M = filt.shape
    ax, ay = (M // 2, N // 2) if anchor is None else anchor
    out = np.empty_like(image)
    fn = getattr(_load(), "oracle_conv2d_" + _suffix(image.dtype))
    rc = fn(_ptr(image), _ptr(out), W, H, _ptr(filt), M, N, int(ax), int(ay), BOUNDARY[boundary])
    if rc != 0:
        raise ValueError("oracle_conv2d rejected its arguments")
    return out


def conv3d(volume: np.ndarray, filt: np.ndarray, boundary: str = "clamp",
           anchor: Optional[Tuple[int, int, int]] = None) -> np.ndarray:
    """volume [D][H][W]; filt [K][N][M]; anchor (ax, ay, az), default (M//2, N//2, K//2)."""
    volume = np.ascontiguousarray(volume)
    filt = np.ascontiguousarray(filt, dtype=volume.dtype)
    D, H, W = volume.shape
    K, N, M = filt.shape
    ax, ay, az = (M // 2, N // 2, K // 2) if anchor is None else anchor
    out = np.empty_like(volume)
    fn = getattr(_load(), "oracle_conv3d_" + _suffix(volume.dtype))
    rc = fn(_ptr(volume), _ptr(out), W, H, D, _ptr(filt), M, N, K, int(ax), int(ay), int(az), BOUNDARY[boundary])
    if rc != 0:
        raise ValueError("oracle_conv3d rejected its arguments")
    return out


def _box_radii(coef: np.ndarray) -> Tuple[int, int, int]:
    if coef.ndim == 2:
        coef = coef[None]
    nz, ny, nx = coef.shape
    if nz % 2 == 0 or ny % 2 == 0 or nx % 2 == 0:
        raise ValueError("coefficient box extents must be odd")
    return nx // 2, ny // 2, nz // 2


def stencil(field: np.ndarray, coef: np.ndarray, boundary: str = "zero") -> np.ndarray:
    """One sweep.  field [H][W] or [D][H][W]; coef [2ry+1][2rx+1] or [2rz+1][2ry+1][2rx+1]."""
    field = np.ascontiguousarray(field)
    coef = np.ascontiguousarray(coef, dtype=field.dtype)
    rx, ry, rz = _box_radii(coef)
    if field.ndim == 2:
        (H, W), D = field.shape, 1
        if rz != 0:
            raise ValueError("3D coefficient box on a 2D field")
    else:
        D, H, W = field.shape
    out = np.empty_like(field)
    fn = getattr(_load(), "oracle_stencil3d_" + _suffix(field.dtype))
    rc = fn(_ptr(field), _ptr(out), W, H, D, _ptr(coef), rx, ry, rz, BOUNDARY[boundary])
    if rc != 0:
        raise ValueError("oracle_stencil3d rejected its arguments")
    return out


def iterate(field: np.ndarray, coef: np.ndarray, steps: int, boundary: str = "zero") -> np.ndarray:
    """`steps` Jacobi sweeps with two buffers; returns the final field (a fresh array)."""
    a = np.array(field, order="C", copy=True)
    b = np.empty_like(a)
    coef = np.ascontiguousarray(coef, dtype=a.dtype)
    rx, ry, rz = _box_radii(coef)
    if a.ndim == 2:
        (H, W), D = a.shape, 1
    else:
        D, H, W = a.shape
    fn = getattr(_load(), "oracle_iterate_" + _suffix(a.dtype))
    which = fn(_ptr(a), _ptr(b), W, H, D, _ptr(coef), rx, ry, rz, BOUNDARY[boundary], int(steps))
    if which < 0:
        raise ValueError("oracle_iterate rejected its arguments")
    return a if which == 0 else b


def scan(values: np.ndarray) -> np.ndarray:
    """Inclusive prefix sums of a 1D array (running total in the accumulation type, each prefix
    rounded to the array's type)."""
    a = np.ascontiguousarray(values)
    if a.ndim != 1:
        raise ValueError("scan takes a 1D array")
    b = np.empty_like(a)
    fn = getattr(_load(), "oracle_scan_" + _suffix(a.dtype))
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_long]
    if fn(_ptr(a) if a.size else None, _ptr(b) if a.size else None, a.size) != 0:
        raise ValueError("oracle_scan rejected its arguments")
    return b
