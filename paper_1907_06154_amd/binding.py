"""Thin ctypes binding of libssam.so: argument marshalling only.

Every step of the computation runs in the HIP kernels behind the C ABI (include/ssam.h).
torch is used for device memory and streams.  There is no CPU fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SSAM_LIB_PATH") or os.path.join(_HERE, "libssam.so")   # override: A/B builds
_lib: Optional[ctypes.CDLL] = None

SSAM_F32, SSAM_F64 = 0, 1
SSAM_BOUNDARY_ZERO, SSAM_BOUNDARY_CLAMP = 0, 1
BOUNDARY = {"zero": SSAM_BOUNDARY_ZERO, "clamp": SSAM_BOUNDARY_CLAMP}
EXPORTS = ["ssam_conv2d", "ssam_conv3d", "ssam_stencil2d", "ssam_stencil3d", "ssam_stencil_iterate",
           "ssam_status_string", "ssam_set_tuning", "ssam_describe", "ssam_probe_copy", "ssam_probe_latency",
           "ssam_scan", "ssam_scan_workspace_bytes", "ssam_scan_static"]


class SsamError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib() -> ctypes.CDLL:
    """Loads libssam.so (built by paper_1907_06154_amd.build); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_1907_06154_amd.build` "
                "(there is no fallback implementation)")
        # A process can drive the GPU through ONE HIP runtime.  torch brings its own copy; if this library
        # were loaded first it would bind to the system's copy, and whichever of the two initialises second
        # finds no device (every launch then returns SSAM_ERR_HIP).  Loading torch first makes both share torch's.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        L.ssam_conv2d.argtypes = [vp, vp, ci, ci, vp, ci, ci, ci, ci, ci, ci, vp]
        L.ssam_conv3d.argtypes = [vp, vp, ci, ci, ci, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp]
        L.ssam_stencil2d.argtypes = [vp, vp, ci, ci, vp, ci, ci, ci, ci, vp]
        L.ssam_stencil3d.argtypes = [vp, vp, ci, ci, ci, vp, ci, ci, ci, ci, ci, vp]
        L.ssam_stencil_iterate.argtypes = [vp, vp, ci, ci, ci, vp, ci, ci, ci, ci, ci, ci, vp,
                                           ctypes.POINTER(vp)]
        L.ssam_status_string.argtypes = [ci]
        L.ssam_status_string.restype = ctypes.c_char_p
        L.ssam_set_tuning.argtypes = [ctypes.c_char_p, ci]
        L.ssam_describe.argtypes = [ci, ci, ci, ci, vp, ci, ci, ci, ci, ci, ctypes.c_char_p, ci]
        L.ssam_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.ssam_probe_latency.argtypes = [ci, ci, ci, ci, vp, ctypes.c_size_t, vp, vp]
        L.ssam_probe_latency.restype = ci
        L.ssam_scan.argtypes = [vp, vp, ctypes.c_longlong, ci, vp, ctypes.c_size_t, vp]
        L.ssam_scan_workspace_bytes.argtypes = [ctypes.c_longlong, ci]
        L.ssam_scan_static.argtypes = [vp, vp, ctypes.c_longlong, ci, vp]
        for name in EXPORTS:
            if name not in ("ssam_status_string", "ssam_scan_workspace_bytes"):
                getattr(L, name).restype = ci
        L.ssam_scan_workspace_bytes.restype = ctypes.c_size_t
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().ssam_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise SsamError(status, where)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return SSAM_F32
    if t.dtype == torch.float64:
        return SSAM_F64
    raise TypeError(f"unsupported dtype {t.dtype}")


def _np_dtype(code: int):
    return np.float32 if code == SSAM_F32 else np.float64


def _device_tensor(t, name: str):
    if not t.is_cuda:
        raise ValueError(f"{name} must live in GPU memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous (dense row-major, x fastest)")
    return t


def _stream_ptr(stream) -> ctypes.c_void_p:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _host_coef(coef, code: int) -> np.ndarray:
    if hasattr(coef, "detach"):
        coef = coef.detach().cpu().numpy()
    return np.ascontiguousarray(coef, dtype=_np_dtype(code))


def ssam_conv2d(d_in, filt, boundary: str = "clamp", anchor: Optional[Tuple[int, int]] = None,
                d_out=None, stream=None):
    """out[y][x] = sum_{n,m} filt[n][m] * IN(x+m-ax, y+n-ay).  d_in: [H][W] GPU tensor; filt: host [N][M]."""
    import torch
    _device_tensor(d_in, "d_in")
    H, W = d_in.shape
    code = _dtype_code(d_in)
    f = _host_coef(filt, code)
    N, M = f.shape
    ax, ay = (-1, -1) if anchor is None else anchor
    if d_out is None:
        d_out = torch.empty_like(d_in)
    _device_tensor(d_out, "d_out")
    st = lib().ssam_conv2d(d_in.data_ptr(), d_out.data_ptr(), W, H, f.ctypes.data, M, N, ax, ay,
                           BOUNDARY[boundary], code, _stream_ptr(stream))
    _check(st, "ssam_conv2d")
    return d_out


def ssam_conv3d(d_in, filt, boundary: str = "clamp", anchor: Optional[Tuple[int, int, int]] = None,
                d_out=None, stream=None):
    """out[z][y][x] = sum_{k,n,m} filt[k][n][m] * IN(x+m-ax, y+n-ay, z+k-az).  d_in: [D][H][W] GPU tensor;
    filt: host [K][N][M]; anchor (ax, ay, az), default the centre (size // 2 per axis)."""
    import torch
    _device_tensor(d_in, "d_in")
    D, H, W = d_in.shape
    code = _dtype_code(d_in)
    f = _host_coef(filt, code)
    K, N, M = f.shape
    ax, ay, az = (-1, -1, -1) if anchor is None else anchor
    if d_out is None:
        d_out = torch.empty_like(d_in)
    _device_tensor(d_out, "d_out")
    st = lib().ssam_conv3d(d_in.data_ptr(), d_out.data_ptr(), W, H, D, f.ctypes.data, M, N, K, ax, ay, az,
                           BOUNDARY[boundary], code, _stream_ptr(stream))
    _check(st, "ssam_conv3d")
    return d_out


def _radii(c: np.ndarray, dims: int) -> Tuple[int, int, int]:
    if c.ndim != dims:
        raise ValueError(f"coefficient box must have {dims} dimensions")
    if any(s % 2 == 0 for s in c.shape):
        raise ValueError("coefficient box extents must be odd (2r+1 per axis)")
    if dims == 2:
        return c.shape[1] // 2, c.shape[0] // 2, 0
    return c.shape[2] // 2, c.shape[1] // 2, c.shape[0] // 2


def ssam_stencil2d(d_in, coef, boundary: str = "zero", d_out=None, stream=None):
    """One sweep; d_in [H][W] GPU tensor; coef host [2ry+1][2rx+1] (exact zero = no tap)."""
    import torch
    _device_tensor(d_in, "d_in")
    H, W = d_in.shape
    code = _dtype_code(d_in)
    c = _host_coef(coef, code)
    rx, ry, _ = _radii(c, 2)
    if d_out is None:
        d_out = torch.empty_like(d_in)
    _device_tensor(d_out, "d_out")
    st = lib().ssam_stencil2d(d_in.data_ptr(), d_out.data_ptr(), W, H, c.ctypes.data, rx, ry,
                              BOUNDARY[boundary], code, _stream_ptr(stream))
    _check(st, "ssam_stencil2d")
    return d_out


def ssam_stencil3d(d_in, coef, boundary: str = "zero", d_out=None, stream=None):
    """One sweep; d_in [D][H][W] GPU tensor; coef host [2rz+1][2ry+1][2rx+1]."""
    import torch
    _device_tensor(d_in, "d_in")
    D, H, W = d_in.shape
    code = _dtype_code(d_in)
    c = _host_coef(coef, code)
    rx, ry, rz = _radii(c, 3)
    if d_out is None:
        d_out = torch.empty_like(d_in)
    _device_tensor(d_out, "d_out")
    st = lib().ssam_stencil3d(d_in.data_ptr(), d_out.data_ptr(), W, H, D, c.ctypes.data, rx, ry, rz,
                              BOUNDARY[boundary], code, _stream_ptr(stream))
    _check(st, "ssam_stencil3d")
    return d_out


def ssam_stencil_iterate(d_a, d_b, coef, steps: int, boundary: str = "zero", stream=None):
    """`steps` Jacobi sweeps ping-ponging d_a -> d_b -> d_a ...; returns the tensor (d_a or d_b)
    that holds the final field.  2D fields are [H][W] with a 2D coefficient box."""
    _device_tensor(d_a, "d_a")
    _device_tensor(d_b, "d_b")
    if d_a.shape != d_b.shape or d_a.dtype != d_b.dtype:
        raise ValueError("d_a and d_b must have the same shape and dtype")
    code = _dtype_code(d_a)
    c = _host_coef(coef, code)
    if d_a.dim() == 2:
        (H, W), D = d_a.shape, 1
        rx, ry, rz = _radii(c, 2)
    else:
        D, H, W = d_a.shape
        rx, ry, rz = _radii(c, 3)
    result = ctypes.c_void_p(0)
    st = lib().ssam_stencil_iterate(d_a.data_ptr(), d_b.data_ptr(), W, H, D, c.ctypes.data, rx, ry, rz,
                                    BOUNDARY[boundary], code, int(steps), _stream_ptr(stream),
                                    ctypes.byref(result))
    _check(st, "ssam_stencil_iterate")
    return d_a if result.value == d_a.data_ptr() else d_b


def ssam_set_tuning(name: str, value: int) -> None:
    _check(lib().ssam_set_tuning(name.encode(), int(value)), "ssam_set_tuning")


def ssam_describe(kind: str, shape, coef, boundary: str = "zero", remaining: int = 0) -> str:
    """Kernel instance and tile geometry the dispatcher picks (host only, nothing is launched).
    kind: "conv2d" (coef [N][M]), "stencil2d", "iterate2d", "stencil3d" or "iterate3d" (coefficient box); shape (H, W) or (D, H, W)."""
    coef = np.ascontiguousarray(coef)
    code = SSAM_F32 if coef.dtype == np.float32 else SSAM_F64
    buf = ctypes.create_string_buffer(512)
    if kind == "conv2d":
        H, W = shape
        N, M = coef.shape
        st = lib().ssam_describe(0, W, H, 1, coef.ctypes.data, M, N, 0, BOUNDARY[boundary], code, buf, 512)
    elif kind == "stencil2d":
        H, W = shape
        rx, ry, _ = _radii(coef, 2)
        st = lib().ssam_describe(1, W, H, 1, coef.ctypes.data, rx, ry, 0, BOUNDARY[boundary], code, buf, 512)
    elif kind == "iterate2d":   # the launch ssam_stencil_iterate issues while `remaining` sweeps are left (0: many)
        H, W = shape
        rx, ry, _ = _radii(coef, 2)
        st = lib().ssam_describe(3, W, H, 1, coef.ctypes.data, rx, ry, int(remaining), BOUNDARY[boundary], code, buf, 512)
    elif kind == "iterate3d":   # the launch ssam_stencil_iterate issues on a 3D grid while >= 2 sweeps are left
        D, H, W = shape
        rx, ry, rz = _radii(coef, 3)
        st = lib().ssam_describe(4, W, H, D, coef.ctypes.data, rx, ry, rz, BOUNDARY[boundary], code, buf, 512)
    elif kind == "stencil3d":
        D, H, W = shape
        rx, ry, rz = _radii(coef, 3)
        st = lib().ssam_describe(2, W, H, D, coef.ctypes.data, rx, ry, rz, BOUNDARY[boundary], code, buf, 512)
    elif kind == "conv3d":
        D, H, W = shape
        K, N, M = coef.shape
        st = lib().ssam_describe(5, W, H, D, coef.ctypes.data, M, N, K, BOUNDARY[boundary], code, buf, 512)
    else:
        raise ValueError(kind)
    _check(st, "ssam_describe")
    return buf.value.decode()


def ssam_scan_workspace_bytes(n: int, dtype) -> int:
    """Workspace size ssam_scan needs for n elements (dtype: a torch or numpy float32/float64)."""
    code = SSAM_F32 if "32" in str(dtype) else SSAM_F64 if "64" in str(dtype) else -1
    return int(lib().ssam_scan_workspace_bytes(int(n), code))


def ssam_scan(d_in, d_out=None, d_work=None, stream=None):
    """Inclusive prefix sums of a 1D device tensor.  d_out: result tensor (default: a new one;
    passing d_in itself scans in place).  d_work: a byte workspace tensor of at least
    ssam_scan_workspace_bytes(n, dtype) bytes (default: a new one)."""
    import torch
    _device_tensor(d_in, "d_in")
    if d_in.dim() != 1:
        raise ValueError("ssam_scan takes a 1D tensor")
    code = _dtype_code(d_in)
    if d_out is None:
        d_out = torch.empty_like(d_in)
    _device_tensor(d_out, "d_out")
    if d_out.shape != d_in.shape or d_out.dtype != d_in.dtype:
        raise ValueError("d_out must match d_in in shape and dtype")
    n = d_in.numel()
    need = int(lib().ssam_scan_workspace_bytes(n, code))
    if d_work is None and need:
        d_work = torch.empty(need, dtype=torch.uint8, device=d_in.device)
        if stream is not None:
            # the workspace dies when this function returns while the kernels that use it are still
            # queued on `stream`: tell the caching allocator, or it may hand the block out again
            d_work.record_stream(stream)
    wp, wb = (d_work.data_ptr(), d_work.numel() * d_work.element_size()) if d_work is not None else (None, 0)
    _check(lib().ssam_scan(d_in.data_ptr() if n else None, d_out.data_ptr() if n else None, n, code,
                           wp, wb, _stream_ptr(stream)), "ssam_scan")
    return d_out


def ssam_scan_static(d_in, d_out, stream=None):
    """ssam_scan with the workspace held by the library (no allocation in the call): both tensors
    are the caller's."""
    _device_tensor(d_in, "d_in")
    _device_tensor(d_out, "d_out")
    if d_in.dim() != 1 or d_out.shape != d_in.shape or d_out.dtype != d_in.dtype:
        raise ValueError("ssam_scan_static takes two 1D tensors of the same shape and dtype")
    n = d_in.numel()
    _check(lib().ssam_scan_static(d_in.data_ptr() if n else None, d_out.data_ptr() if n else None, n,
                                  _dtype_code(d_in), _stream_ptr(stream)), "ssam_scan_static")
    return d_out


def ssam_probe_copy(d_in, d_out, stream=None):
    """Plain device copy of d_in into d_out (same size, contiguous): the 1R+1W bandwidth ceiling."""
    _device_tensor(d_in, "d_in")
    _device_tensor(d_out, "d_out")
    nbytes = d_in.numel() * d_in.element_size()
    if nbytes != d_out.numel() * d_out.element_size():
        raise ValueError("d_in and d_out must have the same size in bytes")
    _check(lib().ssam_probe_copy(d_in.data_ptr(), d_out.data_ptr(), nbytes, _stream_ptr(stream)), "ssam_probe_copy")
    return d_out


PROBE_OPS = ["fma_f32", "fma_f64", "add_f32", "dpp_wave_shr", "dpp_row_shr", "ds_swizzle", "ds_bpermute",
             "lds_read", "load_l1", "load_l2", "shift_f64"]
PROBE_SCRATCH_BYTES = 2 << 20


def ssam_probe_latency(op: str, ilp: int = 1, waves: int = 1, chain: int = 1 << 15, d_scratch=None, stream=None):
    """Cycles (shader clock) and nanoseconds per operation of one dependent chain of `op`
    (a name from PROBE_OPS); synchronises the stream.  d_scratch: a device tensor of at least
    PROBE_SCRATCH_BYTES bytes (allocated here when omitted)."""
    import torch
    if d_scratch is None:
        d_scratch = torch.empty(PROBE_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
    _device_tensor(d_scratch, "d_scratch")
    res = (ctypes.c_double * 2)()
    st = lib().ssam_probe_latency(PROBE_OPS.index(op), int(ilp), int(waves), int(chain), d_scratch.data_ptr(),
                                  d_scratch.numel() * d_scratch.element_size(), res, _stream_ptr(stream))
    _check(st, "ssam_probe_latency")
    return float(res[0]), float(res[1])
