"""MI355X-native software-systolic structured-grid kernels (2D filters, 2D/3D stencils, scan).

The package holds the HIP kernels and C ABI (csrc/, built into libssam.so by build.py) and a
ctypes binding with the same names as the C entry points (binding.py).  Importing the package
loads nothing; the shared library is opened on the first call and a missing library raises.
"""
from .binding import (SsamError, lib, ssam_conv2d, ssam_conv3d, ssam_describe, ssam_probe_copy, ssam_probe_latency, ssam_scan, ssam_scan_static, ssam_scan_workspace_bytes,
                      ssam_set_tuning, ssam_stencil2d,
                      ssam_stencil3d, ssam_stencil_iterate, status_string)

__all__ = ["SsamError", "lib", "ssam_conv2d", "ssam_conv3d", "ssam_stencil2d", "ssam_stencil3d", "ssam_stencil_iterate",
           "ssam_set_tuning", "ssam_describe", "ssam_probe_copy", "ssam_probe_latency", "ssam_scan", "ssam_scan_static", "ssam_scan_workspace_bytes",
           "status_string"]
