// Compiled instances: 25-point star of radius 4 (largest register pressure: nine output planes
// are in flight per lane).  Default: the block-cooperative kernel, whose waves share each
// input plane through LDS so that the eight halo rows are fetched once per block, not once
// per wave.  The one-wave-per-tile kernel stays available as variant 1 (single plane buffer
// for fp64: with two buffers the register allocator spills).
#include "ssam_kernel3d_lds.h"

SSAM_INSTANCE_3D_LDS(float, SSAM_F32, 2, 4, 4, 4, 4, 4, 1, 2, 0);
SSAM_INSTANCE_3D_LDS(double, SSAM_F64, 2, 2, 8, 4, 4, 4, 1, 2, 0);
SSAM_INSTANCE_3D_V(float, SSAM_F32, 2, 4, 4, 4, 4, 1, 1, 2, 1);
SSAM_INSTANCE_3D_V(double, SSAM_F64, 2, 4, 4, 4, 4, 1, 0, 2, 1);
