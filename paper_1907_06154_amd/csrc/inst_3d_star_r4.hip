// Compiled instances: 25-point star of radius 4 (largest register pressure: nine output planes
// are in flight per lane).  Default: the block-cooperative star kernel (ssam_kernel3d_star.h),
// two rows per wave, eight waves per block.  Variant 2: the earlier block-cooperative kernel with
// halo lanes (also the fallback for rows that are not a multiple of 16 bytes); variant 1: the
// one-wave-per-tile kernel (single plane buffer for fp64: with two buffers the register allocator
// spills); variant 10: four rows per wave (fp32; fp64 spills there).
#include "ssam_kernel3d_star.h"

SSAM_INSTANCE_3D_STAR(float, SSAM_F32, 2, 8, 4, 3, 2, (::ssam::launch3d_lds<float, 2, 4, 4, 4, 4, 4, 1, 2>), 0);
SSAM_INSTANCE_3D_STAR(double, SSAM_F64, 2, 8, 4, 3, 2, (::ssam::launch3d_lds<double, 2, 2, 8, 4, 4, 4, 1, 2>), 0);
SSAM_INSTANCE_3D_STAR(float, SSAM_F32, 4, 8, 4, 3, 2, (::ssam::launch3d_lds<float, 2, 4, 4, 4, 4, 4, 1, 2>), 10);
SSAM_INSTANCE_3D_LDS(float, SSAM_F32, 2, 4, 4, 4, 4, 4, 1, 2, 2);
SSAM_INSTANCE_3D_LDS(double, SSAM_F64, 2, 2, 8, 4, 4, 4, 1, 2, 2);
SSAM_INSTANCE_3D_V(float, SSAM_F32, 2, 4, 4, 4, 4, 1, 1, 2, 1);
SSAM_INSTANCE_3D_V(double, SSAM_F64, 2, 4, 4, 4, 4, 1, 0, 2, 1);
