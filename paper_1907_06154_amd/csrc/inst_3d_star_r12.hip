// Compiled instances: 3D stars of radius 1 (7-point) and 2 (13-point) on the block-cooperative star
// kernel.  Fallbacks (rows that are not a multiple of 16 bytes): the one-wave-per-tile instances of
// the same shapes, registered as variant 4 beside the other radius-1 / radius-2 shapes.
// Default: four rows per wave, eight waves per block (7-point fp64 on 512^3: 351 us against 375 us
// with two rows per wave, which stays as variant 10).
#include "ssam_kernel3d_star.h"

SSAM_INSTANCE_3D_STAR(double, SSAM_F64, 2, 8, 1, 3, 2, (::ssam::launch3d<double, 2, 4, 1, 1, 1, 1, 2, true>), 10);
SSAM_INSTANCE_3D_STAR(float, SSAM_F32, 2, 8, 1, 3, 2, (::ssam::launch3d<float, 4, 4, 1, 1, 1, 1, 2, true>), 10);
SSAM_INSTANCE_3D_STAR(double, SSAM_F64, 2, 8, 2, 3, 2, (::ssam::launch3d<double, 2, 4, 2, 2, 2, 1, 2, true>), 10);
SSAM_INSTANCE_3D_STAR(float, SSAM_F32, 2, 8, 2, 3, 2, (::ssam::launch3d<float, 2, 4, 2, 2, 2, 1, 2, true>), 10);
SSAM_INSTANCE_3D_STAR(double, SSAM_F64, 4, 8, 1, 3, 2, (::ssam::launch3d<double, 2, 4, 1, 1, 1, 1, 2, true>), 0);
SSAM_INSTANCE_3D_STAR(float, SSAM_F32, 4, 8, 1, 3, 2, (::ssam::launch3d<float, 4, 4, 1, 1, 1, 1, 2, true>), 0);
SSAM_INSTANCE_3D_STAR(double, SSAM_F64, 4, 8, 2, 3, 2, (::ssam::launch3d<double, 2, 4, 2, 2, 2, 1, 2, true>), 0);
SSAM_INSTANCE_3D_STAR(float, SSAM_F32, 4, 8, 2, 3, 2, (::ssam::launch3d<float, 2, 4, 2, 2, 2, 1, 2, true>), 0);
