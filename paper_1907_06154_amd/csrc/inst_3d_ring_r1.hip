// Compiled instances: radius-1 3D stencils with taps off the axes (19-point faces and edges, 27-point
// box) on the block-cooperative kernel (ssam_kernel3d_star.h), four rows per wave, eight waves per
// block; variant 10: two rows per wave.  Fallbacks: the one-wave-per-tile instances (variant 4).
#include "ssam_kernel3d_star.h"

SSAM_INSTANCE_3D_RING(double, SSAM_F64, 4, 8, 1, 2, 3, 2, (::ssam::launch3d<double, 2, 4, 1, 1, 1, 2, 2, false>), 0);
SSAM_INSTANCE_3D_RING(double, SSAM_F64, 4, 8, 1, 3, 3, 2, (::ssam::launch3d<double, 2, 4, 1, 1, 1, 3, 2, false>), 0);
SSAM_INSTANCE_3D_RING(float, SSAM_F32, 4, 8, 1, 2, 3, 2, (::ssam::launch3d<float, 4, 4, 1, 1, 1, 2, 2, true>), 0);
SSAM_INSTANCE_3D_RING(float, SSAM_F32, 4, 8, 1, 3, 3, 2, (::ssam::launch3d<float, 4, 4, 1, 1, 1, 3, 2, true>), 0);
SSAM_INSTANCE_3D_RING(double, SSAM_F64, 2, 8, 1, 2, 3, 2, (::ssam::launch3d<double, 2, 4, 1, 1, 1, 2, 2, false>), 10);
SSAM_INSTANCE_3D_RING(double, SSAM_F64, 2, 8, 1, 3, 3, 2, (::ssam::launch3d<double, 2, 4, 1, 1, 1, 3, 2, false>), 10);
SSAM_INSTANCE_3D_RING(float, SSAM_F32, 2, 8, 1, 2, 3, 2, (::ssam::launch3d<float, 4, 4, 1, 1, 1, 2, 2, true>), 10);
SSAM_INSTANCE_3D_RING(float, SSAM_F32, 2, 8, 1, 3, 3, 2, (::ssam::launch3d<float, 4, 4, 1, 1, 1, 3, 2, true>), 10);
