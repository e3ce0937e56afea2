// Compiled register-cache instances: radius-1 3D stencils, fp64 (7-point star, 19-point, 27-point box),
// one wave per tile: variant 4, and the fallback of the block-cooperative defaults (inst_3d_ring_r1.hip,
// inst_3d_star_r12.hip) for rows that are not a multiple of 16 bytes.
#include "ssam_kernel3d.h"

SSAM_INSTANCE_3D_V(double, SSAM_F64, 2, 4, 1, 1, 1, 1, 1, 2, 4);   // the star: variant 4 (default: inst_3d_star_r12.hip)
SSAM_INSTANCE_3D_V(double, SSAM_F64, 2, 4, 1, 1, 1, 2, 0, 2, 4);
SSAM_INSTANCE_3D_V(double, SSAM_F64, 2, 4, 1, 1, 1, 3, 0, 2, 4);
