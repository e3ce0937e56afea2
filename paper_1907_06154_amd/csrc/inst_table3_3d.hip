// Compiled instances: remaining 3D shapes of Table 3 (13-point star of order 2, 125-point box).
#include "ssam_kernel3d.h"

SSAM_INSTANCE_3D_V(double, SSAM_F64, 2, 4, 2, 2, 2, 1, 1, 2, 4);   // the stars: variant 4 (default: inst_3d_star_r12.hip)
SSAM_INSTANCE_3D_V(float, SSAM_F32, 2, 4, 2, 2, 2, 1, 1, 2, 4);
SSAM_INSTANCE_3D_V(double, SSAM_F64, 2, 2, 2, 2, 2, 3, 0, 2, 4);   // the boxes: variant 4 (default: inst_3d_ring_box23.hip)
SSAM_INSTANCE_3D_V(float, SSAM_F32, 2, 4, 2, 2, 2, 3, 0, 2, 4);
