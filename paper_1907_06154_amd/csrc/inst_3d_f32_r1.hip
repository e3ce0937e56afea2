// Compiled register-cache instances: inst_3d_f32_r1.hip
#include "ssam_kernel3d.h"

SSAM_INSTANCE_3D_V(float, SSAM_F32, 4, 4, 1, 1, 1, 1, 1, 2, 4);   // the star: variant 4 (default: inst_3d_star_r12.hip)
SSAM_INSTANCE_3D_V(float, SSAM_F32, 4, 4, 1, 1, 1, 2, 1, 2, 4);
SSAM_INSTANCE_3D_V(float, SSAM_F32, 4, 4, 1, 1, 1, 3, 1, 2, 4);
