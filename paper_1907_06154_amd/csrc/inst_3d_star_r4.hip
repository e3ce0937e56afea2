// Compiled register-cache instances: inst_3d_star_r4.hip
#include "ssam_kernel3d.h"

SSAM_INSTANCE_3D(float, SSAM_F32, 4, 4, 4, 4, 4, 1);
SSAM_INSTANCE_3D(double, SSAM_F64, 2, 4, 4, 4, 4, 1);
