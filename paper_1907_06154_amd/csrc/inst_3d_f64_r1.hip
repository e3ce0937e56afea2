// Compiled register-cache instances: inst_3d_f64_r1.hip
#include "ssam_kernel3d.h"

SSAM_INSTANCE_3D(double, SSAM_F64, 2, 4, 1, 1, 1, 1);
SSAM_INSTANCE_3D(double, SSAM_F64, 2, 4, 1, 1, 1, 2);
SSAM_INSTANCE_3D(double, SSAM_F64, 2, 4, 1, 1, 1, 3);
