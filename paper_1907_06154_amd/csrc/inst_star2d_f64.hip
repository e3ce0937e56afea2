// Compiled register-cache instances: inst_star2d_f64.hip
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D(double, SSAM_F64, 2, 8, 3, 3, 1, 1);
SSAM_INSTANCE_2D(double, SSAM_F64, 2, 8, 5, 5, 2, 1);
SSAM_INSTANCE_2D(double, SSAM_F64, 2, 8, 7, 7, 3, 1);
SSAM_INSTANCE_2D(double, SSAM_F64, 2, 8, 9, 9, 4, 1);
