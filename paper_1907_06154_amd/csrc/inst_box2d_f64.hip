// Compiled register-cache instances: inst_box2d_f64.hip
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D(double, SSAM_F64, 2, 8, 3, 3, 1, 2);
SSAM_INSTANCE_2D(double, SSAM_F64, 2, 8, 5, 5, 2, 2);
