// Compiled register-cache instances: inst_star2d_f32.hip
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 3, 3, 1, 1);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 5, 5, 2, 1);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 7, 7, 3, 1);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 9, 9, 4, 1);
