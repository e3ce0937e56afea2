// Compiled register-cache instances: inst_conv_f32_15.hip
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D(float, SSAM_F32, 4, 4, 15, 15, 7, 2);
