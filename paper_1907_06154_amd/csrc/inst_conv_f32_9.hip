// Compiled register-cache instances: inst_conv_f32_9.hip
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 9, 9, 4, 2, 0, 2, 0);
