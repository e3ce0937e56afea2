// Compiled register-cache instances: inst_conv_f32_20.hip
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D(float, SSAM_F32, 4, 4, 20, 20, 10, 2);
