// Compiled register-cache instances: inst_conv_f32_small.hip
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 3, 3, 1, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 5, 5, 2, 2);
// 3 wide, 11 tall: the tall columns suit the matrix cores (+3 %); the vector-unit instance is variant 5
SSAM_INSTANCE_2D_MFMA(4, 3, 11, 1, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 3, 11, 1, 2, 1, 2, 5);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 11, 3, 5, 2);
