// Compiled register-cache instances: one-dimensional fp32 filters (a row or a column of 3 .. 15 taps),
// the separable-filter passes: inst_conv_f32_1d.hip
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 3, 1, 1, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 1, 3, 0, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 5, 1, 2, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 1, 5, 0, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 7, 1, 3, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 1, 7, 0, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 9, 1, 4, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 1, 9, 0, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 11, 1, 5, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 1, 11, 0, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 13, 1, 6, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 1, 13, 0, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 15, 1, 7, 2);
SSAM_INSTANCE_2D(float, SSAM_F32, 4, 8, 1, 15, 0, 2);
