// Compiled register-cache instances: inst_conv_f32_9.hip
#include "ssam_kernel2d.h"

// Default: products on the matrix cores (faster from 7x7 on); variant 5: on the vector unit.

SSAM_INSTANCE_2D_MFMA(4, 9, 9, 4, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 9, 9, 4, 2, 0, 2, 5);
