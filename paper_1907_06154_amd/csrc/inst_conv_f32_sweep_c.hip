// Compiled instances: square filters of the 2x2 .. 20x20 sweep (Sec. 6.2), 13, 14.
#include "ssam_kernel2d.h"

// Default: products on the matrix cores (faster from 7x7 on); variant 5: on the vector unit.

SSAM_INSTANCE_2D_MFMA(4, 13, 13, 6, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 13, 13, 6, 2, 1, 2, 5);
SSAM_INSTANCE_2D_MFMA(4, 14, 14, 7, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 14, 14, 7, 2, 1, 2, 5);
