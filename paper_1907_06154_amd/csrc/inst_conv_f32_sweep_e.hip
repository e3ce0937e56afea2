// Compiled instances: square filters of the 2x2 .. 20x20 sweep (Sec. 6.2), 18, 19.
#include "ssam_kernel2d.h"

// Default: products on the matrix cores (faster from 7x7 on); variant 5: on the vector unit.

SSAM_INSTANCE_2D_MFMA(4, 18, 18, 9, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 18, 18, 9, 2, 1, 2, 5);
SSAM_INSTANCE_2D_MFMA(4, 19, 19, 9, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 19, 19, 9, 2, 1, 2, 5);
