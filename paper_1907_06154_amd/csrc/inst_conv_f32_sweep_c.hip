// Compiled instances: square filters of the 2x2 .. 20x20 sweep (Sec. 6.2), 13, 14.
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 13, 13, 6, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 14, 14, 7, 2, 1, 2, 0);
