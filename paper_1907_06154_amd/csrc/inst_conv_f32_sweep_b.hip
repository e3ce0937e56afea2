// Compiled instances: square filters of the 2x2 .. 20x20 sweep (Sec. 6.2), 10 .. 12.
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 10, 10, 5, 2, 0, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 11, 11, 5, 2, 0, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 12, 12, 6, 2, 1, 2, 0);
