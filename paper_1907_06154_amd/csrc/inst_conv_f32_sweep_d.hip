// Compiled instances: square filters of the 2x2 .. 20x20 sweep (Sec. 6.2), 16, 17.
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 16, 16, 8, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 17, 17, 8, 2, 1, 2, 0);
