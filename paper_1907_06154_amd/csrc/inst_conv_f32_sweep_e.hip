// Compiled instances: square filters of the 2x2 .. 20x20 sweep (Sec. 6.2), 18, 19.
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 18, 18, 9, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 19, 19, 9, 2, 1, 2, 0);
