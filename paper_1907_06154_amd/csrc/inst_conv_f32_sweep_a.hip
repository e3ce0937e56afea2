// Compiled instances: square filters of the 2x2 .. 20x20 sweep (Sec. 6.2), small sizes.
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 2, 2, 1, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 4, 4, 2, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 6, 6, 3, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 7, 7, 3, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 8, 8, 4, 2, 0, 2, 0);
