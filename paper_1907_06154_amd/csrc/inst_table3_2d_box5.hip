// Compiled instances: 11x11 box of Table 3 (2d121pt), fp64 (fp32 is in the filter sweep).
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D_V(double, SSAM_F64, 2, 4, 11, 11, 5, 2, 0, 2, 0);
