// Compiled instances: remaining 2D shapes of Table 3 (stars of order 5 and 6; 7x7, 9x9, 11x11 boxes).
#include "ssam_kernel2d.h"

SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 11, 11, 5, 1, 1, 2, 0);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 13, 13, 6, 1, 1, 2, 0);
SSAM_INSTANCE_2D_V(double, SSAM_F64, 2, 8, 11, 11, 5, 1, 1, 2, 0);
SSAM_INSTANCE_2D_V(double, SSAM_F64, 2, 8, 13, 13, 6, 1, 1, 2, 0);
SSAM_INSTANCE_2D_V(double, SSAM_F64, 2, 8, 7, 7, 3, 2, 0, 2, 0);
SSAM_INSTANCE_2D_V(double, SSAM_F64, 2, 4, 9, 9, 4, 2, 1, 2, 0);
SSAM_INSTANCE_2D_V(double, SSAM_F64, 2, 4, 8, 8, 4, 2, 1, 2, 0);   // 2d64pt: the 8x8 box
