// Multi-sweep (temporally blocked) 2D stencil instances, stars of radius 5 and 6: inst_fused2d_r56.hip
#include "ssam_kernel2d_fused.h"

SSAM_INSTANCE_2D_FUSED(double, SSAM_F64, 2, 4, 5, 1, 2, 2, 0);
SSAM_INSTANCE_2D_FUSED(double, SSAM_F64, 2, 4, 6, 1, 2, 2, 0);
SSAM_INSTANCE_2D_FUSED(float, SSAM_F32, 4, 4, 5, 1, 2, 2, 0);
SSAM_INSTANCE_2D_FUSED(float, SSAM_F32, 4, 4, 6, 1, 2, 2, 0);
