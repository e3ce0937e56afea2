// Multi-sweep (temporally blocked) 2D stencil instances: inst_fused2d_f64_deep.hip
#include "ssam_kernel2d_fused.h"

SSAM_INSTANCE_2D_FUSED(double, SSAM_F64, 2, 4, 1, 1, 6, 2, 0);
SSAM_INSTANCE_2D_FUSED(double, SSAM_F64, 2, 4, 1, 2, 6, 2, 0);
SSAM_INSTANCE_2D_FUSED(double, SSAM_F64, 2, 4, 1, 2, 8, 2, 0);
