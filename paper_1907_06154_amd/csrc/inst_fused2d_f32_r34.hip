// Multi-sweep (temporally blocked) 2D stencil instances: inst_fused2d_f32_r34.hip
#include "ssam_kernel2d_fused.h"

SSAM_INSTANCE_2D_FUSED(float, SSAM_F32, 4, 4, 3, 1, 2, 2, 0);
SSAM_INSTANCE_2D_FUSED(float, SSAM_F32, 4, 4, 3, 1, 3, 2, 0);
SSAM_INSTANCE_2D_FUSED(float, SSAM_F32, 4, 4, 3, 1, 4, 2, 0);
SSAM_INSTANCE_2D_FUSED(float, SSAM_F32, 4, 4, 4, 1, 2, 2, 0);
SSAM_INSTANCE_2D_FUSED(float, SSAM_F32, 4, 4, 4, 1, 3, 2, 0);
