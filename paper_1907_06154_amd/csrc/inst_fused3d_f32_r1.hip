// Two-sweep (temporally blocked) radius-1 3D stencil instances, f32: inst_fused3d_f32_r1.hip
// Variant 0 is the faster of the two on 512^3 (with or without a second plane buffer); variant 1 the other.
#include "ssam_kernel3d_fused.h"

SSAM_INSTANCE_3D_FUSED(float, SSAM_F32, 4, 4, 1, 1, 1, 1, 0, 2, 0);
SSAM_INSTANCE_3D_FUSED(float, SSAM_F32, 4, 4, 1, 1, 1, 2, 0, 2, 0);
