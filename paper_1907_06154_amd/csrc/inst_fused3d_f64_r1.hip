// Two-sweep (temporally blocked) radius-1 3D stencil instances, f64: inst_fused3d_f64_r1.hip
// One wave per tile.  The 7-point star's default is the block-cooperative kernel of inst_fused3d_ring.hip; this
// one is its variant 1 and its fallback (clamp rule, unaligned rows).
#include "ssam_kernel3d_fused.h"

SSAM_INSTANCE_3D_FUSED(double, SSAM_F64, 2, 4, 1, 1, 1, 1, 1, 2, 1);
SSAM_INSTANCE_3D_FUSED(double, SSAM_F64, 2, 4, 1, 1, 1, 2, 0, 2, 0);
SSAM_INSTANCE_3D_FUSED(double, SSAM_F64, 2, 4, 1, 1, 1, 3, 1, 2, 0);
