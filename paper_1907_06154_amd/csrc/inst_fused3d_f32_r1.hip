// Two-sweep (temporally blocked) radius-1 3D stencil instance, f32: inst_fused3d_f32_r1.hip
// Only the 7-point star has one: for the 19- and 27-point shapes and the radius-2 star the
// block-cooperative single-sweep kernel is as fast or faster on 512^3 (19-point: 714 against 688
// GStencil/s, radius-2 star: 706 against 634).  One wave per tile: variant 1 and fallback (clamp rule, unaligned
// rows) of the block-cooperative default in inst_fused3d_ring.hip.
#include "ssam_kernel3d_fused.h"

SSAM_INSTANCE_3D_FUSED(float, SSAM_F32, 4, 4, 1, 1, 1, 1, 0, 2, 1);
