// Two sweeps per launch of the 7-point 3D star on the block-cooperative plane ring: inst_fused3d_ring.hip
// The default two-sweep instances of that shape (512^3: fp64 595 -> 727 GStencil/s, fp32 1155 -> 1370 against the
// one-wave-per-tile two-sweep kernel, which remains as variant 1 and takes the clamp rule and unaligned rows).
// Four rows per wave in fp64, two in fp32 (the other choice measured 1 % slower in each).
#include "ssam_kernel3d_star2.h"

SSAM_INSTANCE_3D_STAR2(double, SSAM_F64, 4, 8, 3, 2, (::ssam::launch3d_fused<double, 2, 4, 1, 1, 1, 1, 2, true>), 0);
SSAM_INSTANCE_3D_STAR2(float, SSAM_F32, 2, 8, 3, 2, (::ssam::launch3d_fused<float, 4, 4, 1, 1, 1, 1, 2, false>), 0);
