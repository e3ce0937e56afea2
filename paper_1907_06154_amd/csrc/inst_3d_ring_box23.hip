// Compiled instances: dense 3D boxes of radius 2 (125 taps) and 3 (343 taps) on the block-cooperative
// kernel -- the 5x5x5 and 7x7x7 filters of ssam_conv3d and the 125-point box of Table 3.  Two rows per
// wave, eight waves per block (fp64 radius 2: four, so that three blocks share a CU -- 137 registers allow three
// waves per SIMD, which one block of eight cannot use; 829 -> 800 us on 512^3; eight waves remain as variant 10).  Fallback for radius 2: the one-wave-per-tile instance (variant 4 in
// inst_table3_3d.hip); radius 3 has none and falls back to the direct kernel through the dispatcher.
#include "ssam_kernel3d_star.h"

SSAM_INSTANCE_3D_RING(float, SSAM_F32, 2, 8, 2, 3, 3, 2, (::ssam::launch3d<float, 2, 4, 2, 2, 2, 3, 2, false>), 0);
SSAM_INSTANCE_3D_RING(double, SSAM_F64, 2, 4, 2, 3, 3, 2, (::ssam::launch3d<double, 2, 2, 2, 2, 2, 3, 2, false>), 0);
SSAM_INSTANCE_3D_RING(double, SSAM_F64, 2, 8, 2, 3, 3, 2, (::ssam::launch3d<double, 2, 2, 2, 2, 2, 3, 2, false>), 10);
SSAM_INSTANCE_3D_RING(float, SSAM_F32, 2, 8, 3, 3, 3, 2, (::ssam::launch3d_unavailable), 0);
SSAM_INSTANCE_3D_RING(double, SSAM_F64, 2, 8, 3, 3, 3, 2, (::ssam::launch3d_unavailable), 0);
