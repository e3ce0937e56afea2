// Two-sweep (temporally blocked) radius-2 3D star instances, fp32: inst_fused3d_r2.hip
// (Five in-flight planes at each of the two levels: the fp64 version spills and is slower than
// single sweeps, so there is none.)
#include "ssam_kernel3d_fused.h"

SSAM_INSTANCE_3D_FUSED(float, SSAM_F32, 2, 4, 2, 2, 2, 1, 1, 2, 0);
