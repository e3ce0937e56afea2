// Compiled register-cache instances: 25-point star of radius 4 (largest register pressure).
// Nine output planes are in flight per lane, so the instances keep one plane buffer (fp64)
// or two narrow ones (fp32 with two columns per lane) to stay clear of register spilling.
#include "ssam_kernel3d.h"

SSAM_INSTANCE_3D_V(float, SSAM_F32, 2, 4, 4, 4, 4, 1, 1, 2, 0);
SSAM_INSTANCE_3D_V(double, SSAM_F64, 2, 4, 4, 4, 4, 1, 0, 2, 0);
