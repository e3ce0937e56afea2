// Block-cooperative (LDS-staged) alternatives for the radius-1 3D shapes (tuning variants).
#include "ssam_kernel3d_lds.h"

SSAM_INSTANCE_3D_LDS(double, SSAM_F64, 2, 4, 4, 1, 1, 1, 1, 2, 7);
SSAM_INSTANCE_3D_LDS(double, SSAM_F64, 2, 4, 4, 1, 1, 1, 3, 2, 7);
SSAM_INSTANCE_3D_LDS(double, SSAM_F64, 2, 4, 4, 1, 1, 1, 2, 2, 7);
SSAM_INSTANCE_3D_LDS(double, SSAM_F64, 2, 2, 4, 1, 1, 1, 1, 2, 8);
SSAM_INSTANCE_3D_LDS(double, SSAM_F64, 2, 2, 4, 1, 1, 1, 3, 2, 8);
SSAM_INSTANCE_3D_LDS(double, SSAM_F64, 2, 2, 4, 1, 1, 1, 2, 2, 8);
SSAM_INSTANCE_3D_LDS(float, SSAM_F32, 2, 4, 4, 1, 1, 1, 1, 2, 7);
SSAM_INSTANCE_3D_LDS(float, SSAM_F32, 2, 4, 4, 1, 1, 1, 3, 2, 7);
SSAM_INSTANCE_3D_LDS(float, SSAM_F32, 2, 4, 4, 4, 4, 4, 1, 2, 7);
SSAM_INSTANCE_3D_LDS(double, SSAM_F64, 2, 4, 4, 4, 4, 4, 1, 2, 7);
SSAM_INSTANCE_3D_LDS(double, SSAM_F64, 2, 2, 4, 4, 4, 4, 1, 2, 8);
SSAM_INSTANCE_3D_LDS(float, SSAM_F32, 4, 2, 4, 4, 4, 4, 1, 2, 8);
