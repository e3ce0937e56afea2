// Alternative instances of shapes that also have a default instance: selectable with the
// "variant" tuning knob, used to compare cache policy, register-cache depth (P), columns per
// lane (V) and in-wave prefetch.
#include "ssam_kernel2d.h"
#include "ssam_kernel3d.h"

SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 3, 3, 1, 2, 0, 2, 1);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 3, 3, 1, 2, 1, 2, 2);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 3, 3, 1, 2, 0, 2, 3);
SSAM_INSTANCE_3D_V(double, SSAM_F64, 2, 4, 1, 1, 1, 1, 0, 2, 1);
SSAM_INSTANCE_3D_V(double, SSAM_F64, 2, 4, 1, 1, 1, 3, 1, 2, 1);
SSAM_INSTANCE_3D_V(float, SSAM_F32, 2, 4, 1, 1, 1, 1, 1, 2, 1);
SSAM_INSTANCE_3D_V(float, SSAM_F32, 2, 4, 1, 1, 1, 3, 1, 2, 1);
SSAM_INSTANCE_3D_V(float, SSAM_F32, 4, 4, 1, 1, 1, 1, 0, 2, 2);
SSAM_INSTANCE_3D_V(float, SSAM_F32, 4, 4, 1, 1, 1, 3, 0, 2, 2);
SSAM_INSTANCE_2D_V(double, SSAM_F64, 2, 8, 3, 3, 1, 2, 1, 3, 1);
SSAM_INSTANCE_2D_V(double, SSAM_F64, 2, 8, 3, 3, 1, 2, 1, 1, 2);
SSAM_INSTANCE_2D_V(double, SSAM_F64, 2, 8, 3, 3, 1, 2, 1, 0, 3);
SSAM_INSTANCE_2D_V(double, SSAM_F64, 2, 4, 3, 3, 1, 2, 1, 2, 4);
SSAM_INSTANCE_2D_V(double, SSAM_F64, 2, 8, 3, 3, 1, 2, 0, 2, 5);
SSAM_INSTANCE_2D_V(double, SSAM_F64, 2, 4, 3, 3, 1, 2, 0, 2, 6);
SSAM_INSTANCE_2D_V(double, SSAM_F64, 2, 16, 3, 3, 1, 2, 0, 2, 7);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 9, 9, 4, 2, 1, 2, 1);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 9, 9, 4, 2, 0, 2, 2);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 3, 11, 1, 2, 1, 2, 1);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 3, 11, 1, 2, 0, 2, 2);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 11, 3, 5, 2, 1, 2, 1);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 8, 11, 3, 5, 2, 0, 2, 2);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 15, 15, 7, 2, 0, 2, 1);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 4, 20, 20, 10, 2, 0, 2, 1);
SSAM_INSTANCE_2D_V(float, SSAM_F32, 4, 2, 20, 20, 10, 2, 1, 2, 2);
