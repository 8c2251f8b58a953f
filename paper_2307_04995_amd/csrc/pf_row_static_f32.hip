// Static row-family kernels, fp32 storage.
#define PF_STATIC_DT DT_F32
#define PF_STATIC_LAUNCH launch_row_static_f32
#include "pf_row_static.inc"
