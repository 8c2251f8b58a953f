// Static row-family kernels, fp16 storage.
#define PF_STATIC_DT DT_F16
#define PF_STATIC_LAUNCH launch_row_static_f16
#include "pf_row_static.inc"
