// Static row-family kernels, bf16 storage.
#define PF_STATIC_DT DT_BF16
#define PF_STATIC_LAUNCH launch_row_static_bf16
#include "pf_row_static.inc"
