// Launchers of the column family (normalisation over a dimension that is not the innermost).
#include "pf_col_kernels.hpp"
#include "pf_launch.h"

namespace pf {

template <int DT, bool RMS>
static hipError_t launch_colnorm_dt(const ColArgs& a, int kc, dim3 grid, hipStream_t st) {
    switch (kc) {
        case 1: hipLaunchKernelGGL((colnorm_kernel<DT, 1, RMS>), grid, dim3(256), 0, st, a); break;
        case 2: hipLaunchKernelGGL((colnorm_kernel<DT, 2, RMS>), grid, dim3(256), 0, st, a); break;
        case 4: hipLaunchKernelGGL((colnorm_kernel<DT, 4, RMS>), grid, dim3(256), 0, st, a); break;
        case 16: hipLaunchKernelGGL((colnorm_kernel<DT, 16, RMS>), grid, dim3(256), 0, st, a); break;
        case 32: hipLaunchKernelGGL((colnorm_kernel<DT, 32, RMS>), grid, dim3(256), 0, st, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_colnorm(int dtype, const ColArgs& a, int kc, bool rms, dim3 grid, hipStream_t st) {
    switch (dtype) {
        case DT_F32: return rms ? launch_colnorm_dt<DT_F32, true>(a, kc, grid, st) : launch_colnorm_dt<DT_F32, false>(a, kc, grid, st);
        case DT_F16: return rms ? launch_colnorm_dt<DT_F16, true>(a, kc, grid, st) : launch_colnorm_dt<DT_F16, false>(a, kc, grid, st);
        case DT_BF16: return rms ? launch_colnorm_dt<DT_BF16, true>(a, kc, grid, st) : launch_colnorm_dt<DT_BF16, false>(a, kc, grid, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace pf
