// Launchers of the column family (normalisation over a dimension that is not the innermost).
#include "pf_col_kernels.hpp"
#include "pf_launch.h"

namespace pf {

template <int DT, bool RMS, bool RAGGED>
static hipError_t launch_colnorm_dt(const ColArgs& a, int kc, dim3 grid, hipStream_t st) {
    switch (kc) {
        case 1: hipLaunchKernelGGL((colnorm_kernel<DT, 1, RMS, RAGGED>), grid, dim3(256), 0, st, a); break;
        case 2: hipLaunchKernelGGL((colnorm_kernel<DT, 2, RMS, RAGGED>), grid, dim3(256), 0, st, a); break;
        case 3: hipLaunchKernelGGL((colnorm_kernel<DT, 3, RMS, RAGGED>), grid, dim3(256), 0, st, a); break;
        case 4: hipLaunchKernelGGL((colnorm_kernel<DT, 4, RMS, RAGGED>), grid, dim3(256), 0, st, a); break;
        case 6: hipLaunchKernelGGL((colnorm_kernel<DT, 6, RMS, RAGGED>), grid, dim3(256), 0, st, a); break;
        case 8: hipLaunchKernelGGL((colnorm_kernel<DT, 8, RMS, RAGGED>), grid, dim3(256), 0, st, a); break;
        case 12: hipLaunchKernelGGL((colnorm_kernel<DT, 12, RMS, RAGGED>), grid, dim3(256), 0, st, a); break;
        case 16: hipLaunchKernelGGL((colnorm_kernel<DT, 16, RMS, RAGGED>), grid, dim3(256), 0, st, a); break;
        case 24: hipLaunchKernelGGL((colnorm_kernel<DT, 24, RMS, RAGGED>), grid, dim3(256), 0, st, a); break;
        case 32: hipLaunchKernelGGL((colnorm_kernel<DT, 32, RMS, RAGGED>), grid, dim3(256), 0, st, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int DT>
static hipError_t launch_colnorm_kind(const ColArgs& a, int kc, bool rms, bool ragged, dim3 grid, hipStream_t st) {
    if (ragged) return rms ? launch_colnorm_dt<DT, true, true>(a, kc, grid, st) : launch_colnorm_dt<DT, false, true>(a, kc, grid, st);
    return rms ? launch_colnorm_dt<DT, true, false>(a, kc, grid, st) : launch_colnorm_dt<DT, false, false>(a, kc, grid, st);
}

hipError_t launch_colnorm(int dtype, const ColArgs& a, int kc, bool rms, bool ragged, dim3 grid, hipStream_t st) {
    switch (dtype) {
        case DT_F32: return launch_colnorm_kind<DT_F32>(a, kc, rms, ragged, grid, st);
        case DT_F16: return launch_colnorm_kind<DT_F16>(a, kc, rms, ragged, grid, st);
        case DT_BF16: return launch_colnorm_kind<DT_BF16>(a, kc, rms, ragged, grid, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace pf
