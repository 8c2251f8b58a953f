// Run-time-interpreted instantiations of the stencil family and their launcher.
#include "pf_launch.h"
#include "pf_stencil_kernels.hpp"

namespace pf {

template <int DT, bool RAGGED>
static hipError_t launch_stencil_dt(const ChainArgs& a, const StencilGeom& g, int variant, int ks, uint32_t lds, dim3 grid, hipStream_t st) {
    if (variant == 2 && ks == 5) hipLaunchKernelGGL((dwconv_strided_kernel<DT, GenericSpec, 5, RAGGED>), grid, dim3(256), 0, st, a, g);
    else if (variant == 2) hipLaunchKernelGGL((dwconv_strided_kernel<DT, GenericSpec, 3, RAGGED>), grid, dim3(256), 0, st, a, g);
    else if (variant == 1 && ks == 5) hipLaunchKernelGGL((dwconv_staged_kernel<DT, GenericSpec, 5, RAGGED>), grid, dim3(256), lds, st, a, g);
    else if (variant == 1) hipLaunchKernelGGL((dwconv_staged_kernel<DT, GenericSpec, 3, RAGGED>), grid, dim3(256), lds, st, a, g);
    else if (ks == 3) hipLaunchKernelGGL((dwconv3x3_kernel<DT, GenericSpec, RAGGED>), grid, dim3(256), 0, st, a, g);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_stencil(int dtype, const ChainArgs& a, const StencilGeom& g, int variant, int ks, uint32_t lds, dim3 grid, hipStream_t st) {
    switch (dtype) {
        case DT_F32: return g.ragged ? launch_stencil_dt<DT_F32, true>(a, g, variant, ks, lds, grid, st) : launch_stencil_dt<DT_F32, false>(a, g, variant, ks, lds, grid, st);
        case DT_F16: return g.ragged ? launch_stencil_dt<DT_F16, true>(a, g, variant, ks, lds, grid, st) : launch_stencil_dt<DT_F16, false>(a, g, variant, ks, lds, grid, st);
        case DT_BF16: return g.ragged ? launch_stencil_dt<DT_BF16, true>(a, g, variant, ks, lds, grid, st) : launch_stencil_dt<DT_BF16, false>(a, g, variant, ks, lds, grid, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace pf
