// Run-time-interpreted instantiations of the stencil family and their launcher.
#include "pf_launch.h"
#include "pf_stencil_kernels.hpp"

namespace pf {

hipError_t launch_stencil(int dtype, const ChainArgs& a, const StencilGeom& g, dim3 grid, hipStream_t st) {
    switch (dtype) {
        case DT_F32: hipLaunchKernelGGL((dwconv3x3_kernel<DT_F32, GenericSpec>), grid, dim3(256), 0, st, a, g); break;
        case DT_F16: hipLaunchKernelGGL((dwconv3x3_kernel<DT_F16, GenericSpec>), grid, dim3(256), 0, st, a, g); break;
        case DT_BF16: hipLaunchKernelGGL((dwconv3x3_kernel<DT_BF16, GenericSpec>), grid, dim3(256), 0, st, a, g); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace pf
