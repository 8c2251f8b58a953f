// Run-time-interpreted instantiations of the pool family and their launcher.
#include "pf_launch.h"
#include "pf_pool_kernels.hpp"

namespace pf {

template <int DT, int OP, bool RAGGED>
static hipError_t launch_pool_nv(const ChainArgs& a, const PoolGeom& g, int nv, dim3 grid, hipStream_t st) {
    switch (nv) {
        case 1: hipLaunchKernelGGL((pool_kernel<DT, 1, GenericSpec, OP, RAGGED>), grid, dim3(512), 0, st, a, g); break;
        case 2: hipLaunchKernelGGL((pool_kernel<DT, 2, GenericSpec, OP, RAGGED>), grid, dim3(512), 0, st, a, g); break;
        case 4: hipLaunchKernelGGL((pool_kernel<DT, 4, GenericSpec, OP, RAGGED>), grid, dim3(512), 0, st, a, g); break;
        case 8: hipLaunchKernelGGL((pool_kernel<DT, 8, GenericSpec, OP, RAGGED>), grid, dim3(512), 0, st, a, g); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int DT>
static hipError_t launch_pool_dt(const ChainArgs& a, const PoolGeom& g, int op, int nv, dim3 grid, hipStream_t st) {
    switch (op) {
        case POOL_SUM: return g.ragged ? launch_pool_nv<DT, POOL_SUM, true>(a, g, nv, grid, st) : launch_pool_nv<DT, POOL_SUM, false>(a, g, nv, grid, st);
        case POOL_MAX: return g.ragged ? launch_pool_nv<DT, POOL_MAX, true>(a, g, nv, grid, st) : launch_pool_nv<DT, POOL_MAX, false>(a, g, nv, grid, st);
        case POOL_MEAN: return g.ragged ? launch_pool_nv<DT, POOL_MEAN, true>(a, g, nv, grid, st) : launch_pool_nv<DT, POOL_MEAN, false>(a, g, nv, grid, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_pool(int dtype, const ChainArgs& a, const PoolGeom& g, int op, int nv, dim3 grid, hipStream_t st) {
    switch (dtype) {
        case DT_F32: return launch_pool_dt<DT_F32>(a, g, op, nv, grid, st);
        case DT_F16: return launch_pool_dt<DT_F16>(a, g, op, nv, grid, st);
        case DT_BF16: return launch_pool_dt<DT_BF16>(a, g, op, nv, grid, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace pf
