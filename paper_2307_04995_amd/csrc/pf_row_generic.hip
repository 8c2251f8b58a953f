// Generic (run-time interpreted) instantiations of the row and element-wise families, and their launchers.
#include "pf_launch.h"
#include "pf_row_kernels.hpp"

namespace pf {

template <int DT, bool RAGGED>
static hipError_t launch_row_dt(const ChainArgs& a, const RowGeom& g, int k, bool reduce_only, dim3 grid, dim3 block,
                                hipStream_t st) {
    const bool small = block.x <= 256;
#define PF_ROW_CASE(KK)                                                                                                \
    case KK:                                                                                                           \
        if (reduce_only) hipLaunchKernelGGL((row_reduce_kernel<DT, KK, RAGGED>), grid, block, 0, st, a, g);           \
        else if (small) hipLaunchKernelGGL((row_kernel<DT, KK, 1, GenericSpec, 256, false, RAGGED>), grid, block, 0, st, a, g); \
        else hipLaunchKernelGGL((row_kernel<DT, KK, 1, GenericSpec, 1024, false, RAGGED>), grid, block, 0, st, a, g);  \
        break;
    switch (k) {
        PF_ROW_CASE(1)
        PF_ROW_CASE(2)
        PF_ROW_CASE(4)
        default: return hipErrorInvalidValue;
    }
#undef PF_ROW_CASE
    return hipGetLastError();
}

hipError_t launch_row_generic(int dtype, const ChainArgs& a, const RowGeom& g, int k, bool reduce_only, bool ragged,
                              dim3 grid, dim3 block, hipStream_t st) {
    switch (dtype) {
        case DT_F32:
            return ragged ? launch_row_dt<DT_F32, true>(a, g, k, reduce_only, grid, block, st)
                          : launch_row_dt<DT_F32, false>(a, g, k, reduce_only, grid, block, st);
        case DT_F16:
            return ragged ? launch_row_dt<DT_F16, true>(a, g, k, reduce_only, grid, block, st)
                          : launch_row_dt<DT_F16, false>(a, g, k, reduce_only, grid, block, st);
        case DT_BF16:
            return ragged ? launch_row_dt<DT_BF16, true>(a, g, k, reduce_only, grid, block, st)
                          : launch_row_dt<DT_BF16, false>(a, g, k, reduce_only, grid, block, st);
        default: return hipErrorInvalidValue;
    }
}

template <int DT, bool RAGGED>
static hipError_t launch_ew_dt(const ChainArgs& a, uint32_t total_vecs, uint32_t vecs_per_row, int k, dim3 grid,
                               hipStream_t st) {
    switch (k) {
        case 1: hipLaunchKernelGGL((ew_kernel<DT, 1, GenericSpec, RAGGED>), grid, dim3(256), 0, st, a, total_vecs, vecs_per_row); break;
        case 2: hipLaunchKernelGGL((ew_kernel<DT, 2, GenericSpec, RAGGED>), grid, dim3(256), 0, st, a, total_vecs, vecs_per_row); break;
        case 4: hipLaunchKernelGGL((ew_kernel<DT, 4, GenericSpec, RAGGED>), grid, dim3(256), 0, st, a, total_vecs, vecs_per_row); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_ew(int dtype, const ChainArgs& a, uint32_t total_vecs, uint32_t vecs_per_row, int k, bool ragged,
                     dim3 grid, hipStream_t st) {
    switch (dtype) {
        case DT_F32:
            return ragged ? launch_ew_dt<DT_F32, true>(a, total_vecs, vecs_per_row, k, grid, st)
                          : launch_ew_dt<DT_F32, false>(a, total_vecs, vecs_per_row, k, grid, st);
        case DT_F16:
            return ragged ? launch_ew_dt<DT_F16, true>(a, total_vecs, vecs_per_row, k, grid, st)
                          : launch_ew_dt<DT_F16, false>(a, total_vecs, vecs_per_row, k, grid, st);
        case DT_BF16:
            return ragged ? launch_ew_dt<DT_BF16, true>(a, total_vecs, vecs_per_row, k, grid, st)
                          : launch_ew_dt<DT_BF16, false>(a, total_vecs, vecs_per_row, k, grid, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace pf
