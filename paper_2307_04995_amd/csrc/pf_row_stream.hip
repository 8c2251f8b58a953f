// Run-time-interpreted instantiations of the streaming row variant and their launcher.
#include "pf_launch.h"
#include "pf_row_stream.hpp"

namespace pf {

template <int DT>
static hipError_t launch_stream_dt(const ChainArgs& a, bool ragged, dim3 grid, hipStream_t st) {
    if (ragged) hipLaunchKernelGGL((row_stream_kernel<DT, true, GenericSpec>), grid, dim3(kStreamThreads), 0, st, a);
    else hipLaunchKernelGGL((row_stream_kernel<DT, false, GenericSpec>), grid, dim3(kStreamThreads), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_row_stream(int dtype, const ChainArgs& a, bool ragged, dim3 grid, hipStream_t st) {
    switch (dtype) {
        case DT_F32: return launch_stream_dt<DT_F32>(a, ragged, grid, st);
        case DT_F16: return launch_stream_dt<DT_F16>(a, ragged, grid, st);
        case DT_BF16: return launch_stream_dt<DT_BF16>(a, ragged, grid, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace pf
