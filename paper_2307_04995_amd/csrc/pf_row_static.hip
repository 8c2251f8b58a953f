// Dispatch of the statically specialised row kernels by storage type.
#include "pf_launch.h"
#include "pf_specs.h"

namespace pf {

hipError_t launch_row_static_f32(int spec_id, const ChainArgs& a, const RowGeom& g, int kc, dim3 grid, dim3 block, hipStream_t st);
hipError_t launch_row_static_f16(int spec_id, const ChainArgs& a, const RowGeom& g, int kc, dim3 grid, dim3 block, hipStream_t st);
hipError_t launch_row_static_bf16(int spec_id, const ChainArgs& a, const RowGeom& g, int kc, dim3 grid, dim3 block, hipStream_t st);

// Whether (spec, vectors per row per lane, rows per wave, block size) has a static instantiation.
bool row_static_available(int spec_id, int kc, int rpw, bool wave_rows, unsigned block_threads) {
    if (block_threads > 256) return false;
    if (kc != 1 && kc != 2 && kc != 4) return false;
    if (rpw != 1 && rpw != 2 && rpw != 4) return false;
    if (!wave_rows && rpw != 1) return false;
    if (kc * rpw > 4) return false;
    switch (spec_id) {
#define PF_CASE(id, ...) case id:
        PF_ROW_SPECS(PF_CASE)
#undef PF_CASE
        return true;
        default: return false;
    }
}

hipError_t launch_row_static(int spec_id, int dtype, const ChainArgs& a, const RowGeom& g, int kc, dim3 grid, dim3 block,
                             hipStream_t st) {
    switch (dtype) {
        case DT_F32: return launch_row_static_f32(spec_id, a, g, kc, grid, block, st);
        case DT_F16: return launch_row_static_f16(spec_id, a, g, kc, grid, block, st);
        case DT_BF16: return launch_row_static_bf16(spec_id, a, g, kc, grid, block, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace pf
