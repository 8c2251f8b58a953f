// Statically specialised instantiations of the row family (one per catalogue entry, storage type and
// vectors-per-lane count) and their launcher.
#include "pf_launch.h"
#include "pf_row_kernels.hpp"
#include "pf_specs.h"

namespace pf {

template <int ID>
struct RowSpecOf;
#define PF_DEF_SPEC(id, nf, nv, nt, core, gamma, beta, pro, epi)                                              \
    template <>                                                                                                \
    struct RowSpecOf<id> {                                                                                     \
        using type = StaticSpec<nf, nv, nt, core, gamma, beta, StaticList<pro>, StaticList<epi>>;              \
    };
PF_ROW_SPECS(PF_DEF_SPEC)
#undef PF_DEF_SPEC

template <int ID, int DT>
static hipError_t launch_spec_dt(const ChainArgs& a, const RowGeom& g, int k, dim3 grid, dim3 block, hipStream_t st) {
    using Spec = typename RowSpecOf<ID>::type;
    if (block.x > 256) return hipErrorInvalidValue;
    const bool wave_rows = g.waves_per_row == 1;
#define PF_K_CASE(KK)                                                                                     \
    case KK:                                                                                              \
        if (wave_rows) hipLaunchKernelGGL((row_kernel<DT, KK, Spec, 256, true>), grid, block, 0, st, a, g); \
        else hipLaunchKernelGGL((row_kernel<DT, KK, Spec, 256, false>), grid, block, 0, st, a, g);        \
        break;
    switch (k) {
        PF_K_CASE(1)
        PF_K_CASE(2)
        PF_K_CASE(4)
        default: return hipErrorInvalidValue;
    }
#undef PF_K_CASE
    return hipGetLastError();
}

template <int ID>
static hipError_t launch_spec(int dtype, const ChainArgs& a, const RowGeom& g, int k, dim3 grid, dim3 block,
                              hipStream_t st) {
    switch (dtype) {
        case DT_F32: return launch_spec_dt<ID, DT_F32>(a, g, k, grid, block, st);
        case DT_F16: return launch_spec_dt<ID, DT_F16>(a, g, k, grid, block, st);
        case DT_BF16: return launch_spec_dt<ID, DT_BF16>(a, g, k, grid, block, st);
        default: return hipErrorInvalidValue;
    }
}

// Whether (spec, k, block size) has a static instantiation.
bool row_static_available(int spec_id, int k, unsigned block_threads) {
    if (block_threads > 256 || (k != 1 && k != 2 && k != 4)) return false;
    switch (spec_id) {
#define PF_CASE(id, ...) case id:
        PF_ROW_SPECS(PF_CASE)
#undef PF_CASE
        return true;
        default: return false;
    }
}

hipError_t launch_row_static(int spec_id, int dtype, const ChainArgs& a, const RowGeom& g, int k, dim3 grid,
                             dim3 block, hipStream_t st) {
    switch (spec_id) {
#define PF_CASE(id, ...) \
    case id: return launch_spec<id>(dtype, a, g, k, grid, block, st);
        PF_ROW_SPECS(PF_CASE)
#undef PF_CASE
        default: return hipErrorInvalidValue;
    }
}

}  // namespace pf
