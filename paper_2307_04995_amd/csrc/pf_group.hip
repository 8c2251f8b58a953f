// Build-time instantiations of the group family (catalogue entries and the run-time-interpreted form) and
// their launcher.
#include "pf_group_kernels.hpp"
#include "pf_launch.h"
#include "pf_specs.h"

namespace pf {

// ---------------------------------------------------------------------------------------------
template <int ID>
struct GroupSpecOf;
#define PF_DEF_SPEC(id, nf, nv, nt, core, gamma, beta, pro, epi)                                              \
    template <>                                                                                                \
    struct GroupSpecOf<id> {                                                                                   \
        using type = StaticSpec<nf, nv, nt, core, gamma, beta, StaticList<pro>, StaticList<epi>>;              \
    };
PF_GROUP_SPECS(PF_DEF_SPEC)
#undef PF_DEF_SPEC
template <>
struct GroupSpecOf<0> {
    using type = GenericSpec;
};

template <int ID, int DT, int PHASE, int GEN>
static hipError_t launch_group_nv(const ChainArgs& a, const GroupGeom& g, int nv, uint32_t tiles, dim3 grid,
                                  dim3 block, uint32_t lds, hipStream_t st) {
    using Spec = typename GroupSpecOf<ID>::type;
    switch (nv) {
        case 4: hipLaunchKernelGGL((group_kernel<DT, 4, Spec, PHASE, GEN>), grid, block, lds, st, a, g, tiles); break;
        case 8: hipLaunchKernelGGL((group_kernel<DT, 8, Spec, PHASE, GEN>), grid, block, lds, st, a, g, tiles); break;
        case 16: hipLaunchKernelGGL((group_kernel<DT, 16, Spec, PHASE, GEN>), grid, block, lds, st, a, g, tiles); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int ID, int DT>
static hipError_t launch_group_dt(int phase, bool general, const ChainArgs& a, const GroupGeom& g, int nv, uint32_t tiles,
                                  dim3 grid, dim3 block, uint32_t lds, hipStream_t st) {
    if (general) {
        // groups of any width: built in the run-time-interpreted, two-launch form only (the rest is specialised when
        // the plan is made)
        if constexpr (ID == 0) {
            if (g.ragged) {
                if (phase == 1) return launch_group_nv<0, DT, 1, 3>(a, g, nv, tiles, grid, block, lds, st);
                if (phase == 2) return launch_group_nv<0, DT, 2, 3>(a, g, nv, tiles, grid, block, lds, st);
            }
            if (phase == 1) return launch_group_nv<0, DT, 1, 1>(a, g, nv, tiles, grid, block, lds, st);
            if (phase == 2) return launch_group_nv<0, DT, 2, 1>(a, g, nv, tiles, grid, block, lds, st);
        }
        return hipErrorInvalidValue;
    }
    if (phase == 1) return launch_group_nv<ID, DT, 1, 0>(a, g, nv, tiles, grid, block, lds, st);
    if (phase == 2) return launch_group_nv<ID, DT, 2, 0>(a, g, nv, tiles, grid, block, lds, st);
    if constexpr (ID != 0) return launch_group_nv<ID, DT, 0, 0>(a, g, nv, tiles, grid, block, lds, st);
    return hipErrorInvalidValue;  // the fused variant exists for catalogue entries only
}

template <int ID>
static hipError_t launch_group_id(int phase, bool general, int dtype, const ChainArgs& a, const GroupGeom& g, int nv, uint32_t tiles,
                                  dim3 grid, dim3 block, uint32_t lds, hipStream_t st) {
    switch (dtype) {
        case DT_F32: return launch_group_dt<ID, DT_F32>(phase, general, a, g, nv, tiles, grid, block, lds, st);
        case DT_F16: return launch_group_dt<ID, DT_F16>(phase, general, a, g, nv, tiles, grid, block, lds, st);
        case DT_BF16: return launch_group_dt<ID, DT_BF16>(phase, general, a, g, nv, tiles, grid, block, lds, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_group(int phase, bool general, int spec_id, int dtype, const ChainArgs& a, const GroupGeom& g, int nv, uint32_t tiles,
                        dim3 grid, dim3 block, uint32_t lds, hipStream_t st) {
    switch (spec_id) {
        case 0: return launch_group_id<0>(phase, general, dtype, a, g, nv, tiles, grid, block, lds, st);
#define PF_CASE(id, ...) \
    case id: return launch_group_id<id>(phase, general, dtype, a, g, nv, tiles, grid, block, lds, st);
            PF_GROUP_SPECS(PF_CASE)
#undef PF_CASE
        default: return hipErrorInvalidValue;
    }
}

// how many workgroups of the fused kernel one compute unit holds (for sizing a co-resident grid)
int group_resident_blocks_per_cu(int spec_id, int dtype, int nv, int block_threads) {
    int n = 0;
#define PF_OCC(ID, DT, NVV)                                                                                          \
    if (spec_id == ID && dtype == DT && nv == NVV)                                                                   \
        (void)hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, group_kernel<DT, NVV, typename GroupSpecOf<ID>::type, 0>, \
                                                           block_threads, 0);
#define PF_OCC_ALL(id, ...)                                                                            \
    PF_OCC(id, DT_F32, 4) PF_OCC(id, DT_F32, 8) PF_OCC(id, DT_F32, 16) PF_OCC(id, DT_F16, 4) PF_OCC(id, DT_F16, 8) \
    PF_OCC(id, DT_F16, 16) PF_OCC(id, DT_BF16, 4) PF_OCC(id, DT_BF16, 8) PF_OCC(id, DT_BF16, 16)
    PF_GROUP_SPECS(PF_OCC_ALL)
#undef PF_OCC_ALL
#undef PF_OCC
    return n;
}

}  // namespace pf
