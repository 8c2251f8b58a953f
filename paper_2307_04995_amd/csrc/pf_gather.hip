// Gather family: chains made only of layout operators (concatenation, slicing, permutation, reshape).
//
// Such a chain moves every output element from exactly one input element: it is a pure index map (the
// ShuffleNet fragment concat -> channel shuffle -> split of paper section 2 is the standard example, and the
// paper's transposes that are fused into neighbouring operators are of the same kind).  The map is evaluated
// once, on the host, when the plan is made -- not per element on the device: the planner finds the longest
// run length R such that every aligned run of R output elements is contiguous in one input, and writes one
// table entry per run.  The kernel is then a copy that looks up its run: 16-byte vectors at element
// alignment, the partial vector at the end of a run element by element, every byte read once and written
// once, no intermediate tensor.
#include "pf_device.hpp"
#include "pf_launch.h"

namespace pf {

template <int DT>
__global__ void __launch_bounds__(256) gather_runs_kernel(const GatherArgs a) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    const uint64_t gv64 = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (gv64 >= (uint64_t)a.n_runs * a.vec_per_run) return;
    const uint32_t gv = (uint32_t)gv64;
    const uint32_t run = fast_div(gv, a.div_vpr);
    const uint32_t v = gv - run * a.vec_per_run;
    const GatherRun e = a.table[run];
    const void* src = a.in[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) src = e.src_id == i ? a.in[i] : src;
    void* dst = a.out[0];
#pragma unroll
    for (int i = 1; i < 3; ++i) dst = e.dst_id == i ? a.out[i] : dst;
    const uint32_t first = v * VEC;
    const uint32_t count = elems_below<VEC>(first, a.run_elems);
    const u32x4 data = load_elems<DT>(src, (uint64_t)e.src_off + first, count, 0u);
    store_elems<DT>(dst, (uint64_t)e.dst_off + first, count, data);
}

hipError_t launch_gather(int dtype, const GatherArgs& a, dim3 grid, hipStream_t st) {
    // the copy only depends on the element size
    if (dtype == DT_F32) hipLaunchKernelGGL((gather_runs_kernel<DT_F32>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((gather_runs_kernel<DT_F16>), grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace pf
