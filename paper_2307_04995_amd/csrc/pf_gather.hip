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

// The same copy with K vectors per lane (a workgroup takes 256 * K consecutive vectors, lane t the vectors t, t + 256,
// ...): the K table look-ups of a lane are in flight together, and so are its K loads when all of them are whole
// vectors (any partial one sends the lane down the element-by-element path, vector by vector).  A lane past the end
// looks up the last vector and moves nothing.
template <int DT, int K>
__global__ void __launch_bounds__(256) gather_runs_multi_kernel(const GatherArgs a) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    const uint64_t total = (uint64_t)a.n_runs * a.vec_per_run;
    const uint64_t g0 = (uint64_t)blockIdx.x * (256u * K) + threadIdx.x;
    GatherRun e[K];
    uint32_t first[K], count[K];
#pragma unroll
    for (int i = 0; i < K; ++i) {
        const uint64_t gv64 = g0 + (uint64_t)i * 256u;
        const bool ok = gv64 < total;
        const uint32_t gv = (uint32_t)(ok ? gv64 : total - 1u);
        const uint32_t run = fast_div(gv, a.div_vpr);
        first[i] = (gv - run * a.vec_per_run) * VEC;
        count[i] = ok ? elems_below<VEC>(first[i], a.run_elems) : 0u;
        e[i] = a.table[run];
    }
    const void* src[K];
    void* dst[K];
    bool whole = true;
#pragma unroll
    for (int i = 0; i < K; ++i) {
        src[i] = a.in[0];
#pragma unroll
        for (int j = 1; j < 8; ++j) src[i] = e[i].src_id == j ? a.in[j] : src[i];
        dst[i] = a.out[0];
#pragma unroll
        for (int j = 1; j < 3; ++j) dst[i] = e[i].dst_id == j ? a.out[j] : dst[i];
        whole = whole && count[i] == (uint32_t)VEC;
    }
    if (whole) {
        u32x4 data[K];
#pragma unroll
        for (int i = 0; i < K; ++i) data[i] = load_elems<DT>(src[i], (uint64_t)e[i].src_off + first[i], (uint32_t)VEC, 0u);
#pragma unroll
        for (int i = 0; i < K; ++i) store_elems<DT>(dst[i], (uint64_t)e[i].dst_off + first[i], (uint32_t)VEC, data[i]);
    } else {
#pragma unroll
        for (int i = 0; i < K; ++i) {
            if (count[i] == 0u) continue;
            const u32x4 data = load_elems<DT>(src[i], (uint64_t)e[i].src_off + first[i], count[i], 0u);
            store_elems<DT>(dst[i], (uint64_t)e[i].dst_off + first[i], count[i], data);
        }
    }
}

hipError_t launch_gather(int dtype, const GatherArgs& a, int k, dim3 grid, hipStream_t st) {
    // the copy only depends on the element size
    if (k == 4) {
        if (dtype == DT_F32) hipLaunchKernelGGL((gather_runs_multi_kernel<DT_F32, 4>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((gather_runs_multi_kernel<DT_F16, 4>), grid, dim3(256), 0, st, a);
    } else if (k == 2) {
        if (dtype == DT_F32) hipLaunchKernelGGL((gather_runs_multi_kernel<DT_F32, 2>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((gather_runs_multi_kernel<DT_F16, 2>), grid, dim3(256), 0, st, a);
    } else if (k == 1) {
        if (dtype == DT_F32) hipLaunchKernelGGL((gather_runs_kernel<DT_F32>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((gather_runs_kernel<DT_F16>), grid, dim3(256), 0, st, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace pf
