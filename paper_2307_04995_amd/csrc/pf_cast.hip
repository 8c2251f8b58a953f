// Storage conversion of a whole tensor: 16-bit <-> fp32.
//
// A chain that runs as several kernels computes in fp32 from its first load to its last store, like a chain that
// is one kernel: its 16-bit inputs are widened once (exact), every tensor between two kernels is fp32, and the
// results are rounded to the storage type once at the end (round to nearest even).  These two copies are the
// widening and the final rounding.
#include "pf_device.hpp"
#include "pf_launch.h"

namespace pf {

// eight elements per lane: one 16-byte vector on the 16-bit side, two on the fp32 side
template <int DT, bool WIDEN>
__global__ void __launch_bounds__(256) cast_kernel(const void* __restrict__ src, void* __restrict__ dst, uint64_t n) {
    using S = Storage<DT>;
    const uint64_t first = ((uint64_t)blockIdx.x * 256u + threadIdx.x) * 8u;
    if (first >= n) return;
    const uint32_t cnt = n - first < 8u ? (uint32_t)(n - first) : 8u;
    float v[8];
    if (WIDEN) {
        const u32x4 raw = load_elems<DT>(src, first, cnt, 0u);
        S::unpack(raw, v);
        u32x4 lo = Storage<DT_F32>::pack(v), hi = Storage<DT_F32>::pack(v + 4);
        store_elems<DT_F32>(dst, first, cnt < 4u ? cnt : 4u, lo);
        if (cnt > 4u) store_elems<DT_F32>(dst, first + 4u, cnt - 4u, hi);
    } else {
        const u32x4 lo = load_elems<DT_F32>(src, first, cnt < 4u ? cnt : 4u, 0u);
        u32x4 hi = {0u, 0u, 0u, 0u};
        if (cnt > 4u) hi = load_elems<DT_F32>(src, first + 4u, cnt - 4u, 0u);
        Storage<DT_F32>::unpack(lo, v);
        Storage<DT_F32>::unpack(hi, v + 4);
        store_elems<DT>(dst, first, cnt, S::pack(v));
    }
}

hipError_t launch_cast(int src_dtype, int dst_dtype, const void* src, void* dst, uint64_t n, hipStream_t st) {
    if (n == 0) return hipSuccess;
    const uint64_t blocks = (n + 2047u) / 2048u;
    if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)blocks), block(256);
    if (src_dtype == DT_F16 && dst_dtype == DT_F32) hipLaunchKernelGGL((cast_kernel<DT_F16, true>), grid, block, 0, st, src, dst, n);
    else if (src_dtype == DT_BF16 && dst_dtype == DT_F32) hipLaunchKernelGGL((cast_kernel<DT_BF16, true>), grid, block, 0, st, src, dst, n);
    else if (src_dtype == DT_F32 && dst_dtype == DT_F16) hipLaunchKernelGGL((cast_kernel<DT_F16, false>), grid, block, 0, st, src, dst, n);
    else if (src_dtype == DT_F32 && dst_dtype == DT_BF16) hipLaunchKernelGGL((cast_kernel<DT_BF16, false>), grid, block, 0, st, src, dst, n);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace pf
