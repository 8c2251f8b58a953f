// Pool family: prologue -> reduction over the positions of a channels-last tensor (sum, maximum or mean over
// every dimension between the first and the last: global pooling of x [n, spatial.., c] into [n, 1.., c]) ->
// epilogue on the pooled values.
//
// This is the reduce basic operator (paper section 6) along dimensions that are not contiguous in memory.  A
// workgroup walks whole positions, so its HBM accesses are fully contiguous, and every lane owns one channel
// vector, so the running reduction lives in registers and no value crosses lanes until the workgroup's slice
// is done (one pass through LDS).  A sample's positions are spread over several workgroups: each publishes its
// per-channel partial result and raises a flag; the sample's last workgroup waits for the flags, merges the
// partial results, runs the epilogue and stores -- the device-scope synchronisation of section 5.1.
#pragma once
#include "pf_row_kernels.hpp"

namespace pf {

enum PoolOp : int32_t { POOL_SUM = 0, POOL_MAX = 1, POOL_MEAN = 2 };


template <int OP>
PF_DEVICE float pool_identity() { return OP == POOL_MAX ? -__builtin_inff() : 0.0f; }
// maximum that keeps a NaN once it has seen one (the operator's definition: a NaN element poisons the result)
template <int OP>
PF_DEVICE float pool_combine(float acc, float x) {
    if (OP != POOL_MAX) return acc + x;
    return (x != x) ? x : ((acc != acc) ? acc : fmaxf(acc, x));
}

template <int DT, int NV, class Spec, int OP>
__global__ void __launch_bounds__(512) pool_kernel(const ChainArgs a, const PoolGeom g) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    __shared__ float lds[512 * VEC];
    const uint32_t t = threadIdx.x;
    const uint32_t pstep = fast_div(t, g.div_cv);
    const uint32_t cvi = t - pstep * g.cv;
    const bool active = pstep < g.pos_per_step;
    const uint32_t sample = blockIdx.x / g.blocks_per_sample;
    const uint32_t bx = blockIdx.x - sample * g.blocks_per_sample;
    const uint32_t p_begin = bx * g.pos_per_block;
    const uint32_t p_count = min(g.hw, p_begin + g.pos_per_block) - p_begin;
    const uint32_t pro_full = Spec::kStatic ? list_operand_mask<typename Spec::Pro>(K_FULL) : ~g.epi_full_mask;
    const uint32_t pro_vec = Spec::kStatic ? list_operand_mask<typename Spec::Pro>(K_VEC) : ~g.epi_vec_mask;
    const uint32_t epi_full = Spec::kStatic ? list_operand_mask<typename Spec::Epi>(K_FULL) : g.epi_full_mask;
    const uint32_t epi_vec = Spec::kStatic ? list_operand_mask<typename Spec::Epi>(K_VEC) : g.epi_vec_mask;

    LaneState<DT, 1, Spec> s;
    s.col[0] = cvi * VEC;

    // ---- the slice in chunks of NV position steps: the primary operand of a chunk first (all its loads in flight),
    // then position by position
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = pool_identity<OP>();
    const uint64_t pos0 = (uint64_t)sample * g.hw + p_begin;
    for (uint32_t chunk = 0; chunk < g.chunks; ++chunk) {
        const uint32_t c0 = chunk * (uint32_t)NV * g.pos_per_step;  // first position of the chunk inside the slice
        if (c0 >= p_count) break;
        auto rel_of = [&](int i) { return c0 + pstep + (uint32_t)i * g.pos_per_step; };
        auto valid_of = [&](int i) { return active && rel_of(i) < p_count; };
        u32x4 raw[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            raw[i] = u32x4{0u, 0u, 0u, 0u};
            if (valid_of(i)) raw[i] = load_stream(a.full[0], ((pos0 + rel_of(i)) * g.channels + cvi * VEC) * S::ESIZE);
        }
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const uint32_t pos = (uint32_t)(pos0 + rel_of(i));
            s.row[0] = pos;
            s.fraw[0][0] = raw[i];
#pragma unroll
            for (int f = 1; f < Spec::NF; ++f)
                if (f < Spec::n_full(a) && ((pro_full >> f) & 1u)) {
                    s.fraw[f][0] = u32x4{0u, 0u, 0u, 0u};
                    if (valid_of(i)) s.fraw[f][0] = load_stream(a.full[f], ((uint64_t)pos * g.channels + cvi * VEC) * S::ESIZE);
                }
#pragma unroll
            for (int v = 0; v < Spec::NV; ++v)
                if (v < Spec::n_vec(a) && ((pro_vec >> v) & 1u)) {
                    s.vraw[v][0] = u32x4{0u, 0u, 0u, 0u};
                    if (valid_of(i)) s.vraw[v][0] = load_vec_operand<DT, Spec::kVecMode>(a.vec[v], pos, s.col[0], g.channels);
                }
            run_program<DT, 1, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStore{});
            if (valid_of(i)) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = pool_combine<OP>(acc[e], s.acc[e]);
            }
        }
    }

    // ---- the position steps of the workgroup, through LDS; lanes 0 .. cv - 1 end up with the slice's result
#pragma unroll
    for (int e = 0; e < VEC; ++e) lds[t * VEC + e] = acc[e];
    __syncthreads();
    const bool owner = t < g.cv;  // pstep 0: lane t holds channel vector t
    if (owner) {
        for (uint32_t q = 1; q < g.pos_per_step; ++q)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = pool_combine<OP>(acc[e], lds[(q * g.cv + t) * VEC + e]);
    }

    if (g.blocks_per_sample > 1u) {
        // ---- publish the slice's partial result, then raise the slice's flag.  The sample's LAST slice (dispatched
        // after the others) waits for all flags, merges, and lowers the flags again for the next launch.
        // (the slice's result goes through LDS once more so that consecutive lanes store consecutive words: a wave
        // then writes 256 contiguous bytes instead of 64 separate words)
        __syncthreads();
        if (owner) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) lds[t * VEC + e] = acc[e];
        }
        __syncthreads();
        float* part = g.ws_partial + (uint64_t)(sample * g.blocks_per_sample + bx) * g.channels;
        for (uint32_t idx = t; idx < g.channels; idx += 512u) __hip_atomic_store(part + idx, lds[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // The flag below must not become visible before these words.  They are device-coherent write-through stores,
        // so nothing has to be written back; what is needed is that every wave's stores have been acknowledged before
        // the barrier lets lane 0 raise the flag.  A workgroup-scope release does not wait for outstanding stores on
        // this device (a workgroup never leaves its compute unit), and an agent-scope one would write back the whole
        // L2: the wait is spelled out instead.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        uint32_t* flags = g.ws_flags + (uint64_t)sample * g.blocks_per_sample;
        if (t == 0) __hip_atomic_store(flags + bx, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (bx + 1u != g.blocks_per_sample) return;
        // every wait is bounded: after spin_limit rounds the error word is set and the merge goes ahead
        for (uint32_t spins = 0;; ++spins) {
            int pending = 0;
            for (uint32_t b = t; b < g.blocks_per_sample; b += 512u)
                pending |= __hip_atomic_load(flags + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u ? 1 : 0;
            if (!__syncthreads_or(pending)) break;
            if (spins >= g.spin_limit) {
                if (t == 0) __hip_atomic_store(g.ws_error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
        for (uint32_t b = t; b < g.blocks_per_sample; b += 512u) __hip_atomic_store(flags + b, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // one channel per lane (consecutive lanes, consecutive words), four slices in flight at a time
        const float* base = g.ws_partial + (uint64_t)sample * g.blocks_per_sample * g.channels;
        __syncthreads();
        for (uint32_t idx = t; idx < g.channels; idx += 512u) {
            float m = pool_identity<OP>();
            for (uint32_t b0 = 0; b0 < g.blocks_per_sample; b0 += 4u) {
                float part4[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t b = b0 + (uint32_t)u;
                    part4[u] = b < g.blocks_per_sample ? __hip_atomic_load(base + (uint64_t)b * g.channels + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                                       : pool_identity<OP>();
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) m = pool_combine<OP>(m, part4[u]);
            }
            lds[idx] = m;
        }
        __syncthreads();
        if (owner) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = lds[t * VEC + e];
        }
    }
    if (!owner) return;

    // ---- epilogue on the pooled values of (sample, channel vector t), addressed in the result's layout [n, c]
    if (OP == POOL_MEAN) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] *= g.inv_hw;
    }
    s.row[0] = sample;
    s.col[0] = t * VEC;
    const uint64_t out_off = ((uint64_t)sample * g.channels + t * VEC) * S::ESIZE;
#pragma unroll
    for (int f = 0; f < Spec::NF; ++f)
        if (f < Spec::n_full(a) && ((epi_full >> f) & 1u)) s.fraw[f][0] = load_cached(a.full[f], out_off);
#pragma unroll
    for (int v = 0; v < Spec::NV; ++v)
        if (v < Spec::n_vec(a) && ((epi_vec >> v) & 1u)) s.vraw[v][0] = load_vec_operand<DT, Spec::kVecMode>(a.vec[v], sample, s.col[0], g.channels);
#pragma unroll
    for (int e = 0; e < VEC; ++e) s.acc[e] = acc[e];
    run_program<DT, 1, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, NoStore{});
    store_stream(a.out[0], out_off, S::pack(s.acc));
}

}  // namespace pf
