// Pool family: prologue -> reduction over the positions of a channels-last tensor (sum, maximum or mean over
// every dimension between the first and the last: global pooling of x [n, spatial.., c] into [n, 1.., c]) ->
// epilogue on the pooled values.
//
// This is the reduce basic operator (paper section 6) along dimensions that are not contiguous in memory.  A
// workgroup walks whole positions, so its HBM accesses are fully contiguous, and every lane owns one channel
// vector, so the running reduction lives in registers and no value crosses lanes until the workgroup's slice
// is done (one pass through LDS).  A sample's positions are spread over several workgroups: each publishes its
// per-channel partial result; the sample's last workgroup waits for those words, merges them, runs the epilogue
// and stores -- the device-scope synchronisation of section 5.1.
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

// A partial result as a published word: all-ones means "not written in this launch" (a NaN that arithmetic never
// produces; a NaN result with that payload is published as the canonical one).
constexpr uint32_t kPoolEmpty = ~0u;
PF_DEVICE uint32_t pool_word(float x) {
    const uint32_t w = __builtin_bit_cast(uint32_t, x);
    return w == kPoolEmpty ? 0x7fc00000u : w;
}

// RAGGED: a channel count that is not a whole number of 16-byte vectors.  A position then starts at element alignment
// and its last vector holds `cnt` channels: elements past them are never read or stored (their accumulator slots carry
// whatever the prologue makes of the fill value and stay in the lane).
template <int DT, int NV, class Spec, int OP, bool RAGGED = false>
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
    const uint32_t cnt = RAGGED ? elems_below<VEC>(cvi * (uint32_t)VEC, g.channels) : (uint32_t)VEC;
    // (what follows a position's partial vector is the next position, unless it is the tensor's last)
    const uint64_t total_elems = (uint64_t)g.samples * g.hw * g.channels;
    auto load_full = [&](const void* base, uint64_t elem) {
        return RAGGED ? load_elems<DT>(base, elem, cnt, 0u, elem + (uint64_t)VEC <= total_elems) : load_stream(base, elem * S::ESIZE);
    };

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
        // (no branch around a load: a lane without a position at step i reads the slice's first vector and leaves it out
        // of the reduction.  Behind guards the compiler loses count of what is in flight and waits for all of the chunk's
        // loads before the first vector is worked on.)
        u32x4 raw[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const uint64_t elem = valid_of(i) ? (pos0 + rel_of(i)) * g.channels + cvi * VEC : pos0 * g.channels;
            raw[i] = load_full(a.full[0], elem);
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
                    if (valid_of(i)) s.fraw[f][0] = load_full(a.full[f], (uint64_t)pos * g.channels + cvi * VEC);
                }
#pragma unroll
            for (int v = 0; v < Spec::NV; ++v)
                if (v < Spec::n_vec(a) && ((pro_vec >> v) & 1u)) {
                    s.vraw[v][0] = u32x4{0u, 0u, 0u, 0u};
                    if (valid_of(i))
                        s.vraw[v][0] = RAGGED ? load_vec_operand_elems<DT, Spec::kVecMode>(a.vec[v], pos, s.col[0], g.channels, cnt)
                                              : load_vec_operand<DT, Spec::kVecMode>(a.vec[v], pos, s.col[0], g.channels);
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
        // ---- a sample split over several workgroups.  Every slice but the last publishes its per-channel partial
        // result as self-describing words (kPoolEmpty = not written in this launch); the sample's LAST slice
        // (dispatched after the others) reads them all, re-reading the ones still empty, puts them back to empty for
        // the next launch and merges.  The critical path is one coherent store followed by one coherent load: no
        // flag, no wait for the stores' acknowledgement in between.
        // (the slice's result goes through LDS so that consecutive lanes store consecutive words: a wave then writes
        // 256 contiguous bytes instead of 64 separate words)
        __syncthreads();
        if (owner) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) lds[t * VEC + e] = acc[e];
        }
        __syncthreads();
        if (bx + 1u != g.blocks_per_sample) {
            uint32_t* part = g.ws_partial + (uint64_t)(sample * g.blocks_per_sample + bx) * g.channels;
            for (uint32_t idx = t; idx < g.channels; idx += 512u)
                __hip_atomic_store(part + idx, pool_word(lds[idx]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        // The merger: merge_rows row groups of threads, each a channel per lane (consecutive lanes, consecutive words);
        // row group r takes the slices r, r + merge_rows, ..., eight of them in flight at a time.  Every wait is
        // bounded: after spin_limit re-reads the error word is set and the missing slice is left out.
        const uint32_t others = g.blocks_per_sample - 1u;
        const uint32_t r = t / g.channels;  // 0 for every thread when a position has 512 channels or more
        uint32_t* base = g.ws_partial + (uint64_t)sample * g.blocks_per_sample * g.channels;
        uint32_t spins = 0;
        float merged[VEC];  // (channels > 512: a thread owns channels t, t + 512, ...: at most VEC of them)
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const uint32_t idx = t - r * g.channels + (uint32_t)k * 512u;
            float m = pool_identity<OP>();
            if (r < g.merge_rows && idx < g.channels && (k == 0 || g.channels > 512u)) {
                if (r == 0u) m = lds[idx];  // the merger's own slice
                for (uint32_t b0 = r; b0 < others; b0 += 8u * g.merge_rows) {
                    uint32_t w[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const uint32_t b = b0 + (uint32_t)u * g.merge_rows;
                        w[u] = b < others ? __hip_atomic_load(base + (uint64_t)b * g.channels + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                          : pool_word(pool_identity<OP>());
                    }
                    // words still empty are re-read together (one trip to memory per round, not one per word)
                    for (;;) {
                        bool waiting = false;
#pragma unroll
                        for (int u = 0; u < 8; ++u) waiting = waiting || w[u] == kPoolEmpty;
                        if (!waiting) break;
                        if (++spins > g.spin_limit) {
                            __hip_atomic_store(g.ws_error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            break;
                        }
                        __builtin_amdgcn_s_sleep(8);
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const uint32_t b = b0 + (uint32_t)u * g.merge_rows;
                            if (w[u] == kPoolEmpty) w[u] = __hip_atomic_load(base + (uint64_t)b * g.channels + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const uint32_t b = b0 + (uint32_t)u * g.merge_rows;
                        if (b >= others || w[u] == kPoolEmpty) continue;
                        __hip_atomic_store(base + (uint64_t)b * g.channels + idx, kPoolEmpty, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        m = pool_combine<OP>(m, __builtin_bit_cast(float, w[u]));
                    }
                }
            }
            merged[k] = m;
        }
        __syncthreads();  // (everyone has read its own slice's values)
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const uint32_t idx = t - r * g.channels + (uint32_t)k * 512u;
            if (r < g.merge_rows && idx < g.channels && (k == 0 || g.channels > 512u)) lds[r * g.channels + idx] = merged[k];
        }
        __syncthreads();
        if (owner) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                float m = lds[t * VEC + e];
                for (uint32_t q = 1; q < g.merge_rows; ++q) m = pool_combine<OP>(m, lds[q * g.channels + t * VEC + e]);
                acc[e] = m;
            }
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
    const uint64_t out_elem = (uint64_t)sample * g.channels + t * VEC;
    const uint64_t out_off = out_elem * S::ESIZE;
#pragma unroll
    for (int f = 0; f < Spec::NF; ++f)
        if (f < Spec::n_full(a) && ((epi_full >> f) & 1u)) s.fraw[f][0] = RAGGED ? load_elems<DT>(a.full[f], out_elem, cnt, 0u) : load_cached(a.full[f], out_off);
#pragma unroll
    for (int v = 0; v < Spec::NV; ++v)
        if (v < Spec::n_vec(a) && ((epi_vec >> v) & 1u))
            s.vraw[v][0] = RAGGED ? load_vec_operand_elems<DT, Spec::kVecMode>(a.vec[v], sample, s.col[0], g.channels, cnt)
                                  : load_vec_operand<DT, Spec::kVecMode>(a.vec[v], sample, s.col[0], g.channels);
#pragma unroll
    for (int e = 0; e < VEC; ++e) s.acc[e] = acc[e];
    run_program<DT, 1, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, NoStore{});
    if (RAGGED) store_elems<DT>(a.out[0], out_elem, cnt, S::pack(s.acc));
    else store_stream(a.out[0], out_off, S::pack(s.acc));
}

}  // namespace pf
