// Group family: prologue -> GroupNorm on a channels-last tensor -> epilogue.
//
// A (sample, group) pair owns hw * (channels / groups) elements scattered as short pieces at a stride of
// one position (channels elements).  A workgroup walks whole positions, so its HBM accesses are fully
// contiguous; the price is that a group's statistics are spread over many workgroups and have to be
// exchanged at device scope -- the widest synchronisation scope of the paper's scheme (section 5.1), the
// one it pays a DRAM round trip for.  Two variants:
//
//   TWO_PASS  kernel 1 writes per-workgroup partial statistics, kernel 2 combines them and normalises.
//             x is read twice (the second read usually hits the last-level cache).
//   RESIDENT  one kernel.  Every workgroup keeps its slice of x in registers, publishes partial
//             statistics, waits on a per-sample arrival counter (device-scope release / acquire), combines
//             and normalises straight from registers.  x is read once: compulsory traffic only.
//
// Statistics are (count, mean, M2) triples merged with the parallel-variance update, each lane summing
// deviations from its first element, so a large common offset does not cancel catastrophically in fp32.
#include "pf_device.hpp"
#include "pf_launch.h"
#include "pf_row_kernels.hpp"
#include "pf_specs.h"

namespace pf {

struct Stat {
    float n, mean, m2;
};

PF_DEVICE Stat stat_merge(Stat a, Stat b) {
    const float n = a.n + b.n;
    const float inv = n > 0.0f ? 1.0f / n : 0.0f;
    const float delta = b.mean - a.mean;
    Stat r;
    r.n = n;
    r.mean = a.mean + delta * (b.n * inv);
    r.m2 = a.m2 + b.m2 + delta * delta * (a.n * b.n * inv);
    return r;
}

PF_DEVICE Stat stat_shfl_xor(Stat s, int mask) {
    Stat r;
    r.n = __shfl_xor(s.n, mask, 64);
    r.mean = __shfl_xor(s.mean, mask, 64);
    r.m2 = __shfl_xor(s.m2, mask, 64);
    return r;
}

// running sums of deviations from a pivot
struct LaneAcc {
    float n = 0.0f, s = 0.0f, ss = 0.0f, pivot = 0.0f;
    template <int VEC>
    PF_DEVICE void add_vector(const float* x) {
        if (n == 0.0f) pivot = x[0];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float d = x[e] - pivot;
            s += d;
            ss += d * d;
        }
        n += (float)VEC;
    }
    PF_DEVICE Stat finish() const {
        Stat r;
        r.n = n;
        const float inv = n > 0.0f ? 1.0f / n : 0.0f;
        r.mean = pivot + s * inv;
        r.m2 = fmaxf(ss - s * s * inv, 0.0f);
        return r;
    }
};

// lanes of one group are vpg adjacent lanes; afterwards the group's first lane holds the merged triple
PF_DEVICE Stat group_lanes_merge(Stat st, uint32_t log2_vpg) {
    for (uint32_t b = 0; b < log2_vpg; ++b) st = stat_merge(st, stat_shfl_xor(st, 1 << b));
    return st;
}

// workgroup partial: merge over the position steps of the workgroup and publish
PF_DEVICE void block_partial(const GroupGeom& g, Stat st, uint32_t pstep, uint32_t cvi, bool active, float* lds,
                             float* dst /* [groups][4] */) {
    const uint32_t grp = cvi >> g.log2_vpg;
    if (active && (cvi & (g.vpg - 1u)) == 0u) {
        float* p = lds + (pstep * g.groups + grp) * 3u;
        p[0] = st.n;
        p[1] = st.mean;
        p[2] = st.m2;
    }
    __syncthreads();
    if (threadIdx.x < g.groups) {
        Stat acc = {0.0f, 0.0f, 0.0f};
        for (uint32_t s = 0; s < g.pos_per_step; ++s) {
            const float* p = lds + (s * g.groups + threadIdx.x) * 3u;
            acc = stat_merge(acc, Stat{p[0], p[1], p[2]});
        }
        float* o = dst + threadIdx.x * 4u;
        o[0] = acc.n;
        o[1] = acc.mean;
        o[2] = acc.m2;
        o[3] = 0.0f;
        __threadfence();  // the partial must be visible device-wide before this workgroup signals arrival
    }
}

// merge the published partials of one sample; every workgroup does it for all groups.  The fetch is spread
// over the workgroup (one triple per lane) so its latency is paid once, then one lane per group merges
// from LDS.  blocks_per_sample * groups <= PF_GROUP_MAX_PARTIALS is guaranteed by the planner.
#define PF_GROUP_MAX_PARTIALS 2048
template <bool COHERENT>
PF_DEVICE void combine_sample(const GroupGeom& g, uint32_t sample, float eps, float* lds_part /* [partials][3] */,
                              float* lds_stat /* [groups][2] */) {
    const uint32_t n_part = g.blocks_per_sample * g.groups;
    const float* base = g.ws_partial + (uint64_t)sample * n_part * 4u;
    for (uint32_t i = threadIdx.x; i < n_part; i += blockDim.x) {
        const float* p = base + (uint64_t)i * 4u;
        float n, mean, m2;
        if (COHERENT) {
            n = __hip_atomic_load(p + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            mean = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            m2 = __hip_atomic_load(p + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            n = p[0];
            mean = p[1];
            m2 = p[2];
        }
        lds_part[i * 3u] = n;
        lds_part[i * 3u + 1u] = mean;
        lds_part[i * 3u + 2u] = m2;
    }
    __syncthreads();
    if (threadIdx.x < g.groups) {
        Stat acc = {0.0f, 0.0f, 0.0f};
        for (uint32_t b = 0; b < g.blocks_per_sample; ++b) {
            const float* p = lds_part + (b * g.groups + threadIdx.x) * 3u;
            acc = stat_merge(acc, Stat{p[0], p[1], p[2]});
        }
        const float var = acc.n > 0.0f ? acc.m2 / acc.n : 0.0f;
        lds_stat[threadIdx.x * 2u] = acc.mean;
        lds_stat[threadIdx.x * 2u + 1u] = 1.0f / sqrtf(var + eps);
    }
    __syncthreads();
}

template <int DT, int K, class Spec>
PF_DEVICE void group_load(const ChainArgs& a, const GroupGeom& g, LaneState<DT, K, Spec>& s, uint32_t sample, const uint32_t* pos,
                          uint32_t cvi, const bool* valid) {
    using S = Storage<DT>;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        s.row[k] = sample * g.hw + pos[k];
        s.col[k] = cvi * S::VEC;
    }
#pragma unroll
    for (int f = 0; f < Spec::NF; ++f) {
        if (f < Spec::n_full(a)) {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                s.fraw[f][k] = u32x4{0u, 0u, 0u, 0u};
                if (valid[k])
                    s.fraw[f][k] = load_stream(a.full[f], ((uint64_t)s.row[k] * g.channels + s.col[k]) * S::ESIZE);
            }
        }
    }
#pragma unroll
    for (int v = 0; v < Spec::NV; ++v) {
        if (v < Spec::n_vec(a)) {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                s.vraw[v][k] = u32x4{0u, 0u, 0u, 0u};
                if (valid[k]) s.vraw[v][k] = load_vec_operand<DT>(a.vec[v], s.row[k], s.col[k], g.channels);
            }
        }
    }
}

template <int DT, int K, class Spec>
PF_DEVICE void group_normalise(const ChainArgs& a, const GroupGeom& g, LaneState<DT, K, Spec>& s, uint32_t cvi, const float* lds_stat) {
    constexpr int E = LaneState<DT, K, Spec>::E;
    const uint32_t grp = cvi >> g.log2_vpg;
    const float mean = lds_stat[grp * 2u], rstd = lds_stat[grp * 2u + 1u];
    float gm[E], bt[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        gm[e] = 1.0f;
        bt[e] = 0.0f;
    }
    if (Spec::gamma(a) >= 0) fetch_vec<DT, K, Spec>(s, Spec::gamma(a), gm);
    if (Spec::beta(a) >= 0) fetch_vec<DT, K, Spec>(s, Spec::beta(a), bt);
#pragma unroll
    for (int e = 0; e < E; ++e) s.acc[e] = (s.acc[e] - mean) * rstd * gm[e] + bt[e];
}

// ---- two-pass, kernel 1: partial statistics
template <int DT, int K, class Spec>
__global__ void __launch_bounds__(1024) group_stats_kernel(const ChainArgs a, const GroupGeom g) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    __shared__ float g_lds_part[1024 * 3];
    const uint32_t t = threadIdx.x;
    const uint32_t pstep = fast_div(t, g.div_cv);
    const uint32_t cvi = t - pstep * g.cv;
    const bool active = pstep < g.pos_per_step;
    const uint32_t sample = blockIdx.y;
    const uint32_t p_begin = blockIdx.x * g.pos_per_block;
    const uint32_t p_end = min(g.hw, p_begin + g.pos_per_block);
    LaneAcc la;
    LaneState<DT, K, Spec> s;
    for (uint32_t p0 = p_begin; p0 < p_end; p0 += g.pos_per_step * K) {  // uniform trip count
        uint32_t pos[K];
        bool valid[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            pos[k] = p0 + pstep + k * g.pos_per_step;
            valid[k] = active && pos[k] < p_end;
        }
        group_load<DT, K, Spec>(a, g, s, sample, pos, cvi, valid);
        run_program<DT, K, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStore{});
#pragma unroll
        for (int k = 0; k < K; ++k)
            if (valid[k]) la.template add_vector<VEC>(s.acc + k * VEC);
    }
    const Stat st = group_lanes_merge(la.finish(), g.log2_vpg);
    float* dst = g.ws_partial + ((uint64_t)(sample * g.blocks_per_sample + blockIdx.x) * g.groups) * 4u;
    block_partial(g, st, pstep, cvi, active, g_lds_part, dst);
}

// ---- two-pass, kernel 2: combine and normalise
template <int DT, int K, class Spec>
__global__ void __launch_bounds__(1024) group_apply_kernel(const ChainArgs a, const GroupGeom g) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    __shared__ float g_lds_part[PF_GROUP_MAX_PARTIALS * 3];
    __shared__ float g_lds_stat[1024 * 2];
    const uint32_t t = threadIdx.x;
    const uint32_t pstep = fast_div(t, g.div_cv);
    const uint32_t cvi = t - pstep * g.cv;
    const bool active = pstep < g.pos_per_step;
    const uint32_t sample = blockIdx.y;
    const uint32_t p_begin = blockIdx.x * g.pos_per_block;
    const uint32_t p_end = min(g.hw, p_begin + g.pos_per_block);
    combine_sample<false>(g, sample, a.eps, g_lds_part, g_lds_stat);
    LaneState<DT, K, Spec> s;
    for (uint32_t p0 = p_begin; p0 < p_end; p0 += g.pos_per_step * K) {
        uint32_t pos[K];
        bool valid[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            pos[k] = p0 + pstep + k * g.pos_per_step;
            valid[k] = active && pos[k] < p_end;
        }
        group_load<DT, K, Spec>(a, g, s, sample, pos, cvi, valid);
        run_program<DT, K, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStore{});
        group_normalise<DT, K, Spec>(a, g, s, cvi, g_lds_stat);
        run_program<DT, K, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, NoStore{});
#pragma unroll
        for (int k = 0; k < K; ++k)
            if (valid[k])
                store_stream(a.out[0], ((uint64_t)s.row[k] * g.channels + s.col[k]) * S::ESIZE, S::pack(s.acc + k * VEC));
    }
}

// ---- resident: one kernel, x stays in registers across the device-scope exchange.
// Requirements checked by the planner: one full operand; the workgroup's NV position steps cover its
// whole slice; all workgroups of a launch are co-resident (the grid is sized to what the device holds
// and a workgroup loops over its tiles), so every wait below ends.  The wait is bounded anyway: when
// spin_limit polls pass without the counter arriving, the error word is set and the kernel carries on.
template <int DT, int NV, class Spec>
__global__ void __launch_bounds__(1024) group_resident_kernel(const ChainArgs a, const GroupGeom g, const uint32_t tiles,
                                                              const uint32_t tiles_per_round) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    __shared__ float g_lds_part[PF_GROUP_MAX_PARTIALS * 3];
    __shared__ float g_lds_stat[1024 * 2];
    const uint32_t t = threadIdx.x;
    const uint32_t pstep = fast_div(t, g.div_cv);
    const uint32_t cvi = t - pstep * g.cv;
    const bool active = pstep < g.pos_per_step;
    uint32_t round = 0;
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += tiles_per_round, ++round) {
        const uint32_t sample = tile / g.blocks_per_sample;
        const uint32_t bx = tile - sample * g.blocks_per_sample;
        const uint32_t p_begin = bx * g.pos_per_block;
        const uint32_t p_end = min(g.hw, p_begin + g.pos_per_block);
        // ---- the whole slice into registers, every load issued before the first use
        u32x4 raw[NV];
        bool valid[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const uint32_t pos = p_begin + pstep + i * g.pos_per_step;
            valid[i] = active && pos < p_end;
            raw[i] = u32x4{0u, 0u, 0u, 0u};
            if (valid[i])
                raw[i] = load_stream(a.full[0], ((uint64_t)(sample * g.hw + pos) * g.channels + cvi * VEC) * S::ESIZE);
        }
        LaneState<DT, 1, Spec> s;
        s.col[0] = cvi * VEC;
#pragma unroll
        for (int v = 0; v < Spec::NV; ++v) {
            if (v < Spec::n_vec(a)) {
                // broadcast operands of this family are per channel: the same vector for every position
                s.vraw[v][0] = u32x4{0u, 0u, 0u, 0u};
                if (active) s.vraw[v][0] = load_vec_operand<DT>(a.vec[v], 0u, s.col[0], g.channels);
            }
        }
        // ---- partial statistics from registers
        LaneAcc la;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            s.row[0] = sample * g.hw + p_begin + pstep + i * g.pos_per_step;
            s.fraw[0][0] = raw[i];
            run_program<DT, 1, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStore{});
            if (valid[i]) la.template add_vector<VEC>(s.acc);
        }
        const Stat st = group_lanes_merge(la.finish(), g.log2_vpg);
        float* dst = g.ws_partial + ((uint64_t)(sample * g.blocks_per_sample + bx) * g.groups) * 4u;
        block_partial(g, st, pstep, cvi, active, g_lds_part, dst);
        // ---- device-scope exchange: publish, arrive, wait for the sample's other workgroups
        __syncthreads();  // all partial stores of this workgroup are issued
        if (t == 0) {
            __hip_atomic_fetch_add(g.ws_counter + sample, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
            const uint32_t target = g.epoch * g.blocks_per_sample;
            uint32_t spins = 0;
            while ((int32_t)(__hip_atomic_load(g.ws_counter + sample, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
                if (++spins >= g.spin_limit) {
                    __hip_atomic_store(g.ws_error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(8);
            }
        }
        __syncthreads();
        combine_sample<true>(g, sample, a.eps, g_lds_part, g_lds_stat);
        // ---- normalise straight from registers
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            s.row[0] = sample * g.hw + p_begin + pstep + i * g.pos_per_step;
            s.fraw[0][0] = raw[i];
            run_program<DT, 1, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStore{});
            group_normalise<DT, 1, Spec>(a, g, s, cvi, g_lds_stat);
            run_program<DT, 1, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, NoStore{});
            if (valid[i])
                store_stream(a.out[0], ((uint64_t)s.row[0] * g.channels + s.col[0]) * S::ESIZE, S::pack(s.acc));
        }
        __syncthreads();  // LDS staging is reused by the next tile
    }
}

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

template <int ID, int DT>
static hipError_t launch_group_dt(int which, const ChainArgs& a, const GroupGeom& g, int nv, uint32_t tiles, dim3 grid,
                                  dim3 block, hipStream_t st) {
    using Spec = typename GroupSpecOf<ID>::type;
    if (which == 0) hipLaunchKernelGGL((group_stats_kernel<DT, 2, Spec>), grid, block, 0, st, a, g);
    else if (which == 1) hipLaunchKernelGGL((group_apply_kernel<DT, 2, Spec>), grid, block, 0, st, a, g);
    else {
        if (ID == 0) return hipErrorInvalidValue;  // the resident variant exists for catalogue entries only
        if constexpr (ID != 0) {
            switch (nv) {
                case 4: hipLaunchKernelGGL((group_resident_kernel<DT, 4, Spec>), grid, block, 0, st, a, g, tiles, grid.x); break;
                case 8: hipLaunchKernelGGL((group_resident_kernel<DT, 8, Spec>), grid, block, 0, st, a, g, tiles, grid.x); break;
                case 16: hipLaunchKernelGGL((group_resident_kernel<DT, 16, Spec>), grid, block, 0, st, a, g, tiles, grid.x); break;
                default: return hipErrorInvalidValue;
            }
        }
    }
    return hipGetLastError();
}

template <int ID>
static hipError_t launch_group_id(int which, int dtype, const ChainArgs& a, const GroupGeom& g, int nv, uint32_t tiles,
                                  dim3 grid, dim3 block, hipStream_t st) {
    switch (dtype) {
        case DT_F32: return launch_group_dt<ID, DT_F32>(which, a, g, nv, tiles, grid, block, st);
        case DT_F16: return launch_group_dt<ID, DT_F16>(which, a, g, nv, tiles, grid, block, st);
        case DT_BF16: return launch_group_dt<ID, DT_BF16>(which, a, g, nv, tiles, grid, block, st);
        default: return hipErrorInvalidValue;
    }
}

static hipError_t launch_group_any(int which, int spec_id, int dtype, const ChainArgs& a, const GroupGeom& g, int nv,
                                   uint32_t tiles, dim3 grid, dim3 block, hipStream_t st) {
    switch (spec_id) {
        case 0: return launch_group_id<0>(which, dtype, a, g, nv, tiles, grid, block, st);
#define PF_CASE(id, ...) \
    case id: return launch_group_id<id>(which, dtype, a, g, nv, tiles, grid, block, st);
            PF_GROUP_SPECS(PF_CASE)
#undef PF_CASE
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_group_stats(int spec_id, int dtype, const ChainArgs& a, const GroupGeom& g, dim3 grid, dim3 block, hipStream_t st) {
    return launch_group_any(0, spec_id, dtype, a, g, 0, 0, grid, block, st);
}
hipError_t launch_group_apply(int spec_id, int dtype, const ChainArgs& a, const GroupGeom& g, dim3 grid, dim3 block, hipStream_t st) {
    return launch_group_any(1, spec_id, dtype, a, g, 0, 0, grid, block, st);
}
hipError_t launch_group_resident(int spec_id, int dtype, const ChainArgs& a, const GroupGeom& g, int nv, uint32_t tiles, dim3 grid,
                                 dim3 block, hipStream_t st) {
    return launch_group_any(2, spec_id, dtype, a, g, nv, tiles, grid, block, st);
}

// how many workgroups of the resident kernel one compute unit holds (for sizing a co-resident grid)
int group_resident_blocks_per_cu(int spec_id, int dtype, int nv, int block_threads) {
    int n = 0;
#define PF_OCC(ID, DT, NVV)                                                                                          \
    if (spec_id == ID && dtype == DT && nv == NVV)                                                                   \
        (void)hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, group_resident_kernel<DT, NVV, typename GroupSpecOf<ID>::type>, \
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
