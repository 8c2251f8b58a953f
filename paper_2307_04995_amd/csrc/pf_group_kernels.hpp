// Group family: prologue -> GroupNorm on a channels-last tensor -> epilogue.
//
// A (sample, group) pair owns hw * (channels / groups) elements scattered as short pieces at a stride of
// one position (channels elements).  A workgroup walks whole positions, so its HBM accesses are fully
// contiguous; the price is that a group's statistics are spread over many workgroups and have to be
// exchanged at device scope -- the widest synchronisation scope of the paper's scheme (section 5.1), the
// one it pays a DRAM round trip for.  Two variants:
//
//   TWO_PASS  launch 1 writes per-workgroup partial statistics, launch 2 merges them and normalises.
//             x is read twice (the second read usually hits the last-level cache).
//   RESIDENT  one launch.  Every workgroup keeps its slice of x in registers, publishes partial
//             statistics, takes part in a per-sample device-scope exchange and normalises straight from
//             registers.  x is read once: compulsory traffic only.
//
// Statistics are (count, mean, M2) triples merged with the parallel-variance update.  A lane reduces each of
// its vectors on its own (mean, then squared deviations from it) before merging, so neither a large common
// offset nor a spread that is tiny against the values cancels in fp32.
#pragma once
#include "pf_row_kernels.hpp"

namespace pf {

// Statistics straight from the packed 16-bit vector, without widening every element: two dot-product
// instructions per pair of elements accumulate the sum and the sum of squares in fp32.  Products of 16-bit
// values are exact in fp32 and a lane sums at most a few dozen elements, so the only cancellation left is
// in the lane's own M2 = ss - s^2/n, whose relative error is about 1e-7 * mean^2 / var: harmless for any
// offset a 16-bit type can carry over its spread (beyond mean/std of a few hundred the storage type itself
// cannot resolve the spread).  Lanes are then merged with the offset-safe parallel-variance update.
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// plain sums for the packed statistics below
struct LeanAcc {
    float n = 0.0f, s = 0.0f, ss = 0.0f;
    PF_DEVICE Stat finish() const {
        const float inv = n > 0.0f ? 1.0f / n : 0.0f;
        return Stat{n, s * inv, fmaxf(ss - s * s * inv, 0.0f)};
    }
};

template <int DT>
PF_DEVICE void lean_add_vector(LeanAcc& la, u32x4 raw) {
    if (DT == DT_F16) {
        const f16x2 ones = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t w = raw[j];  // (a bit cast applied directly to a vector element is miscompiled)
            const f16x2 x = __builtin_bit_cast(f16x2, w);
            la.s = __builtin_amdgcn_fdot2(x, ones, la.s, false);
            la.ss = __builtin_amdgcn_fdot2(x, x, la.ss, false);
        }
    } else {
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t w = raw[j];
            const bf16x2 x = __builtin_bit_cast(bf16x2, w);
            la.s = __builtin_amdgcn_fdot2_f32_bf16(x, ones, la.s, false);
            la.ss = __builtin_amdgcn_fdot2_f32_bf16(x, x, la.ss, false);
        }
    }
    la.n += 8.0f;
}

// lanes of one group are vpg adjacent lanes; afterwards the group's first lane holds the merged triple
PF_DEVICE Stat group_lanes_merge(Stat st, uint32_t log2_vpg) {
    for (uint32_t b = 0; b < log2_vpg; ++b) st = stat_merge(st, stat_shfl_xor(st, 1 << b));
    return st;
}

// workgroup partial of the two-launch variant: merge over the position steps of the workgroup and write
// [groups][4] floats for the second launch
PF_DEVICE void block_partial(const GroupGeom& g, Stat st, uint32_t pstep, uint32_t cvi, bool active, float* lds, float* dst) {
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
    }
}

// Merge the partials a previous launch wrote for one sample into (mean, rstd) per group.  lanes_per_group (a power of
// two, <= 64) adjacent lanes share a group: each merges a strided subset of the sample's partials straight
// from memory, then the lanes are merged by a shuffle tree.  Returns true in the lane that holds a group's
// result (its group index in *grp_out).
PF_DEVICE bool combine_sample(const GroupGeom& g, uint32_t sample, float eps, uint32_t* grp_out, float* mean_out, float* rstd_out) {
    const uint32_t lpg = g.lanes_per_group;
    const uint32_t grp = threadIdx.x / lpg, j = threadIdx.x - grp * lpg;
    const bool in_range = grp < g.groups;
    const float* base = g.ws_partial + ((uint64_t)sample * g.blocks_per_sample * g.groups + (in_range ? grp : 0u)) * 4u;
    Stat acc = {0.0f, 0.0f, 0.0f};
    for (uint32_t b = j; b < g.blocks_per_sample; b += lpg) {
        const float* p = base + (uint64_t)b * g.groups * 4u;
        Stat q = {0.0f, 0.0f, 0.0f};
        if (in_range) {
            q.n = p[0];
            q.mean = p[1];
            q.m2 = p[2];
        }
        acc = stat_merge(acc, q);
    }
    for (uint32_t m = 1; m < lpg; m <<= 1) acc = stat_merge(acc, stat_shfl_xor(acc, (int)m));
    const float var = acc.n > 0.0f ? acc.m2 / acc.n : 0.0f;
    *grp_out = grp;
    *mean_out = acc.mean;
    *rstd_out = 1.0f / sqrtf(var + eps);
    return in_range && j == 0u;
}

// ---- device-scope exchange of the fused kernel: an all-gather of self-describing words ----------------
// A workgroup publishes, per group, ONE 8-byte word (mean, M2) of its tile (the count follows from the tile's
// position in the sample) into a slot of its own, with a device-coherent store.  A slot that still reads
// all-ones has not been written in this launch.  Every workgroup of the sample then reads all slots of the
// sample itself, re-reading the ones that are still empty, and merges them: the critical path is one
// coherent store followed by one coherent load, with no counter, no elected merger and no second
// publish/poll round trip behind it.  Slots exist twice, selected by the parity of the launch number; a
// workgroup re-arms its slots of the other parity, which nobody reads before the next launch.
constexpr uint64_t kSlotEmpty = ~0ull;  // (NaN, NaN) with an all-ones payload: arithmetic never produces it

PF_DEVICE uint64_t pack_slot(float mean, float m2) {
    uint64_t w = (uint64_t)__builtin_bit_cast(uint32_t, mean) | ((uint64_t)__builtin_bit_cast(uint32_t, m2) << 32);
    if (w == kSlotEmpty) w = 0x7fc000007fc00000ull;  // keep NaN statistics distinguishable from "empty"
    return w;
}

// LDS-merge the position steps of the workgroup, then publish one word per group.
PF_DEVICE void publish_tile(const GroupGeom& g, Stat st, uint32_t pstep, uint32_t cvi, bool active, float* lds, uint32_t sample,
                            uint32_t bx) {
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
        const uint64_t per_parity = (uint64_t)g.samples * g.groups * g.blocks_per_sample;
        const uint64_t slot = ((uint64_t)sample * g.groups + threadIdx.x) * g.blocks_per_sample + bx;
        const uint32_t par = g.epoch & 1u;
        __hip_atomic_store(g.ws_gather + (par ^ 1u) * per_parity + slot, kSlotEmpty, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(g.ws_gather + par * per_parity + slot, pack_slot(acc.mean, acc.m2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Gather and merge the words of one sample.  Thread mapping as in combine_sample: lanes_per_group adjacent
// lanes share a group, each takes a strided subset of the sample's tiles.  Every wait is bounded: after
// spin_limit re-reads the error word is set and the tile is left out.
PF_DEVICE bool gather_sample(const GroupGeom& g, uint32_t sample, float eps, uint32_t* grp_out, float* mean_out, float* rstd_out) {
    const uint32_t lpg = g.lanes_per_group;
    const uint32_t grp = threadIdx.x / lpg, j = threadIdx.x - grp * lpg;
    const bool in_range = grp < g.groups;
    const uint64_t per_parity = (uint64_t)g.samples * g.groups * g.blocks_per_sample;
    const uint64_t* base = g.ws_gather + (g.epoch & 1u) * per_parity + ((uint64_t)sample * g.groups + (in_range ? grp : 0u)) * g.blocks_per_sample;
    const float per_pos = (float)(g.channels / g.groups);
    Stat acc = {0.0f, 0.0f, 0.0f};
    uint32_t spins = 0;
    for (uint32_t b = j; b < g.blocks_per_sample; b += lpg) {
        if (!in_range) break;
        uint64_t w;
        for (;;) {
            w = __hip_atomic_load(base + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (w != kSlotEmpty) break;
            if (++spins >= g.spin_limit) {
                __hip_atomic_store(g.ws_error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
        if (w == kSlotEmpty) continue;
        const uint32_t p0 = b * g.pos_per_block;
        Stat q;
        q.n = (float)(min(g.hw, p0 + g.pos_per_block) - p0) * per_pos;
        q.mean = __builtin_bit_cast(float, (uint32_t)w);
        q.m2 = __builtin_bit_cast(float, (uint32_t)(w >> 32));
        acc = stat_merge(acc, q);
    }
    for (uint32_t m = 1; m < lpg; m <<= 1) acc = stat_merge(acc, stat_shfl_xor(acc, (int)m));
    const float var = acc.n > 0.0f ? acc.m2 / acc.n : 0.0f;
    *grp_out = grp;
    *mean_out = acc.mean;
    *rstd_out = 1.0f / sqrtf(var + eps);
    return in_range && j == 0u;
}

// ---- groups of any width (GEN instantiations) ---------------------------------------------------------
// When the channels of a group are not a power-of-two number of whole 16-byte vectors (10 channels per group
// in a 320-channel layer, 4 in a 128-channel one), a lane's vector can straddle groups and the lanes of a
// group are no aligned power-of-two run.  Every lane then keeps a running (mean, M2) per element slot over its
// positions, merges the slots of each part (one part per group its vector touches; they are adjacent) and parks
// one (count, mean, M2) triple per part in LDS; the triples of a group are merged by lanes_per_group threads
// that walk the lanes whose vectors touch that group.
// Returns true in the thread that ends up with group *grp_out's merged triple.
template <int VEC>
PF_DEVICE bool merge_parts_of_block(const GroupGeom& g, const float* lds_gen, uint32_t* grp_out, Stat* out) {
    const uint32_t lpg = g.lanes_per_group;
    const uint32_t grp = threadIdx.x / lpg, j = threadIdx.x - grp * lpg;
    const bool in_range = grp < g.groups;
    Stat acc = {0.0f, 0.0f, 0.0f};
    if (in_range) {
        const uint32_t cv_lo = (grp * g.cpg) / (uint32_t)VEC, cv_hi = ((grp + 1u) * g.cpg - 1u) / (uint32_t)VEC;
        const uint32_t ncv = cv_hi - cv_lo + 1u, entries = ncv * g.pos_per_step;
        for (uint32_t idx = j; idx < entries; idx += lpg) {
            const uint32_t ps = idx / ncv, cvx = cv_lo + (idx - ps * ncv);
            const uint32_t part = grp - fast_div(cvx * (uint32_t)VEC, g.div_cpg);
            const float* q = lds_gen + ((ps * g.cv + cvx) * g.parts + part) * 3u;
            acc = stat_merge(acc, Stat{q[0], q[1], q[2]});
        }
    }
    for (uint32_t m = 1; m < lpg; m <<= 1) acc = stat_merge(acc, stat_shfl_xor(acc, (int)m));
    *grp_out = grp;
    *out = acc;
    return in_range && j == 0u;
}

// One kernel template, three phases:
//   PHASE 0  fused: statistics, device-scope exchange and normalisation in one launch (RESIDENT variant)
//   PHASE 1  statistics only: writes the workgroup partials               (TWO_PASS, first launch)
//   PHASE 2  normalisation only: re-reads x, merges the partials itself   (TWO_PASS, second launch)
//
// A workgroup owns tiles blockIdx.x, blockIdx.x + gridDim.x, ... of NV position steps each; a lane holds NV
// 16-byte vectors of x in registers, all loads issued before the first use.  Workgroups start at different
// steps of their slice (register i holds step (i + rot) mod NV): all slices begin at multiples of the same
// power of two, and walking them in lockstep would keep every workgroup on the same few HBM channels.
//
// PHASE 0 requirements, checked by the planner: one full operand, per-channel broadcast operands only, and
// all workgroups of a launch co-resident (the grid is sized to what the device holds and is a multiple of
// the workgroups per sample), so every wait below ends.  Waits are bounded anyway: after spin_limit polls the
// error word is set and the kernel carries on.
//
// Exchange of PHASE 0: see publish_tile / gather_sample above.  All shared words travel by device-coherent
// (agent-scope atomic) accesses, so no cache write-back or invalidate is needed around them -- a write-back
// here would wait for every output line other workgroups have just stored.
//
// GEN != 0: groups of any width (see merge_parts_of_block; 2 and 3 are described at their use); needs 512 * parts * 12 bytes of dynamic LDS, `parts`
// being the most groups one vector touches.
// GC: RuntimeGroupGeom ("read the geometry argument"), or a type generated when the plan is made that holds the
// launch's geometry as constants: every tile is then known to be whole and every lane in use, so the loads and stores
// of a tile carry no test, and the index arithmetic folds.
struct RuntimeGroupGeom {
    static constexpr bool kConst = false;
};
template <int DT, int NV, class Spec, int PHASE, int GEN = 0, class GC = RuntimeGroupGeom>
__global__ void __launch_bounds__(512, 4) group_kernel(const ChainArgs a, const GroupGeom g_arg, const uint32_t tiles_arg) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    GroupGeom g = g_arg;
    uint32_t tiles = tiles_arg;
    bool whole_tiles = false, all_active = false, one_tile = false;
    if constexpr (GC::kConst) {
        g.samples = GC::samples;
        g.hw = GC::hw;
        g.channels = GC::channels;
        g.groups = GC::groups;
        g.cv = GC::cv;
        g.vpg = GC::vpg;
        g.log2_vpg = GC::log2_vpg;
        g.pos_per_step = GC::pos_per_step;
        g.pos_per_block = GC::pos_per_block;
        g.lanes_per_group = GC::lanes_per_group;
        g.blocks_per_sample = GC::blocks_per_sample;
        tiles = GC::tiles;
        whole_tiles = GC::hw % GC::pos_per_block == 0u;
        all_active = GC::cv * GC::pos_per_step == GC::threads;
        one_tile = GC::grid == GC::tiles;
    }
    // kLean: 16-bit storage and nothing but the load in front of the normalisation
    constexpr bool kLean = Spec::kStatic && Spec::Pro::n == 1 && DT != DT_F32 && !GEN;
    // GEN == 2: the same for the general kernels, planned when a group holds an even number of channels
    // (GEN == 4: the same with a channel count that is not a whole number of vectors)
    constexpr bool kLeanGen = (GEN == 2 || GEN == 4) && Spec::kStatic && Spec::Pro::n == 1 && DT != DT_F32;
    __shared__ float lds_part[GEN ? 1 : 512 * 3];
    __shared__ float lds_stat[512 * 2];
    extern __shared__ float lds_gen[];  // GEN: [lane][part] (count, mean, M2)
    const uint32_t t = threadIdx.x;
    uint32_t pstep;
    if constexpr (GC::kConst) pstep = t / GC::cv;
    else pstep = fast_div(t, g.div_cv);
    const uint32_t cvi = t - pstep * g.cv;
    const bool active = all_active || pstep < g.pos_per_step;
    // GEN: the part (group, relative to the lane's first group) each element of the lane's vector belongs to,
    // four bits per element
    uint32_t part_code = 0, first_grp = 0;
    // GEN == 3: general kernels for channel counts that are not whole vectors: a position then starts at element
    // alignment and its last vector holds `cnt` channels (elements past them are never read, counted or stored)
    constexpr bool ragged = GEN == 3 || GEN == 4;
    const uint32_t cnt = ragged ? elems_below<VEC>(cvi * (uint32_t)VEC, g.channels) : (uint32_t)VEC;
    if (GEN) {
        first_grp = fast_div(cvi * (uint32_t)VEC, g.div_cpg);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const uint32_t ch = min(cvi * (uint32_t)VEC + (uint32_t)e, g.channels - 1u);  // (slots past the last channel: its part, count 0)
            part_code |= (fast_div(ch, g.div_cpg) - first_grp) << (4 * e);
        }
    }
    auto part_of = [&](int e) { return (part_code >> (4 * e)) & 15u; };

    // The fused kernel is only planned for per-channel broadcast operands; making that a compile-time fact keeps
    // the per-position operand loads (and the waits the compiler puts at their control-flow joins, which would
    // also wait for every output store just issued) out of its loops.
    const bool vec_per_channel = PHASE == 0 ? true : g.vec_per_channel != 0u;

    LaneState<DT, 1, Spec> s;
    s.col[0] = cvi * VEC;
    // broadcast operands that are per channel: the same vector for every position and tile.  The one-launch kernel
    // asks for them behind its tile's loads (they come back in order, so in front of them they would hold up the first
    // byte of the tile by a trip to memory; they are first needed when the tile is complete anyway).
    auto load_channel_operands = [&]() {
#pragma unroll
        for (int v = 0; v < Spec::NV; ++v) {
            if (v < Spec::n_vec(a)) {
                s.vraw[v][0] = u32x4{0u, 0u, 0u, 0u};
                if (active)
                    s.vraw[v][0] = ragged ? load_vec_operand_elems<DT, Spec::kVecMode>(a.vec[v], 0u, s.col[0], g.channels, cnt)
                                          : load_vec_operand<DT, Spec::kVecMode>(a.vec[v], 0u, s.col[0], g.channels);
            }
        }
    };
    if (vec_per_channel && PHASE != 0) load_channel_operands();

    for (uint32_t tile = blockIdx.x; tile < tiles; tile += (one_tile ? tiles : gridDim.x)) {
        const uint32_t sample = tile / g.blocks_per_sample;
        const uint32_t bx = tile - sample * g.blocks_per_sample;
        const uint32_t p_begin = bx * g.pos_per_block;
        const uint32_t p_end = min(g.hw, p_begin + g.pos_per_block);

        // ---- the whole slice into registers (positions and validity are recomputed where needed rather than
        // kept: the registers are for data)
        u32x4 raw[NV];
        const uint32_t rot = tile % NV;
        const uint32_t p_count = whole_tiles ? g.pos_per_block : p_end - p_begin;
        auto rel_of = [&](int i) { return pstep + (((uint32_t)i + rot) % NV) * g.pos_per_step; };
        auto valid_of = [&](int i) { return (whole_tiles && all_active) || (active && rel_of(i) < p_count); };
        // A vector's address = the tile's base + the step's share (the same for the whole workgroup: scalar registers)
        // + the lane's share (the same for every step: one vector register).  Written so on purpose: one offset register
        // per step, sixteen of them live from the loads to the stores, is what made the kernel spill.
        const uint32_t step_bytes = g.pos_per_step * g.channels * (uint32_t)S::ESIZE;
        const uint32_t lane_bytes = (pstep * g.channels + cvi * VEC) * (uint32_t)S::ESIZE;
        auto step_of = [&](int i) { return ((uint32_t)i + rot) % NV; };
        const char* in_base = static_cast<const char*>(a.full[0]) + ((uint64_t)sample * g.hw + p_begin) * g.channels * S::ESIZE;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            if (ragged) {
                raw[i] = u32x4{0u, 0u, 0u, 0u};
                // (what follows a position's partial vector is the next position, unless it is the tensor's last)
                // (addressed like the whole-vector tiles: a scalar base per step plus one lane offset)
                if (valid_of(i))
                    raw[i] = load_elems<DT>(in_base + (size_t)step_of(i) * step_bytes, lane_bytes / (uint32_t)S::ESIZE, cnt, 0u,
                                            (uint64_t)sample * g.hw + p_begin + rel_of(i) + 1u < (uint64_t)g.samples * g.hw);
                continue;
            }
            // No branch around a load: a step wholly past the tile's end reads step 0 instead, a lane without a position
            // at this step the step's first vector, and what they read is left out of the statistics and never stored.
            // (Behind guards the compiler loses count of what is in flight and waits for every load of the tile before it
            // works on the first.)
            const bool sure = whole_tiles && all_active;
            const uint32_t st = (sure || step_of(i) * g.pos_per_step < p_count) ? step_of(i) : 0u;
            const uint32_t lo = (sure || valid_of(i)) ? lane_bytes : 0u;
            // (the statistics launch leaves x in the caches for the launch that re-reads it: C5 in two launches
            // 39.2 -> 35.2 us; a one-launch tile is touched once and streams past them)
            if (PHASE == 1) raw[i] = load_cached(in_base + (size_t)st * step_bytes, (uint64_t)lo);
            else raw[i] = load_stream(in_base + (size_t)st * step_bytes, lo);
        }

        if (PHASE == 0) load_channel_operands();

        // Run the prologue on slice i (lean chains have none).
        auto prologue = [&](int i) {
            s.row[0] = sample * g.hw + p_begin + rel_of(i);
            s.fraw[0][0] = raw[i];
            if (PHASE != 0) {
                // further full-shape operands (a residual added in front of or behind the normalisation) are not kept
                // in registers: each is read where the programs run (the fused variant is planned for one only)
#pragma unroll
                for (int f = 1; f < Spec::NF; ++f) {
                    if (f < Spec::n_full(a)) {
                        s.fraw[f][0] = u32x4{0u, 0u, 0u, 0u};
                        if (valid_of(i)) {
                            const uint64_t elem = ((uint64_t)sample * g.hw + p_begin + rel_of(i)) * g.channels + cvi * VEC;
                            s.fraw[f][0] = ragged ? load_elems<DT>(a.full[f], elem, cnt, 0u) : load_stream(a.full[f], elem * S::ESIZE);
                        }
                    }
                }
            }
            if (!vec_per_channel) {
#pragma unroll
                for (int v = 0; v < Spec::NV; ++v) {
                    if (v < Spec::n_vec(a)) {
                        s.vraw[v][0] = u32x4{0u, 0u, 0u, 0u};
                        if (valid_of(i))
                            s.vraw[v][0] = ragged ? load_vec_operand_elems<DT, Spec::kVecMode>(a.vec[v], s.row[0], s.col[0], g.channels, cnt)
                                                  : load_vec_operand<DT, Spec::kVecMode>(a.vec[v], s.row[0], s.col[0], g.channels);
                    }
                }
            }
            if (kLean) Storage<DT>::unpack(raw[i], s.acc);
            else run_program<DT, 1, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStore{});
        };

        if (PHASE != 2 && GEN && kLeanGen) {
            // ---- partial statistics straight from the packed values: plain sums per PAIR of elements (a pair never
            // straddles groups when a group holds an even number of channels), two dot-product instructions per pair
            float npos = 0.0f, sp[4], ssp[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) sp[j] = ssp[j] = 0.0f;
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                if (!valid_of(i)) continue;
                npos += 1.0f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t w = raw[i][j];
                    if (DT == DT_F16) {
                        const f16x2 x = __builtin_bit_cast(f16x2, w), ones = {(_Float16)1.0f, (_Float16)1.0f};
                        sp[j] = __builtin_amdgcn_fdot2(x, ones, sp[j], false);
                        ssp[j] = __builtin_amdgcn_fdot2(x, x, ssp[j], false);
                    } else {
                        const bf16x2 x = __builtin_bit_cast(bf16x2, w), ones = {(__bf16)1.0f, (__bf16)1.0f};
                        sp[j] = __builtin_amdgcn_fdot2_f32_bf16(x, ones, sp[j], false);
                        ssp[j] = __builtin_amdgcn_fdot2_f32_bf16(x, x, ssp[j], false);
                    }
                }
            }
            const float n_pair = active ? 2.0f * npos : 0.0f;
            const float inv = n_pair > 0.0f ? 1.0f / n_pair : 0.0f;
            // (a pair past the last channel of a ragged position was read as zeros and counts nothing; the channel count
            // is even here, so a pair is whole or absent)
            auto pair_stat = [&](int j) {
                const bool there = !ragged || (uint32_t)(2 * j) < cnt;
                return Stat{there ? n_pair : 0.0f, sp[j] * inv, fmaxf(ssp[j] - sp[j] * sp[j] * inv, 0.0f)};
            };
            Stat cur = pair_stat(0);
#pragma unroll
            for (int j = 1; j <= 4; ++j) {
                const bool flush = j == 4 || part_of(2 * (j % 4)) != part_of(2 * (j - 1));
                if (flush) {
                    float* q = lds_gen + (t * g.parts + part_of(2 * (j - 1))) * 3u;
                    q[0] = cur.n;
                    q[1] = cur.mean;
                    q[2] = cur.m2;
                }
                if (j < 4) cur = flush ? pair_stat(j % 4) : stat_merge(cur, pair_stat(j % 4));
            }
            for (uint32_t part = part_of(VEC - 1) + 1u; part < g.parts; ++part) {
                float* q = lds_gen + (t * g.parts + part) * 3u;
                q[0] = 0.0f;
                q[1] = 0.0f;
                q[2] = 0.0f;
            }
        }
        if (PHASE != 2 && GEN && !kLeanGen) {
            // ---- partial statistics: a running (mean, M2) per element slot over the lane's positions (one shared
            // count), then the slots of each part merged into one (count, mean, M2) triple per part in LDS
            float npos = 0.0f, mean_e[VEC], m2_e[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) mean_e[e] = m2_e[e] = 0.0f;
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                prologue(i);
                if (valid_of(i)) {
                    npos += 1.0f;
                    const float inv = __builtin_amdgcn_rcpf(npos);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const float d = s.acc[e] - mean_e[e];
                        mean_e[e] = __builtin_fmaf(d, inv, mean_e[e]);
                        m2_e[e] = __builtin_fmaf(d, s.acc[e] - mean_e[e], m2_e[e]);
                    }
                }
            }
            // slots of one part are adjacent: walk them once, flushing a part when the next one begins
            const float n_lane = active ? npos : 0.0f;
            auto n_of = [&](int e) { return (uint32_t)e < cnt ? n_lane : 0.0f; };
            Stat cur = {n_of(0), mean_e[0], m2_e[0]};
#pragma unroll
            for (int e = 1; e <= VEC; ++e) {
                const bool flush = e == VEC || part_of(e % VEC) != part_of(e - 1);
                if (flush) {
                    float* q = lds_gen + (t * g.parts + part_of(e - 1)) * 3u;
                    q[0] = cur.n;
                    q[1] = cur.mean;
                    q[2] = cur.m2;
                }
                if (e < VEC) {
                    const Stat slot = {n_of(e % VEC), mean_e[e % VEC], m2_e[e % VEC]};
                    cur = flush ? slot : stat_merge(cur, slot);
                }
            }
            // parts this lane's vector does not reach stay empty
            for (uint32_t part = part_of(VEC - 1) + 1u; part < g.parts; ++part) {
                float* q = lds_gen + (t * g.parts + part) * 3u;
                q[0] = 0.0f;
                q[1] = 0.0f;
                q[2] = 0.0f;
            }
        }
        if (PHASE != 2 && GEN) {
            __syncthreads();
            uint32_t grp;
            Stat acc;
            if (merge_parts_of_block<VEC>(g, lds_gen, &grp, &acc)) {
                if (PHASE == 0) {
                    const uint64_t per_parity = (uint64_t)g.samples * g.groups * g.blocks_per_sample;
                    const uint64_t slot = ((uint64_t)sample * g.groups + grp) * g.blocks_per_sample + bx;
                    const uint32_t par = g.epoch & 1u;
                    __hip_atomic_store(g.ws_gather + (par ^ 1u) * per_parity + slot, kSlotEmpty, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(g.ws_gather + par * per_parity + slot, pack_slot(acc.mean, acc.m2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    float* o = g.ws_partial + ((uint64_t)(sample * g.blocks_per_sample + bx) * g.groups + grp) * 4u;
                    o[0] = acc.n;
                    o[1] = acc.mean;
                    o[2] = acc.m2;
                }
            }
        }
        if (PHASE != 2 && !GEN) {
            // ---- partial statistics from registers
            LaneAcc la;
            LeanAcc lean;
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                if (kLean) {
                    if (valid_of(i)) lean_add_vector<DT>(lean, raw[i]);
                } else {
                    prologue(i);
                    if (valid_of(i)) la.template add_vector<VEC>(s.acc);
                }
            }
            const Stat st = group_lanes_merge(kLean ? lean.finish() : la.finish(), g.log2_vpg);
            if (PHASE == 0) {
                publish_tile(g, st, pstep, cvi, active, lds_part, sample, bx);
            } else {
                float* dst = g.ws_partial + ((uint64_t)(sample * g.blocks_per_sample + bx) * g.groups) * 4u;
                block_partial(g, st, pstep, cvi, active, lds_part, dst);
            }
        }
        if (PHASE == 1) {
            __syncthreads();  // LDS staging is reused by the next tile
            continue;
        }

        if (PHASE == 0) {
            // ---- device-scope exchange
            uint32_t grp;
            float mean, rstd;
            if (gather_sample(g, sample, a.eps, &grp, &mean, &rstd)) {
                lds_stat[grp * 2u] = mean;
                lds_stat[grp * 2u + 1u] = rstd;
            }
            __syncthreads();
        } else {
            // PHASE 2: the partials were written by the previous launch
            uint32_t grp;
            float mean, rstd;
            if (combine_sample(g, sample, a.eps, &grp, &mean, &rstd)) {
                lds_stat[grp * 2u] = mean;
                lds_stat[grp * 2u + 1u] = rstd;
            }
            __syncthreads();
        }

        if (PHASE == 0 && !kLean && !kLeanGen) {
            // The prologue is run again on the packed values below.  Without this fence the compiler keeps the
            // widened values of the statistics pass alive across the exchange instead (NV * VEC more registers).
#pragma unroll
            for (int i = 0; i < NV; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    uint32_t w = raw[i][j];
                    asm volatile("" : "+v"(w));
                    raw[i][j] = w;
                }
        }
        // ---- normalise straight from registers: y = x * A + B with A = rstd * gamma, B = beta - mean * A per
        // channel, so each element costs one fused multiply-add (taken directly from the fp16 value)
        const uint32_t my_grp = GEN ? first_grp : cvi >> g.log2_vpg;
        const float mean = lds_stat[my_grp * 2u], rstd = lds_stat[my_grp * 2u + 1u];
        // fp32 chains subtract the mean first ((x - mean) * A + beta): folded into one multiply-add, a group whose
        // spread is tiny against its mean loses eps_fp32 * |mean| * rstd, up to 3e-5 per unit of mean at rstd = 1 / sqrt(eps)
        constexpr bool kCentre = DT == DT_F32;
        float A[VEC], B[VEC], M[kCentre ? VEC : 1];
        auto affine = [&]() {
            float gm[VEC], bt[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                gm[e] = 1.0f;
                bt[e] = 0.0f;
            }
            if (Spec::gamma(a) >= 0) fetch_vec<DT, 1, Spec>(s, Spec::gamma(a), gm);
            if (Spec::beta(a) >= 0) fetch_vec<DT, 1, Spec>(s, Spec::beta(a), bt);
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                // GEN: the element's own group (its statistics sit part_of[e] entries further)
                const float r = GEN ? lds_stat[(my_grp + part_of(e)) * 2u + 1u] : rstd;
                const float m = GEN ? lds_stat[(my_grp + part_of(e)) * 2u] : mean;
                A[e] = r * gm[e];
                B[e] = kCentre ? bt[e] : bt[e] - m * A[e];
                if (kCentre) M[e % (kCentre ? VEC : 1)] = m;
            }
        };
        if (vec_per_channel) affine();
        char* out_base = static_cast<char*>(a.out[0]) + ((uint64_t)sample * g.hw + p_begin) * g.channels * S::ESIZE;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            prologue(i);
            if (!vec_per_channel) affine();
#pragma unroll
            for (int e = 0; e < VEC; ++e) s.acc[e] = __builtin_fmaf(kCentre ? s.acc[e] - M[e % (kCentre ? VEC : 1)] : s.acc[e], A[e], B[e]);
            run_program<DT, 1, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, NoStore{});
            if (valid_of(i)) {
                if (ragged) store_elems<DT>(out_base + (size_t)step_of(i) * step_bytes, lane_bytes / (uint32_t)S::ESIZE, cnt, S::pack(s.acc));
                else store_stream(out_base + (size_t)step_of(i) * step_bytes, lane_bytes, S::pack(s.acc));
            }
        }
        __syncthreads();  // LDS staging is reused by the next tile
    }
}

}  // namespace pf
