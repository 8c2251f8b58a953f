// Row family and element-wise family kernel templates.
//
// Row family: prologue -> reduction over the innermost dimension -> broadcast -> epilogue, one kernel.
// The row's elements stay in registers from the load to the store, so the chain moves exactly its
// compulsory bytes.  The reduction is exchanged at the narrowest scope that covers a row (paper section
// 5.1, synchronisation insertion): inside one 64-lane wave by DPP permutations when a wave owns the row;
// through LDS and one workgroup barrier when several waves share it.
//
// Element-wise family: the same interpreter on a flat stream of 16-byte vectors; lane scope only.
#pragma once
#include "pf_device.hpp"

namespace pf {

// Secondary-output stores (U_STORE) for layouts where a value's position equals the input's.
struct RowStore {
    void* out0;
    void* out1;
    uint64_t row_byte;
    uint32_t limit;
    template <int DT, int K, class Spec>
    PF_DEVICE void operator()(int slot, const LaneState<DT, K, Spec>& st) const {
        using S = Storage<DT>;
        void* dst = slot == 0 ? out0 : out1;
#pragma unroll
        for (int k = 0; k < K; ++k)
            if (st.col[k] < limit)
                store_stream(dst, row_byte + (uint64_t)st.col[k] * S::ESIZE, S::pack(st.acc + k * S::VEC));
    }
};
struct FlatStore {
    void* out0;
    void* out1;
    uint32_t total_vecs, vecs_per_row;
    template <int DT, int K, class Spec>
    PF_DEVICE void operator()(int slot, const LaneState<DT, K, Spec>& st) const {
        using S = Storage<DT>;
        void* dst = slot == 0 ? out0 : out1;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const uint32_t gv = st.row[k] * vecs_per_row + st.col[k] / S::VEC;
            if (gv < total_vecs) store_stream(dst, (uint64_t)gv * 16u, S::pack(st.acc + k * S::VEC));
        }
    }
};

// Combine per-wave partials of the waves that share a row through LDS (block scope).  `red` must be a
// staging area no earlier reduction of this workgroup may still be reading.
template <class Op>
PF_DEVICE float row_allreduce(float v, uint32_t waves_per_row, uint32_t wave, uint32_t lane, float* red) {
    v = wave_allreduce<Op>(v);
    if (waves_per_row == 1) return v;
    if (lane == 0) red[wave] = v;
    __syncthreads();
    const uint32_t first = (wave / waves_per_row) * waves_per_row;
    float r = red[first];
    for (uint32_t i = 1; i < waves_per_row; ++i) r = Op::apply(r, red[first + i]);
    return r;
}

// Issue the loads of every operand of a row tile before anything is used.  `row_byte` is wave-uniform,
// so each load is a scalar base plus a 32-bit lane offset.  Vectors that are not loaded read as `fill`.
// The KC vectors starting at k0 belong to the row at `row_byte`.
template <int DT, int K, int KC, class Spec>
PF_DEVICE void load_row_operands(const ChainArgs& a, LaneState<DT, K, Spec>& s, int k0, uint64_t row_byte, uint32_t row,
                                 uint32_t load_limit, uint32_t limit, uint32_t fill) {
    using S = Storage<DT>;
#pragma unroll
    for (int f = 0; f < Spec::NF; ++f) {
        if (f < Spec::n_full(a)) {
            const char* base = static_cast<const char*>(a.full[f]) + row_byte;
#pragma unroll
            for (int c = 0; c < KC; ++c) {
                const int k = k0 + c;
                s.fraw[f][k] = u32x4{fill, fill, fill, fill};
                if (s.col[k] < load_limit) s.fraw[f][k] = load_stream(base, s.col[k] * (uint32_t)S::ESIZE);
            }
        }
    }
#pragma unroll
    for (int v = 0; v < Spec::NV; ++v) {
        if (v < Spec::n_vec(a)) {
#pragma unroll
            for (int c = 0; c < KC; ++c) {
                const int k = k0 + c;
                s.vraw[v][k] = u32x4{0u, 0u, 0u, 0u};
                if (s.col[k] < limit) s.vraw[v][k] = load_vec_operand<DT>(a.vec[v], row, s.col[k], a.n_inner);
            }
        }
    }
}

// Row kernel.  Each lane holds KC 16-byte vectors of each of RPW rows (K = KC * RPW vectors in all).
//   WPR1 = true : a wave owns RPW whole rows; reductions never leave the wave (no LDS, no barrier).  Several
//                 rows per wave put more loads in flight per wave, which is what short rows need to cover
//                 the HBM latency.
//   WPR1 = false: waves_per_row waves of a workgroup share one row (RPW must be 1).
template <int DT, int KC, int RPW, class Spec, int MAXT, bool WPR1>
__global__ void __launch_bounds__(MAXT) row_kernel(const ChainArgs a, const RowGeom g) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    constexpr int K = KC * RPW;
    constexpr int EC = KC * VEC;  // elements per lane per row
    constexpr bool PR = S::PRECISE;
    static_assert(WPR1 || RPW == 1, "several rows per wave only when a wave owns its rows");
    __shared__ float red[2][16];

    const uint32_t lane = threadIdx.x & 63u;
    // the wave index is the same for all 64 lanes: keep it, and everything derived from it, in scalar registers
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t wpr = WPR1 ? 1u : g.waves_per_row;
    const uint32_t slot_in_block = WPR1 ? wave : wave / wpr;
    const uint64_t row0 = ((uint64_t)blockIdx.x * g.rows_per_block + slot_in_block) * RPW;
    if (WPR1 && row0 >= a.rows) return;  // wave-uniform; this configuration has no barrier
    const uint32_t n = a.n_inner;
    const uint32_t lane_in_row = WPR1 ? lane : (wave - slot_in_block * wpr) * 64u + lane;

    LaneState<DT, K, Spec> s;
    uint32_t limit[RPW], i_row[RPW];
    uint64_t row_byte[RPW];
    const bool fill_inf = a.core_mask == 2u;
    const uint32_t fill = fill_inf ? (DT == DT_F32 ? 0xff800000u : (DT == DT_F16 ? 0xfc00fc00u : 0xff80ff80u)) : 0u;
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const uint64_t row64 = row0 + r;
        const uint32_t row = (uint32_t)row64;
        limit[r] = row64 < a.rows ? n : 0u;
        uint32_t load_limit = limit[r];
        i_row[r] = 0;
        if (a.mask_si != 0u) {
            // columns beyond the diagonal are overwritten by the mask before they are used: skip their loads
            i_row[r] = row - fast_div(row, a.mask_div) * a.mask_si;
            const uint32_t keep_vec = (i_row[r] + VEC) / VEC * VEC;
            load_limit = load_limit < keep_vec ? load_limit : keep_vec;
        }
#pragma unroll
        for (int c = 0; c < KC; ++c) {
            s.row[r * KC + c] = row;
            s.col[r * KC + c] = (lane_in_row + 64u * wpr * c) * VEC;
        }
        row_byte[r] = row64 * n * S::ESIZE;
        load_row_operands<DT, K, KC, Spec>(a, s, r * KC, row_byte[r], row, load_limit, limit[r], fill);
    }

    // secondary outputs (U_STORE) are supported for one row per wave only; the planner enforces it
    const RowStore store_fn{a.out[0], a.out[1], row_byte[0], limit[0]};
    run_program<DT, K, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, store_fn);

    // Lanes past the end of a row that does not fill the lanes exactly must not disturb the reductions.
    const bool exact = n == 64u * wpr * (uint32_t)EC;
    const float inv_n = 1.0f / (float)n;
    const int core = Spec::core(a);
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        float* acc = s.acc + r * EC;
        bool valid[KC];
#pragma unroll
        for (int c = 0; c < KC; ++c) valid[c] = s.col[r * KC + c] < limit[r];
        const bool all_valid = exact && limit[r] != 0u;
        if (core == CORE_SOFTMAX) {
            if (a.core_mask == 2u) {
                // causal mask folded into the core, nothing but the load in front of it.  Vectors wholly right
                // of the diagonal were never loaded and already hold -inf; only the vector that contains the
                // diagonal needs element-wise masking.  Which of its elements are masked is the same for the
                // whole wave (scalar compares); which lane holds it is one vector compare.
                const uint32_t diag_col = i_row[r] / VEC * VEC;
                const uint32_t last = i_row[r] - diag_col;  // last unmasked element inside the diagonal vector
#pragma unroll
                for (int c = 0; c < KC; ++c) {
                    const bool is_diag = s.col[r * KC + c] == diag_col;
#pragma unroll
                    for (int e = 1; e < VEC; ++e)
                        acc[c * VEC + e] = (is_diag && (uint32_t)e > last) ? -__builtin_inff() : acc[c * VEC + e];
                }
            } else if (a.core_mask == 1u) {
                // causal mask folded into the core after other prologue steps: mask every element by position
#pragma unroll
                for (int c = 0; c < KC; ++c) {
                    const int32_t last = (int32_t)i_row[r] - (int32_t)s.col[r * KC + c];
#pragma unroll
                    for (int e = 0; e < VEC; ++e) acc[c * VEC + e] = (e > last) ? -__builtin_inff() : acc[c * VEC + e];
                }
            }
            if (!all_valid) {
#pragma unroll
                for (int c = 0; c < KC; ++c)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) acc[c * VEC + e] = valid[c] ? acc[c * VEC + e] : -__builtin_inff();
            }
            float m = acc[0];
#pragma unroll
            for (int e = 1; e < EC; ++e) m = fmaxf(m, acc[e]);
            m = row_allreduce<OpMax>(m, wpr, wave, lane, red[0]);
            // exp(c * (x - m)); c is the folded scale (1 when there is none).  -inf - m = -inf -> 0; an all
            // -inf row gives -inf - -inf = NaN, as the definition does.
            const float cs = a.core_scale;
            float sum = 0.0f;
            if (PR) {
#pragma unroll
                for (int e = 0; e < EC; ++e) {
                    acc[e] = expf((acc[e] - m) * cs);
                    sum += acc[e];
                }
            } else {
                const float c2 = cs * kLog2e;
                const float mc = -m * c2;
#pragma unroll
                for (int e = 0; e < EC; ++e) {
                    acc[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[e], c2, mc));
                    sum += acc[e];
                }
            }
            sum = row_allreduce<OpSum>(sum, wpr, wave, lane, red[1]);
            const float inv = pf_rcp<PR>(sum);
#pragma unroll
            for (int e = 0; e < EC; ++e) acc[e] *= inv;
        } else if (core == CORE_LAYERNORM) {
            if (!all_valid) {
#pragma unroll
                for (int c = 0; c < KC; ++c)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) acc[c * VEC + e] = valid[c] ? acc[c * VEC + e] : 0.0f;
            }
            float s1 = 0.0f;
#pragma unroll
            for (int e = 0; e < EC; ++e) s1 += acc[e];
            const float mean = row_allreduce<OpSum>(s1, wpr, wave, lane, red[0]) * inv_n;
            float s2 = 0.0f;
#pragma unroll
            for (int c = 0; c < KC; ++c)
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float d = acc[c * VEC + e] - mean;
                    acc[c * VEC + e] = d;
                    s2 += (all_valid || valid[c]) ? d * d : 0.0f;
                }
            const float var = row_allreduce<OpSum>(s2, wpr, wave, lane, red[1]) * inv_n;
            const float rstd = pf_rsqrt<PR>(var + a.eps);
            float gm[EC], bt[EC];
#pragma unroll
            for (int e = 0; e < EC; ++e) {
                gm[e] = 1.0f;
                bt[e] = 0.0f;
            }
            if (Spec::gamma(a) >= 0) fetch_vec_part<DT, K, KC, Spec>(s, Spec::gamma(a), r * KC, gm);
            if (Spec::beta(a) >= 0) fetch_vec_part<DT, K, KC, Spec>(s, Spec::beta(a), r * KC, bt);
#pragma unroll
            for (int e = 0; e < EC; ++e) acc[e] = acc[e] * rstd * gm[e] + bt[e];
        } else if (core == CORE_RMSNORM) {
            float s2 = 0.0f;
#pragma unroll
            for (int c = 0; c < KC; ++c)
#pragma unroll
                for (int e = 0; e < VEC; ++e) s2 += (all_valid || valid[c]) ? acc[c * VEC + e] * acc[c * VEC + e] : 0.0f;
            const float ms = row_allreduce<OpSum>(s2, wpr, wave, lane, red[0]) * inv_n;
            const float rstd = pf_rsqrt<PR>(ms + a.eps);
            float gm[EC];
#pragma unroll
            for (int e = 0; e < EC; ++e) gm[e] = 1.0f;
            if (Spec::gamma(a) >= 0) fetch_vec_part<DT, K, KC, Spec>(s, Spec::gamma(a), r * KC, gm);
#pragma unroll
            for (int e = 0; e < EC; ++e) acc[e] = acc[e] * rstd * gm[e];
        }
    }

    run_program<DT, K, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, store_fn);

#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        char* out_row = static_cast<char*>(a.out[0]) + row_byte[r];
#pragma unroll
        for (int c = 0; c < KC; ++c) {
            const int k = r * KC + c;
            if (s.col[k] < limit[r]) store_stream(out_row, s.col[k] * (uint32_t)S::ESIZE, S::pack(s.acc + k * VEC));
        }
    }
}

// Reduction cores whose result is one value per row (REDUCE_SUM / MAX / MEAN, keepdim): the epilogue runs
// on that single value and one lane stores it.
template <int DT, int K>
__global__ void __launch_bounds__(1024) row_reduce_kernel(const ChainArgs a, const RowGeom g) {
    using S = Storage<DT>;
    using Spec = GenericSpec;
    constexpr int VEC = S::VEC;
    __shared__ float red[2][16];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t wpr = g.waves_per_row;
    const uint64_t row64 = (uint64_t)blockIdx.x * g.rows_per_block + wave / wpr;
    const bool row_ok = row64 < a.rows;
    if (wpr == 1 && !row_ok) return;
    const uint32_t row = (uint32_t)row64;
    const uint32_t n = a.n_inner;
    LaneState<DT, K, Spec> s;
    const uint32_t lane_in_row = (wave % wpr) * 64u + lane;
    const uint32_t limit = row_ok ? n : 0u;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        s.row[k] = row;
        s.col[k] = (lane_in_row + 64u * wpr * k) * VEC;
    }
    const uint64_t row_byte = row64 * n * S::ESIZE;
    load_row_operands<DT, K, K, Spec>(a, s, 0, row_byte, row, limit, limit, 0u);
    run_program<DT, K, Spec>(ProgView<DynList>{a.pro}, s, NoStore{});
    float r;
    if (a.core == CORE_REDUCE_MAX) {
        float m = -__builtin_inff();
        float nan_seen = 0.0f;
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float x = s.acc[k * VEC + e];
                if (s.col[k] < limit) {
                    m = fmaxf(m, x);
                    nan_seen = (x != x) ? 1.0f : nan_seen;
                }
            }
        m = row_allreduce<OpMax>(m, wpr, wave, lane, red[0]);
        nan_seen = row_allreduce<OpMax>(nan_seen, wpr, wave, lane, red[1]);
        r = nan_seen > 0.0f ? __builtin_nanf("") : m;
    } else {
        float sum = 0.0f;
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
            for (int e = 0; e < VEC; ++e) sum += (s.col[k] < limit) ? s.acc[k * VEC + e] : 0.0f;
        r = row_allreduce<OpSum>(sum, wpr, wave, lane, red[0]);
        if (a.core == CORE_REDUCE_MEAN) r = r / (float)n;
    }
    // epilogue on the row value: immediates and unary steps only (the planner guarantees it)
    LaneState<DT, 1, Spec> t;
    t.row[0] = row;
    t.col[0] = 0;
#pragma unroll
    for (int e = 0; e < VEC; ++e) t.acc[e] = r;
    run_program<DT, 1, Spec>(ProgView<DynList>{a.epi}, t, NoStore{});
    if (row_ok && lane_in_row == 0) {
        if (DT == DT_F32) {
            static_cast<float*>(a.out[0])[row64] = t.acc[0];
        } else {
            const u32x4 packed = S::pack(t.acc);
            static_cast<uint16_t*>(a.out[0])[row64] = (uint16_t)(packed[0] & 0xffffu);
        }
    }
}

// Element-wise family: a flat stream of vectors, K per lane, lanes of a workgroup adjacent for each k.
template <int DT, int K, class Spec>
__global__ void __launch_bounds__(256) ew_kernel(const ChainArgs a, const uint32_t total_vecs, const uint32_t vecs_per_row) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    LaneState<DT, K, Spec> s;
    const uint32_t base = blockIdx.x * (256u * K) + threadIdx.x;
    uint32_t gv[K];
    bool valid[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        gv[k] = base + 256u * k;
        valid[k] = gv[k] < total_vecs;
        s.row[k] = gv[k] / vecs_per_row;
        s.col[k] = (gv[k] - s.row[k] * vecs_per_row) * VEC;
    }
#pragma unroll
    for (int f = 0; f < Spec::NF; ++f) {
        if (f < Spec::n_full(a)) {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                s.fraw[f][k] = u32x4{0u, 0u, 0u, 0u};
                if (valid[k]) s.fraw[f][k] = load_stream(a.full[f], (uint64_t)gv[k] * 16u);
            }
        }
    }
#pragma unroll
    for (int v = 0; v < Spec::NV; ++v) {
        if (v < Spec::n_vec(a)) {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                s.vraw[v][k] = u32x4{0u, 0u, 0u, 0u};
                if (valid[k]) s.vraw[v][k] = load_vec_operand<DT>(a.vec[v], s.row[k], s.col[k], a.n_inner);
            }
        }
    }
    const FlatStore store_fn{a.out[0], a.out[1], total_vecs, vecs_per_row};
    run_program<DT, K, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, store_fn);
#pragma unroll
    for (int k = 0; k < K; ++k)
        if (valid[k]) store_stream(a.out[0], (uint64_t)gv[k] * 16u, S::pack(s.acc + k * VEC));
}

// Static program lists: each step packed as code | kind << 8 | slot << 16.
template <uint32_t... Us>
struct StaticList {
    static constexpr bool kDynamic = false;
    static constexpr int n = sizeof...(Us);
    static constexpr UopC at(int i) {
        constexpr uint32_t arr[sizeof...(Us) + 1] = {Us..., 0u};
        return UopC{(uint8_t)(arr[i] & 0xffu), (uint8_t)((arr[i] >> 8) & 0xffu), (uint8_t)((arr[i] >> 16) & 0xffu)};
    }
};

}  // namespace pf
