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
template <bool RAGGED = false>
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
        for (int k = 0; k < K; ++k) {
            if (RAGGED)
                store_elems<DT>(dst, row_byte / S::ESIZE + st.col[k], elems_below<S::VEC>(st.col[k], limit), S::pack(st.acc + k * S::VEC));
            else if (st.col[k] < limit)
                store_stream(dst, row_byte + (uint64_t)st.col[k] * S::ESIZE, S::pack(st.acc + k * S::VEC));
        }
    }
};
template <bool RAGGED = false>
struct FlatStore {
    void* out0;
    void* out1;
    uint32_t total_vecs, vecs_per_row;
    uint64_t total_elems;
    template <int DT, int K, class Spec>
    PF_DEVICE void operator()(int slot, const LaneState<DT, K, Spec>& st, const uint32_t (&gv)[K]) const {
        using S = Storage<DT>;
        void* dst = slot == 0 ? out0 : out1;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (RAGGED) {
                const uint64_t first = (uint64_t)gv[k] * S::VEC;
                const uint32_t cnt = first < total_elems ? (uint32_t)(total_elems - first < S::VEC ? total_elems - first : S::VEC) : 0u;
                store_elems<DT>(dst, first, cnt, S::pack(st.acc + k * S::VEC));
            } else if (gv[k] < total_vecs) {
                store_stream(dst, (uint64_t)gv[k] * 16u, S::pack(st.acc + k * S::VEC));
            }
        }
    }
};

// Combine per-wave partials of the waves that share a row through LDS (block scope).  `red` must be a
// staging area no earlier reduction of this workgroup may still be reading.
// LOG2L < 6: a row occupies an aligned segment of 2^LOG2L lanes of one wave (waves_per_row is then 1).
template <class Op, int LOG2L = 6>
PF_DEVICE float row_allreduce(float v, uint32_t waves_per_row, uint32_t wave, uint32_t first_wave, uint32_t lane, float* red) {
    v = seg_allreduce<Op, LOG2L>(v);
    if (waves_per_row == 1) return v;
    if (lane == 0) red[wave] = v;
    __syncthreads();
    // at most 16 waves share a row (first_wave is the first of them): lane j of every 16 lanes reads the partial of the
    // row's wave j, and four lane permutations leave the row's value in every lane -- one LDS read, no loop
    const uint32_t j = lane & 15u;
    const float p = j < waves_per_row ? red[first_wave + j] : Op::identity();
    return subrow_allreduce<Op, 4>(p);
}

// What the interpreter calls back into from inside the row kernel: secondary-output stores, and the row
// reductions of a row program.  A reduction leaves the accumulator as it is and puts each row's value, the
// same in every lane, into rowv[slot][k] for the vectors k of that row (a wave may hold RPW rows of KC
// vectors).  Successive reductions alternate between the two LDS staging areas; one barrier per reduction
// separates their reuse (several waves per row imply RPW = 1).
template <bool RAGGED, int KC, int RPW, int LOG2L = 6>
struct RowHooks {
    RowStore<RAGGED> store;
    uint32_t wpr, wave, first_wave, lane;
    const uint32_t* limit;  // [RPW] row lengths (0 for rows past the end)
    float inv_n;
    float (*red)[16];
    uint32_t* flip;
    template <int DT, int K, class Spec>
    PF_DEVICE void operator()(int slot, const LaneState<DT, K, Spec>& st) const {
        store(slot, st);
    }
};

template <bool RAGGED, int KC, int RPW, int LOG2L, int DT, int K, class Spec>
PF_DEVICE void hook_reduce(const RowHooks<RAGGED, KC, RPW, LOG2L>& h, int code, int slot, LaneState<DT, K, Spec>& s) {
    constexpr int VEC = Storage<DT>::VEC;
    static_assert(K == KC * RPW, "row hooks and lane state disagree");
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const uint32_t limit = h.limit[r];
        float* stage = h.red[*h.flip & 1u];
        *h.flip += 1u;
        float v;
        if (code == U_RED_MAX) {
            float m = -__builtin_inff(), nan_seen = 0.0f;
#pragma unroll
            for (int c = 0; c < KC; ++c)
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const int k = r * KC + c;
                    const bool valid = RAGGED ? s.col[k] + (uint32_t)e < limit : s.col[k] < limit;
                    const float x = s.acc[k * VEC + e];
                    m = valid ? fmaxf(m, x) : m;
                    nan_seen = (valid && x != x) ? 1.0f : nan_seen;
                }
            // a NaN anywhere in the row makes the row's maximum NaN
            if (h.wpr == 1u && LOG2L == 6) {
                // the wave reduction runs on order-preserving integer keys in which a positive NaN ranks above +inf
                v = wave_allreduce<OpMax>(nan_seen > 0.0f ? __builtin_nanf("") : m);
            } else {
                m = row_allreduce<OpMax, LOG2L>(m, h.wpr, h.wave, h.first_wave, h.lane, stage);
                nan_seen = row_allreduce<OpMax, LOG2L>(nan_seen, h.wpr, h.wave, h.first_wave, h.lane, h.red[*h.flip & 1u]);
                *h.flip += 1u;
                v = nan_seen > 0.0f ? __builtin_nanf("") : m;
            }
        } else {
            float sum = 0.0f;
#pragma unroll
            for (int c = 0; c < KC; ++c)
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const int k = r * KC + c;
                    const bool valid = RAGGED ? s.col[k] + (uint32_t)e < limit : s.col[k] < limit;
                    sum += valid ? s.acc[k * VEC + e] : 0.0f;
                }
            v = row_allreduce<OpSum, LOG2L>(sum, h.wpr, h.wave, h.first_wave, h.lane, stage);
            if (code == U_RED_MEAN) v *= h.inv_n;
        }
#pragma unroll
        for (int t = 0; t < PF_DEV_MAX_ROWV; ++t)
            if (slot == t) {
#pragma unroll
                for (int c = 0; c < KC; ++c) s.rowv[t][r * KC + c] = v;
            }
    }
}

// The shape of a launch as a compile-time fact.  A row kernel's waves are short (one to four rows each), so what a
// wave executes before its first load and the branches it takes on the way are a visible share of its life: whether
// its rows fill the lanes, whether there is a causal mask and of what period, how the mask is applied, how many waves
// share a row.  For large tensors the planner hands the run-time compiler a type that holds these as constants
// (kConst = true and the members read below); RuntimeRowShape stands for "read the kernel arguments".
struct RuntimeRowShape {
    static constexpr bool kConst = false;
};
template <class RS>
struct RowShape {
    static PF_DEVICE uint32_t n_inner(const ChainArgs& a) {
        if constexpr (RS::kConst) return RS::n_inner;
        else return a.n_inner;
    }
    static PF_DEVICE uint64_t rows(const ChainArgs& a) {
        if constexpr (RS::kConst) return RS::rows;
        else return a.rows;
    }
    static PF_DEVICE uint32_t mask_si(const ChainArgs& a) {
        if constexpr (RS::kConst) return RS::mask_si;
        else return a.mask_si;
    }
    static PF_DEVICE uint32_t core_mask(const ChainArgs& a) {
        if constexpr (RS::kConst) return RS::core_mask;
        else return a.core_mask;
    }
    static PF_DEVICE uint32_t vec_plain_all(const ChainArgs& a) {
        if constexpr (RS::kConst) return RS::vec_plain_all;
        else return a.vec_plain_all;
    }
    static PF_DEVICE uint32_t waves_per_row(const RowGeom& g) {
        if constexpr (RS::kConst) return RS::waves_per_row;
        else return g.waves_per_row;
    }
    static PF_DEVICE uint32_t rows_per_block(const RowGeom& g) {
        if constexpr (RS::kConst) return RS::rows_per_block;
        else return g.rows_per_block;
    }
    // row mod mask_si
    static PF_DEVICE uint32_t row_in_mask(const ChainArgs& a, uint32_t row) {
        if constexpr (RS::kConst) return row % (RS::mask_si ? RS::mask_si : 1u);
        else return row - fast_div(row, a.mask_div) * a.mask_si;
    }
};

// Issue the loads of every operand of a row tile before anything is used.  `row_byte` is wave-uniform,
// so each load is a scalar base plus a 32-bit lane offset.  Vectors that are not loaded read as `fill`.
// The KC vectors starting at k0 belong to the row at `row_byte`.
// RAGGED: the row's byte length is not a multiple of 16; its vectors are gathered element by element.
// WHOLE: every vector of the tile lies inside its row, nothing is skipped and every broadcast operand is a vector of the
// row's length, so the loads carry no condition and no index arithmetic: they are issued back to back, and no register has to be merged with a fill value (a merge the compiler resolves by
// waiting for the load).
template <int DT, int K, int KC, class Spec, bool RAGGED = false, bool WHOLE = false>
PF_DEVICE void load_row_operands(const ChainArgs& a, LaneState<DT, K, Spec>& s, int k0, uint64_t row_byte, uint32_t row,
                                 uint32_t load_limit, uint32_t limit, uint32_t fill, uint32_t n_inner) {
    using S = Storage<DT>;
    static_assert(!(RAGGED && WHOLE), "a ragged row has a partial vector");
#pragma unroll
    for (int f = 0; f < Spec::NF; ++f) {
        if (f < Spec::n_full(a)) {
            const char* base = static_cast<const char*>(a.full[f]) + row_byte;
#pragma unroll
            for (int c = 0; c < KC; ++c) {
                const int k = k0 + c;
                if (WHOLE) {
                    s.fraw[f][k] = load_stream(base, s.col[k] * (uint32_t)S::ESIZE);
                    continue;
                }
                if (RAGGED) {
                    s.fraw[f][k] = u32x4{fill, fill, fill, fill};
                    // (what follows a partial vector is the next row of the same tensor, unless this is the last row)
                    s.fraw[f][k] = load_elems<DT>(base, s.col[k], elems_below<S::VEC>(s.col[k], load_limit), fill,
                                                  (uint64_t)row + 1u < a.rows || s.col[k] + (uint32_t)S::VEC <= n_inner);
                } else {
                    // No branch around the load: a lane past the limit reads the last vector inside it (the same
                    // memory line as its neighbour: no extra traffic; `row_byte` always addresses a row that
                    // exists) and the fill value is selected afterwards.  A guarded load would merge with the fill
                    // value at the join, which the compiler resolves by waiting for the load: every later load of
                    // the wave would then be issued one memory round trip late.
                    const uint32_t lim = load_limit != 0u ? load_limit : n_inner;
                    const uint32_t colc = min(s.col[k], lim - (uint32_t)S::VEC);
                    const u32x4 got = load_stream(base, colc * (uint32_t)S::ESIZE);
                    const bool keep = s.col[k] < load_limit;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t w = got[j];
                        s.fraw[f][k][j] = keep ? w : fill;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int v = 0; v < Spec::NV; ++v) {
        if (v < Spec::n_vec(a)) {
#pragma unroll
            for (int c = 0; c < KC; ++c) {
                const int k = k0 + c;
                if (WHOLE) {
                    // a vector of the row's length: the same for every row the wave holds, loaded for the first only
                    if (k0 > 0) s.vraw[v][k] = s.vraw[v][c];
                    else s.vraw[v][k] = load_cached(a.vec[v].ptr, (uint64_t)s.col[k] * S::ESIZE);
                    continue;
                }
                if (RAGGED) {
                    s.vraw[v][k] = u32x4{0u, 0u, 0u, 0u};
                    s.vraw[v][k] = load_vec_operand_elems<DT, Spec::kVecMode>(a.vec[v], row, s.col[k], n_inner, elems_below<S::VEC>(s.col[k], limit));
                } else {
                    // (as above; values of lanes past the row's end are never used)
                    const uint32_t colc = min(s.col[k], n_inner - (uint32_t)S::VEC);
                    s.vraw[v][k] = load_vec_operand<DT, Spec::kVecMode>(a.vec[v], row, colc, n_inner);
                }
            }
        }
    }
}

// Row kernel.  Each lane holds KC 16-byte vectors of each of RPW rows (K = KC * RPW vectors in all).
//   WPR1 = true : a wave owns RPW whole rows; reductions never leave the wave (no LDS, no barrier).  Several
//                 rows per wave put more loads in flight per wave, which is what short rows need to cover
//                 the HBM latency.
//   WPR1 = false: waves_per_row waves of a workgroup share one row (RPW must be 1).
//   RAGGED      : the row length is not a multiple of a 16-byte vector (element-aligned vector access, a
//                 partial last vector, element-granular validity).
//   LOG2L       : (WPR1 only) a row occupies an aligned segment of 2^LOG2L lanes, so a wave holds 64 >> LOG2L
//                 rows side by side (times RPW in registers): short rows no longer leave most lanes idle.
//                 Row addressing is then per lane instead of per wave.
template <int DT, int KC, int RPW, class Spec, int MAXT, bool WPR1, bool RAGGED = false, int LOG2L = 6, class RS = RuntimeRowShape>
__global__ void __launch_bounds__(MAXT) row_kernel(const ChainArgs a, const RowGeom g) {
    using Sh = RowShape<RS>;
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    constexpr int K = KC * RPW;
    constexpr int EC = KC * VEC;  // elements per lane per row
    constexpr bool PR = S::PRECISE;
    static_assert(WPR1 || RPW == 1, "several rows per wave only when a wave owns its rows");
    static_assert(WPR1 || LOG2L == 6, "rows side by side in a wave only when a wave owns its rows");
    constexpr uint32_t LPR = 1u << LOG2L;   // lanes per row inside a wave
    constexpr uint32_t SUB = 64u >> LOG2L;  // rows side by side in a wave
    __shared__ float red[2][16];
    // (a launch of many workgroups finds the arguments in the scalar cache after the first one per compute unit)
    if constexpr (!RS::kConst) warm_chain_arguments<Spec>();
    else if constexpr (RS::rows * RS::n_inner <= (4u << 20)) warm_chain_arguments<Spec>();

    const uint32_t lane = threadIdx.x & 63u;
    // the wave index is the same for all 64 lanes: keep it, and everything derived from it, in scalar registers
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t wpr = WPR1 ? 1u : Sh::waves_per_row(g);
    const uint32_t rows_per_block = Sh::rows_per_block(g);
    const uint64_t n_rows = Sh::rows(a);
    const uint32_t mask_si = Sh::mask_si(a), core_mask = Sh::core_mask(a);
    const uint32_t slot_in_block = WPR1 ? wave : (rows_per_block == 1u ? 0u : wave / wpr);
    const uint32_t first_wave = WPR1 ? wave : slot_in_block * wpr;  // first of the waves that share this wave's row
    const uint64_t row0 = ((uint64_t)blockIdx.x * rows_per_block + slot_in_block) * (RPW * SUB);
    // wave-uniform; this configuration has no barrier (and a row count known to be a whole number of workgroups needs no test)
    const bool all_waves_have_rows = RS::kConst && n_rows % ((uint64_t)rows_per_block * (RPW * SUB)) == 0u;
    if (WPR1 && !all_waves_have_rows && row0 >= n_rows) return;
    const uint32_t n = Sh::n_inner(a);
    const uint32_t sub = LOG2L == 6 ? 0u : lane >> LOG2L;  // which of the wave's side-by-side rows this lane serves
    const uint32_t lane_in_row = WPR1 ? (lane & (LPR - 1u)) : (wave - slot_in_block * wpr) * 64u + lane;

    LaneState<DT, K, Spec> s;
    uint32_t limit[RPW], i_row[RPW];
    uint64_t row_byte[RPW];
    const bool fill_inf = core_mask == 2u;
    const uint32_t fill = fill_inf ? (DT == DT_F32 ? 0xff800000u : (DT == DT_F16 ? 0xfc00fc00u : 0xff80ff80u)) : 0u;
    // the usual tile: rows that fill the lanes exactly, all of them inside the tensor, no causal skipping
    // (with the shape known when the kernel is compiled, a row count that is a whole number of workgroups needs no test)
    const bool rows_whole = all_waves_have_rows || row0 + (uint64_t)(RPW * SUB) <= n_rows;
    const bool whole_tile = !RAGGED && n == LPR * wpr * (uint32_t)EC && mask_si == 0u && Sh::vec_plain_all(a) != 0u && rows_whole;
    if (!RAGGED && whole_tile) {
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            const uint64_t row64 = row0 + (uint32_t)r * SUB + sub;
            limit[r] = n;
            i_row[r] = 0;
#pragma unroll
            for (int c = 0; c < KC; ++c) {
                s.row[r * KC + c] = (uint32_t)row64;
                s.col[r * KC + c] = (lane_in_row + LPR * wpr * c) * VEC;
            }
            row_byte[r] = row64 * n * S::ESIZE;
            load_row_operands<DT, K, KC, Spec, false, !RAGGED>(a, s, r * KC, row_byte[r], (uint32_t)row64, n, n, fill, n);
        }
    } else
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const uint64_t row64 = row0 + (uint32_t)r * SUB + sub;
        const uint32_t row = (uint32_t)row64;
        limit[r] = (all_waves_have_rows || row64 < n_rows) ? n : 0u;
        uint32_t load_limit = limit[r];
        i_row[r] = 0;
        if (mask_si != 0u) {
            // columns beyond the diagonal are overwritten by the mask before they are used: skip their loads
            i_row[r] = Sh::row_in_mask(a, row);
            const uint32_t keep_vec = (i_row[r] + VEC) / VEC * VEC;
            load_limit = load_limit < keep_vec ? load_limit : keep_vec;
        }
#pragma unroll
        for (int c = 0; c < KC; ++c) {
            s.row[r * KC + c] = row;
            s.col[r * KC + c] = (lane_in_row + LPR * wpr * c) * VEC;
        }
        row_byte[r] = row64 * n * S::ESIZE;
        // (loads of a row past the end of the tensor are aimed at the last row and discarded)
        const uint64_t row_in = (RAGGED || all_waves_have_rows) ? row64 : min(row64, n_rows - 1u);
        load_row_operands<DT, K, KC, Spec, RAGGED>(a, s, r * KC, row_in * n * S::ESIZE, (uint32_t)row_in, load_limit, limit[r], fill, n);
    }

    // secondary outputs (U_STORE) are supported for one row per wave only; the planner enforces it
    const float inv_n = 1.0f / (float)n;
    uint32_t flip = 0;
    const RowHooks<RAGGED, KC, RPW, LOG2L> store_fn{RowStore<RAGGED>{a.out[0], a.out[1], row_byte[0], limit[0]}, wpr, wave, first_wave, lane, limit, inv_n, red, &flip};
    run_program<DT, K, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, store_fn);

    // Lanes past the end of a row that does not fill the lanes exactly must not disturb the reductions.
    const bool exact = n == LPR * wpr * (uint32_t)EC;
    const int core = Spec::core(a);
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        float* acc = s.acc + r * EC;
        uint32_t nvalid[KC];  // valid elements of vector c: 0 or VEC unless the row is ragged
#pragma unroll
        for (int c = 0; c < KC; ++c)
            nvalid[c] = RAGGED ? elems_below<VEC>(s.col[r * KC + c], limit[r]) : (s.col[r * KC + c] < limit[r] ? (uint32_t)VEC : 0u);
        auto valid_elem = [&](int c, int e) { return RAGGED ? (uint32_t)e < nvalid[c] : nvalid[c] != 0u; };
        const bool all_valid = exact && limit[r] != 0u;
        if (core == CORE_SOFTMAX) {
            if (core_mask == 2u) {
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
            } else if (core_mask == 1u) {
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
                    for (int e = 0; e < VEC; ++e) acc[c * VEC + e] = valid_elem(c, e) ? acc[c * VEC + e] : -__builtin_inff();
            }
            float m = acc[0];
#pragma unroll
            for (int e = 1; e < EC; ++e) m = fmaxf(m, acc[e]);
            m = row_allreduce<OpMax, LOG2L>(m, wpr, wave, first_wave, lane, red[0]);
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
            sum = row_allreduce<OpSum, LOG2L>(sum, wpr, wave, first_wave, lane, red[1]);
            const float inv = pf_rcp<PR>(sum);
#pragma unroll
            for (int e = 0; e < EC; ++e) acc[e] *= inv;
        } else if (core == CORE_LAYERNORM) {
            if (!all_valid) {
#pragma unroll
                for (int c = 0; c < KC; ++c)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) acc[c * VEC + e] = valid_elem(c, e) ? acc[c * VEC + e] : 0.0f;
            }
            float s1 = 0.0f;
#pragma unroll
            for (int e = 0; e < EC; ++e) s1 += acc[e];
            const float mean = row_allreduce<OpSum, LOG2L>(s1, wpr, wave, first_wave, lane, red[0]) * inv_n;
            float s2 = 0.0f;
#pragma unroll
            for (int c = 0; c < KC; ++c)
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float d = acc[c * VEC + e] - mean;
                    acc[c * VEC + e] = d;
                    s2 += (all_valid || valid_elem(c, e)) ? d * d : 0.0f;
                }
            const float var = row_allreduce<OpSum, LOG2L>(s2, wpr, wave, first_wave, lane, red[1]) * inv_n;
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
                for (int e = 0; e < VEC; ++e) s2 += (all_valid || valid_elem(c, e)) ? acc[c * VEC + e] * acc[c * VEC + e] : 0.0f;
            const float ms = row_allreduce<OpSum, LOG2L>(s2, wpr, wave, first_wave, lane, red[0]) * inv_n;
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
            if (RAGGED) store_elems<DT>(out_row, s.col[k], elems_below<VEC>(s.col[k], limit[r]), S::pack(s.acc + k * VEC));
            else if (s.col[k] < limit[r]) store_stream(out_row, s.col[k] * (uint32_t)S::ESIZE, S::pack(s.acc + k * VEC));
        }
    }
}

// Reduction cores whose result is one value per row (REDUCE_SUM / MAX / MEAN, keepdim): the epilogue runs
// on that single value and one lane stores it.
template <int DT, int K, bool RAGGED = false, class Spec = GenericSpec>
__global__ void __launch_bounds__(1024) row_reduce_kernel(const ChainArgs a, const RowGeom g) {
    using S = Storage<DT>;
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
    const uint32_t first_wave = wave / wpr * wpr;
    const uint32_t lane_in_row = (wave - first_wave) * 64u + lane;
    const uint32_t limit = row_ok ? n : 0u;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        s.row[k] = row;
        s.col[k] = (lane_in_row + 64u * wpr * k) * VEC;
    }
    const uint64_t row_in = RAGGED ? row64 : min(row64, a.rows - 1u);  // (a row past the end: loads aimed at the last row, discarded)
    load_row_operands<DT, K, K, Spec, RAGGED>(a, s, 0, row_in * n * S::ESIZE, (uint32_t)row_in, limit, limit, 0u, n);
    run_program<DT, K, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStore{});
    auto valid_elem = [&](int k, int e) { return RAGGED ? s.col[k] + (uint32_t)e < limit : s.col[k] < limit; };
    float r;
    if (Spec::core(a) == CORE_REDUCE_MAX) {
        float m = -__builtin_inff();
        float nan_seen = 0.0f;
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float x = s.acc[k * VEC + e];
                if (valid_elem(k, e)) {
                    m = fmaxf(m, x);
                    nan_seen = (x != x) ? 1.0f : nan_seen;
                }
            }
        m = row_allreduce<OpMax>(m, wpr, wave, first_wave, lane, red[0]);
        nan_seen = row_allreduce<OpMax>(nan_seen, wpr, wave, first_wave, lane, red[1]);
        r = nan_seen > 0.0f ? __builtin_nanf("") : m;
    } else {
        float sum = 0.0f;
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
            for (int e = 0; e < VEC; ++e) sum += valid_elem(k, e) ? s.acc[k * VEC + e] : 0.0f;
        r = row_allreduce<OpSum>(sum, wpr, wave, first_wave, lane, red[0]);
        if (Spec::core(a) == CORE_REDUCE_MEAN) r = r / (float)n;
    }
    // epilogue on the row value: immediates and unary steps only (the planner guarantees it)
    LaneState<DT, 1, Spec> t;
    t.row[0] = row;
    t.col[0] = 0;
#pragma unroll
    for (int e = 0; e < VEC; ++e) t.acc[e] = r;
    run_program<DT, 1, Spec>(ProgView<typename Spec::Epi>{a.epi}, t, NoStore{});
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
// RAGGED: the innermost extent is not a multiple of a vector.  The tensors themselves are still 16-byte
// aligned streams (only the last vector is partial), but a vector no longer lies inside one row: broadcast
// operands are gathered per element at (flat index mod operand size).
template <int DT, int K, class Spec, bool RAGGED = false>
__global__ void __launch_bounds__(256) ew_kernel(const ChainArgs a, const uint32_t total_vecs, const uint32_t vecs_per_row) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    LaneState<DT, K, Spec> s;
    const uint32_t base = blockIdx.x * (256u * K) + threadIdx.x;
    const uint64_t total_elems = a.rows * a.n_inner;
    uint32_t gv[K], cnt[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        gv[k] = base + 256u * k;
        if (RAGGED) {
            const uint64_t first = (uint64_t)gv[k] * VEC;
            cnt[k] = first < total_elems ? (uint32_t)(total_elems - first < VEC ? total_elems - first : VEC) : 0u;
            s.row[k] = (uint32_t)(first / a.n_inner);
            s.col[k] = (uint32_t)(first - (uint64_t)s.row[k] * a.n_inner);
        } else {
            cnt[k] = gv[k] < total_vecs ? (uint32_t)VEC : 0u;
            s.row[k] = gv[k] / vecs_per_row;
            s.col[k] = (gv[k] - s.row[k] * vecs_per_row) * VEC;
        }
    }
#pragma unroll
    for (int f = 0; f < Spec::NF; ++f) {
        if (f < Spec::n_full(a)) {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                s.fraw[f][k] = u32x4{0u, 0u, 0u, 0u};
                if (RAGGED && cnt[k] != (uint32_t)VEC) s.fraw[f][k] = load_elems<DT>(a.full[f], (uint64_t)gv[k] * VEC, cnt[k], 0u);
                else if (cnt[k] != 0u) s.fraw[f][k] = load_stream(a.full[f], (uint64_t)gv[k] * 16u);
            }
        }
    }
#pragma unroll
    for (int v = 0; v < Spec::NV; ++v) {
        if (v < Spec::n_vec(a)) {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                s.vraw[v][k] = u32x4{0u, 0u, 0u, 0u};
                if (RAGGED) {
                    // a flat position's element of a broadcast operand is (flat index mod operand size) in every
                    // supported broadcast pattern
                    const VecArg& va = a.vec[v];
                    if (va.numel == 1) {
                        s.vraw[v][k] = S::splat(va.ptr);
                    } else if (Spec::kBcast && va.n_terms != 0u) {
                        // general broadcasting: (row, column) of every element; a vector may run over row ends
                        uint32_t bits[VEC], r = s.row[k], cc = s.col[k];
#pragma unroll
                        for (int e = 0; e < VEC; ++e) {
                            while (cc >= a.n_inner) {
                                cc -= a.n_inner;
                                ++r;
                            }
                            bits[e] = 0u;
                            if ((uint32_t)e < cnt[k]) {
                                const uint32_t off = vec_offset<Spec::kBcast>(va, r, cc, a.n_inner);
                                bits[e] = DT == DT_F32 ? static_cast<const uint32_t*>(va.ptr)[off] : (uint32_t) static_cast<const uint16_t*>(va.ptr)[off];
                            }
                            ++cc;
                        }
                        if (DT == DT_F32) s.vraw[v][k] = u32x4{bits[0], bits[1], bits[2], bits[3]};
                        else
                            s.vraw[v][k] = u32x4{bits[0] | (bits[1 % VEC] << 16), bits[2 % VEC] | (bits[3 % VEC] << 16),
                                                 bits[4 % VEC] | (bits[5 % VEC] << 16), bits[6 % VEC] | (bits[7 % VEC] << 16)};
                    } else {
                        const uint32_t m0 = (uint32_t)(((uint64_t)gv[k] * VEC) % va.numel);
                        uint32_t bits[VEC];
#pragma unroll
                        for (int e = 0; e < VEC; ++e) {
                            uint32_t off = m0 + (uint32_t)e;
                            off = off >= va.numel ? off % va.numel : off;
                            bits[e] = 0u;
                            if ((uint32_t)e < cnt[k])
                                bits[e] = DT == DT_F32 ? static_cast<const uint32_t*>(va.ptr)[off] : (uint32_t) static_cast<const uint16_t*>(va.ptr)[off];
                        }
                        if (DT == DT_F32) s.vraw[v][k] = u32x4{bits[0], bits[1], bits[2], bits[3]};
                        else
                            s.vraw[v][k] = u32x4{bits[0] | (bits[1 % VEC] << 16), bits[2 % VEC] | (bits[3 % VEC] << 16),
                                                 bits[4 % VEC] | (bits[5 % VEC] << 16), bits[6 % VEC] | (bits[7 % VEC] << 16)};
                    }
                } else if (cnt[k] != 0u) {
                    s.vraw[v][k] = load_vec_operand<DT, Spec::kVecMode>(a.vec[v], s.row[k], s.col[k], a.n_inner);
                }
            }
        }
    }
    const FlatStore<RAGGED> flat{a.out[0], a.out[1], total_vecs, vecs_per_row, total_elems};
    auto store_fn = [&](int slot, const LaneState<DT, K, Spec>& st) { flat(slot, st, gv); };
    run_program<DT, K, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, store_fn);
#pragma unroll
    for (int k = 0; k < K; ++k) {
        if (RAGGED && cnt[k] != (uint32_t)VEC) store_elems<DT>(a.out[0], (uint64_t)gv[k] * VEC, cnt[k], S::pack(s.acc + k * VEC));
        else if (cnt[k] != 0u) store_stream(a.out[0], (uint64_t)gv[k] * 16u, S::pack(s.acc + k * VEC));
    }
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
