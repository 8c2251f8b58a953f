// Row family, streaming variant: rows that do not fit the registers of one workgroup.
//
// A workgroup owns a row and walks it twice in chunks of blockDim * K vectors.  The first walk runs the
// prologue and accumulates the row statistics per lane in a form that can be merged (running maximum and
// rescaled sum for softmax, (count, mean, M2) for LayerNorm, a sum of squares for RMSNorm, a sum or a
// maximum for the keep-dim reductions); one block-scope exchange merges them.  The second walk re-reads the
// operands (the row was just touched, so this read is served by the caches for rows of up to a few MB),
// re-runs the prologue, normalises, runs the epilogue and stores.  HBM traffic stays at one read and one
// write per element as long as a row fits the last-level cache; what the register-resident kernels keep in
// registers this one recomputes.
//
// The synchronisation structure is the same as in the resident kernels (paper section 5.1: one
// reduce -> broadcast exchange at workgroup scope); only the slice held per lane differs.
#pragma once
#include "pf_row_kernels.hpp"

namespace pf {

constexpr int kStreamThreads = 512;
constexpr int kStreamWaves = kStreamThreads / 64;

// merge (count, mean, M2) triples over the workgroup; every thread gets the result
PF_DEVICE Stat block_merge_stat(Stat st, uint32_t wave, uint32_t lane, float* lds) {
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) st = stat_merge(st, stat_shfl_xor(st, m));
    if (lane == 0) {
        lds[wave * 3 + 0] = st.n;
        lds[wave * 3 + 1] = st.mean;
        lds[wave * 3 + 2] = st.m2;
    }
    __syncthreads();
    Stat r = {lds[0], lds[1], lds[2]};
    for (int w = 1; w < kStreamWaves; ++w) r = stat_merge(r, Stat{lds[w * 3], lds[w * 3 + 1], lds[w * 3 + 2]});
    return r;
}

template <int DT, bool RAGGED, class Spec>
__global__ void __launch_bounds__(kStreamThreads) row_stream_kernel(const ChainArgs a) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    constexpr int K = 2;
    constexpr int E = K * VEC;
    constexpr bool PR = S::PRECISE;
    __shared__ float red[2][16];
    __shared__ float lds_stat[kStreamWaves * 3];

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t row = blockIdx.x;
    const uint32_t n = a.n_inner;
    const uint64_t row_byte = (uint64_t)row * n * S::ESIZE;
    const uint32_t chunk = (uint32_t)kStreamThreads * E;
    const int core = Spec::core(a);

    // causal mask: columns beyond the diagonal never need loading (they are overwritten by the mask, or the
    // folded mask treats them as -inf)
    uint32_t i_row = 0, load_limit = n;
    if (a.mask_si != 0u) {
        i_row = row - fast_div(row, a.mask_div) * a.mask_si;
        const uint32_t keep = (i_row + VEC) / VEC * VEC;
        load_limit = n < keep ? n : keep;
    }
    const bool fill_inf = a.core_mask == 2u;
    const uint32_t fill = fill_inf ? (DT == DT_F32 ? 0xff800000u : (DT == DT_F16 ? 0xfc00fc00u : 0xff80ff80u)) : 0u;
    const float cs = a.core_scale;
    const float c2 = cs * kLog2e;

    LaneState<DT, K, Spec> s;
    auto load_chunk = [&](uint32_t c0) {
#pragma unroll
        for (int k = 0; k < K; ++k) {
            s.row[k] = row;
            s.col[k] = c0 + ((uint32_t)k * kStreamThreads + threadIdx.x) * VEC;
        }
        load_row_operands<DT, K, K, Spec, RAGGED>(a, s, 0, row_byte, row, load_limit, n, fill, n);
    };
    // the mask folded into a softmax core, applied by position
    auto folded_mask = [&]() {
        if (core == CORE_SOFTMAX && a.core_mask != 0u) {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const int32_t last = (int32_t)i_row - (int32_t)s.col[k];
#pragma unroll
                for (int e = 0; e < VEC; ++e) s.acc[k * VEC + e] = (e > last) ? -__builtin_inff() : s.acc[k * VEC + e];
            }
        }
    };
    auto valid_elem = [&](int k, int e) { return RAGGED ? s.col[k] + (uint32_t)e < n : s.col[k] < n; };

    // ---- first walk: statistics
    float run_max = -__builtin_inff(), run_sum = 0.0f, nan_seen = 0.0f;
    LaneAcc la;
    for (uint32_t c0 = 0; c0 < n; c0 += chunk) {
        load_chunk(c0);
        run_program<DT, K, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStore{});
        folded_mask();
        if (core == CORE_SOFTMAX) {
            float cm = -__builtin_inff();
#pragma unroll
            for (int k = 0; k < K; ++k)
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    s.acc[k * VEC + e] = valid_elem(k, e) ? s.acc[k * VEC + e] : -__builtin_inff();
                    cm = fmaxf(cm, s.acc[k * VEC + e]);
                }
            const float m_new = fmaxf(run_max, cm);
            // exp(c * (x - m)) with m the running maximum; -inf terms contribute nothing.  A NaN element slips
            // past the maximum but poisons the sum, hence the whole row, as the definition does.
            if (m_new != run_max) run_sum *= PR ? expf((run_max - m_new) * cs) : __builtin_amdgcn_exp2f((run_max - m_new) * c2);
            run_max = m_new;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float x = s.acc[e];
                const float t = PR ? expf((x - m_new) * cs) : __builtin_amdgcn_exp2f((x - m_new) * c2);
                run_sum += (x == -__builtin_inff()) ? 0.0f : t;
            }
        } else if (core == CORE_LAYERNORM) {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                if (!RAGGED || s.col[k] + (uint32_t)VEC <= n) {
                    if (s.col[k] < n) la.template add_vector<VEC>(s.acc + k * VEC);
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e)
                        if (s.col[k] + (uint32_t)e < n) la.template add_vector<1>(s.acc + k * VEC + e);
                }
            }
        } else if (core == CORE_REDUCE_MAX) {
#pragma unroll
            for (int k = 0; k < K; ++k)
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float x = s.acc[k * VEC + e];
                    if (valid_elem(k, e)) {
                        run_max = fmaxf(run_max, x);
                        nan_seen = (x != x) ? 1.0f : nan_seen;
                    }
                }
        } else {  // RMSNorm: sum of squares; REDUCE_SUM / REDUCE_MEAN: sum
            const bool sq = core == CORE_RMSNORM;
#pragma unroll
            for (int k = 0; k < K; ++k)
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float x = s.acc[k * VEC + e];
                    run_sum += valid_elem(k, e) ? (sq ? x * x : x) : 0.0f;
                }
        }
    }

    // ---- block-scope exchange
    float row_max = 0.0f, row_inv = 0.0f, mean = 0.0f, rstd = 0.0f, value = 0.0f;
    if (core == CORE_SOFTMAX) {
        row_max = row_allreduce<OpMax>(run_max, kStreamWaves, wave, 0u, lane, red[0]);
        if (run_max != row_max) run_sum *= PR ? expf((run_max - row_max) * cs) : __builtin_amdgcn_exp2f((run_max - row_max) * c2);
        const float sum = row_allreduce<OpSum>(run_sum, kStreamWaves, wave, 0u, lane, red[1]);
        row_inv = pf_rcp<PR>(sum);
    } else if (core == CORE_LAYERNORM) {
        const Stat st = block_merge_stat(la.finish(), wave, lane, lds_stat);
        mean = st.mean;
        rstd = pf_rsqrt<PR>(st.m2 / (float)n + a.eps);
    } else if (core == CORE_RMSNORM) {
        const float ss = row_allreduce<OpSum>(run_sum, kStreamWaves, wave, 0u, lane, red[0]);
        rstd = pf_rsqrt<PR>(ss / (float)n + a.eps);
    } else if (core == CORE_REDUCE_MAX) {
        const float m = row_allreduce<OpMax>(run_max, kStreamWaves, wave, 0u, lane, red[0]);
        const float ns = row_allreduce<OpMax>(nan_seen, kStreamWaves, wave, 0u, lane, red[1]);
        value = ns > 0.0f ? __builtin_nanf("") : m;
    } else {
        value = row_allreduce<OpSum>(run_sum, kStreamWaves, wave, 0u, lane, red[0]);
        if (core == CORE_REDUCE_MEAN) value = value / (float)n;
    }

    if (core == CORE_REDUCE_SUM || core == CORE_REDUCE_MAX || core == CORE_REDUCE_MEAN) {
        // one value per row: the epilogue (unary and constant steps only) runs on it, one lane stores it
        LaneState<DT, 1, Spec> t;
        t.row[0] = row;
        t.col[0] = 0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) t.acc[e] = value;
        run_program<DT, 1, Spec>(ProgView<typename Spec::Epi>{a.epi}, t, NoStore{});
        if (threadIdx.x == 0) {
            if (DT == DT_F32) {
                static_cast<float*>(a.out[0])[row] = t.acc[0];
            } else {
                const u32x4 packed = S::pack(t.acc);
                static_cast<uint16_t*>(a.out[0])[row] = (uint16_t)(packed[0] & 0xffffu);
            }
        }
        return;
    }

    // ---- second walk: normalise and store
    const RowStore<RAGGED> store_fn{a.out[0], a.out[1], row_byte, n};
    char* out_row = static_cast<char*>(a.out[0]) + row_byte;
    for (uint32_t c0 = 0; c0 < n; c0 += chunk) {
        load_chunk(c0);
        run_program<DT, K, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, store_fn);
        folded_mask();
        if (core == CORE_SOFTMAX) {
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float t = PR ? expf((s.acc[e] - row_max) * cs) : __builtin_amdgcn_exp2f((s.acc[e] - row_max) * c2);
                s.acc[e] = t * row_inv;
            }
        } else {
            float gm[E], bt[E];
#pragma unroll
            for (int e = 0; e < E; ++e) {
                gm[e] = 1.0f;
                bt[e] = 0.0f;
            }
            if (Spec::gamma(a) >= 0) fetch_vec<DT, K, Spec>(s, Spec::gamma(a), gm);
            if (core == CORE_LAYERNORM && Spec::beta(a) >= 0) fetch_vec<DT, K, Spec>(s, Spec::beta(a), bt);
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = (s.acc[e] - mean) * rstd * gm[e] + bt[e];
        }
        run_program<DT, K, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, store_fn);
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (RAGGED) store_elems<DT>(out_row, s.col[k], elems_below<VEC>(s.col[k], n), S::pack(s.acc + k * VEC));
            else if (s.col[k] < n) store_stream(out_row, s.col[k] * (uint32_t)S::ESIZE, S::pack(s.acc + k * VEC));
        }
    }
}

}  // namespace pf
