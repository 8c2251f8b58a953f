// Attention family: one new token against cached keys and values, as ONE memory-bound kernel.
//
//   K' = concat(K, k),  V' = concat(V, v),  s = K' q * scale,  p = softmax(s),  o = p V'
//
// With a sequence length of one both matrix products of the attention layer are matrix-vector products,
// bound by reading the cache once (paper section 8, the GPT-2 case study).  The two products have the same
// shape but are laid out differently here, as in the paper's best plan: the first contracts the contiguous
// head dimension, so the lanes that share a cache row combine their partial dot products by lane
// permutations; the second contracts the row dimension, so every lane accumulates its own columns over the
// rows it has seen and the row groups are combined once at the end.  Keys and values are loaded once, as
// 16-byte vectors, all loads of a workgroup's slice in flight before the first use; scores and probabilities
// never leave registers; the concatenations cost nothing unless the grown caches are asked for as outputs.
//
// A head's rows are split over several workgroups (a head alone would leave most of the device idle).
// Each split produces a partial result in the usual mergeable form (maximum, sum of exponentials, weighted
// value sum); the workgroup whose arrival completes the head's counter merges them -- a device-scope
// synchronisation (section 5.1) in which nobody waits: every workgroup but the last simply ends.
#include "pf_device.hpp"
#include "pf_launch.h"

namespace pf {

PF_DEVICE float shfl_xor_f(float v, int mask) { return __shfl_xor(v, mask, 64); }

// Publish a slice's partial result (weighted value sum of column `tid` in o_mine, maximum m, sum of exponentials
// l_blk); the workgroup whose arrival completes the head's counter merges all slices and writes the output row.
// lds_o is workgroup scratch of 4 x 256 floats, s_last one shared word.
template <int DT>
PF_DEVICE void finish_slice(const AttnArgs& a, uint32_t head, uint32_t split, float o_mine, float m, float l_blk,
                            float (*lds_o)[256], uint32_t* s_last_p) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    constexpr bool PR = S::PRECISE;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t d = a.d;
    const uint32_t n_split = gridDim.x;
    float* part = a.ws_partial + ((uint64_t)head * n_split + split) * a.part_stride;
    if (n_split == 1u) {
        if (tid < d) {
            const float r = PR ? o_mine / l_blk : o_mine * __builtin_amdgcn_rcpf(l_blk);
            if (DT == DT_F32) static_cast<float*>(a.o)[(uint64_t)head * d + tid] = r;
            else {
                float tmp[VEC] = {r};
                static_cast<uint16_t*>(a.o)[(uint64_t)head * d + tid] = (uint16_t)(S::pack(tmp)[0] & 0xffffu);
            }
        }
        return;
    }
    // published with device-coherent stores: the merging workgroup may run on another compute die
    if (tid < d) __hip_atomic_store(part + tid, o_mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tid == 0) {
        __hip_atomic_store(part + d, m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(part + d + 1u, l_blk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // The arrival below must not become visible before these words: every wave waits until its device-coherent
    // (write-through) stores have been acknowledged, then the barrier lets lane 0 count the slice in.  (A
    // workgroup-scope release does not wait for outstanding stores on this device; an agent-scope one would write
    // back the whole L2.)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
        const uint32_t before = __hip_atomic_fetch_add(a.ws_counter + head, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = before + 1u == n_split;
        // nobody touches the counter again before the next launch on this stream: re-arm it
        if (last) __hip_atomic_store(a.ws_counter + head, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_last_p = last ? 1u : 0u;
    }
    __syncthreads();
    if (!*s_last_p) return;

    // ---- the last workgroup of the head merges the slices: o = sum_s o_s e^(m_s - M) / sum_s l_s e^(m_s - M).
    // All 256 threads take part: thread (g, c) sums column c over the slices s = g, g + G, ... (G = 256 / d'
    // groups, d' = d rounded up to a power of two), so the loads of many slices are in flight together; the
    // groups are then combined through LDS.
    const float* base = a.ws_partial + (uint64_t)head * n_split * a.part_stride;
    uint32_t dp = 1;
    while (dp < d) dp <<= 1;
    const uint32_t groups = 256u / dp, g = tid / dp, c = tid - g * dp;
    float big = -__builtin_inff();
    for (uint32_t s = lane; s < n_split; s += 64u)
        big = fmaxf(big, __hip_atomic_load(base + (uint64_t)s * a.part_stride + d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    for (int msk = 1; msk < 64; msk <<= 1) big = fmaxf(big, shfl_xor_f(big, msk));  // every wave finds the same maximum
    float num = 0.0f, den = 0.0f;
    for (uint32_t s = g; s < n_split; s += groups) {
        const float* ps = base + (uint64_t)s * a.part_stride;
        const float ms = __hip_atomic_load(ps + d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float ls = __hip_atomic_load(ps + d + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float os = c < d ? __hip_atomic_load(ps + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0f;
        const float w = PR ? expf(ms - big) : __builtin_amdgcn_exp2f((ms - big) * kLog2e);
        num = __builtin_fmaf(os, w, num);
        den = __builtin_fmaf(ls, w, den);
    }
    float* red_num = &lds_o[0][0];  // [groups][dp] (the per-wave partials are no longer needed)
    float* red_den = &lds_o[2][0];
    __syncthreads();
    red_num[tid] = num;
    red_den[tid] = den;
    __syncthreads();
    if (tid < d) {
        num = 0.0f;
        den = 0.0f;
        for (uint32_t gg = 0; gg < groups; ++gg) {
            num += red_num[gg * dp + tid];
            den += red_den[gg * dp + tid];
        }
        const float r = PR ? num / den : num * __builtin_amdgcn_rcpf(den);
        if (DT == DT_F32) static_cast<float*>(a.o)[(uint64_t)head * d + tid] = r;
        else {
            float tmp[VEC] = {r};
            static_cast<uint16_t*>(a.o)[(uint64_t)head * d + tid] = (uint16_t)(S::pack(tmp)[0] & 0xffffu);
        }
    }
}

// The 16-byte pieces of one key row and one value row, without a branch: rows below t come from the caches, row t (the
// appended one) from the new vectors; a row past the end reads memory that exists (the new vectors, or the last cache
// row) and is zeroed.  Behind a guard
// every load would merge with a fill value at the join, which the compiler resolves by waiting for it: the loads of a
// lane, all independent, would then go to memory one round trip after the other.
template <int DT>
PF_DEVICE void load_key_value(const AttnArgs& a, uint32_t head, uint32_t row, uint32_t in_row, uint64_t head_vec, u32x4& k, u32x4& v) {
    using S = Storage<DT>;
    // (a chain that does not append has no new vectors: rows past the end then read the last cache row, which exists
    // because such a chain has t = t_total >= 1)
    const bool from_cache = row < a.t || a.k_new == nullptr || a.v_new == nullptr;
    const uint32_t row_c = min(row, a.t - 1u);  // (only used when from_cache, and then t >= 1)
    const uint64_t off = (from_cache ? ((uint64_t)head * a.t + row_c) * a.d + in_row * S::VEC : head_vec) * S::ESIZE;
    const u32x4 gk = load_stream(from_cache ? a.k_cache : a.k_new, off);
    const u32x4 gv = load_stream(from_cache ? a.v_cache : a.v_new, off);
    const bool keep = row < a.t_total;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t wk = gk[j], wv = gv[j];
        k[j] = keep ? wk : 0u;
        v[j] = keep ? wv : 0u;
    }
}

// ---- polled merge ---------------------------------------------------------------------------------------------
// Every slice, the head's last one included, publishes its partial result as self-describing words: all-ones means
// "not written in this launch" (a NaN that arithmetic does not produce; a result with that payload is published as the
// canonical NaN).  The head's last slice -- dispatched after the others, which never wait, so its wait ends -- reads
// the words of all slices, re-reading the ones still empty, puts them back to all-ones for the next launch and merges.
// The critical path is one coherent store and one coherent load; the counted merge above has four trips behind each
// other (the stores' acknowledgement, the counter, the maxima, the partial results), which is most of what a decode
// step at batch 1 costs.  Every wait is bounded: after spin_limit re-reads the error word is set and what is missing is
// left out.
constexpr uint32_t kAttnEmpty = ~0u;
PF_DEVICE uint32_t attn_word(float x) {
    const uint32_t w = __builtin_bit_cast(uint32_t, x);
    return w == kAttnEmpty ? 0x7fc00000u : w;
}
PF_DEVICE uint32_t attn_wait(const AttnArgs& a, uint32_t* word, uint32_t* spins) {
    for (;;) {
        const uint32_t w = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (w != kAttnEmpty) return w;
        if (++*spins > a.spin_limit) {
            __hip_atomic_store(a.ws_error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return kAttnEmpty;
        }
        __builtin_amdgcn_s_sleep(4);
    }
}

template <int DT>
PF_DEVICE void finish_slice_polled(const AttnArgs& a, uint32_t head, uint32_t split, float o_mine, float m, float l_blk, float (*lds_o)[256]) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    constexpr bool PR = S::PRECISE;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t d = a.d;
    const uint32_t n_split = gridDim.x;
    uint32_t* words = reinterpret_cast<uint32_t*>(a.ws_partial);
    uint32_t* part = words + ((uint64_t)head * n_split + split) * a.part_stride;
    if (tid < d) __hip_atomic_store(part + tid, attn_word(o_mine), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tid == 0) {
        __hip_atomic_store(part + d, attn_word(m), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(part + d + 1u, attn_word(l_blk), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (split + 1u != n_split) return;

    // ---- the head's last slice merges: o = sum_s o_s e^(m_s - M) / sum_s l_s e^(m_s - M), thread (g, c) summing column c
    // over the slices s = g, g + G, ... as in the counted merge
    uint32_t* base = words + (uint64_t)head * n_split * a.part_stride;
    uint32_t spins = 0;
    uint32_t dp = 1;
    while (dp < d) dp <<= 1;
    const uint32_t groups = 256u / dp, g = tid / dp, c = tid - g * dp;
    float big = -__builtin_inff();
    for (uint32_t s = lane; s < n_split; s += 64u) {  // every wave finds the same maximum
        const uint32_t w = attn_wait(a, base + (uint64_t)s * a.part_stride + d, &spins);
        if (w != kAttnEmpty) big = fmaxf(big, __builtin_bit_cast(float, w));
    }
    for (int msk = 1; msk < 64; msk <<= 1) big = fmaxf(big, shfl_xor_f(big, msk));
    float num = 0.0f, den = 0.0f;
    for (uint32_t s = g; s < n_split; s += groups) {
        uint32_t* ps = base + (uint64_t)s * a.part_stride;
        // the three words of a slice are asked for together; what is still empty is waited for afterwards
        uint32_t wm = __hip_atomic_load(ps + d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t wl = __hip_atomic_load(ps + d + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t wo = c < d ? __hip_atomic_load(ps + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
        if (wm == kAttnEmpty) wm = attn_wait(a, ps + d, &spins);
        if (wl == kAttnEmpty) wl = attn_wait(a, ps + d + 1u, &spins);
        if (wo == kAttnEmpty) wo = attn_wait(a, ps + c, &spins);
        if (c < d) __hip_atomic_store(ps + c, kAttnEmpty, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // (nobody else reads this word)
        if (wm == kAttnEmpty || wl == kAttnEmpty || wo == kAttnEmpty) continue;  // a wait gave up: the slice is left out
        const float ms = __builtin_bit_cast(float, wm), ls = __builtin_bit_cast(float, wl), os = __builtin_bit_cast(float, wo);
        const float w = PR ? expf(ms - big) : __builtin_amdgcn_exp2f((ms - big) * kLog2e);
        num = __builtin_fmaf(os, w, num);
        den = __builtin_fmaf(ls, w, den);
    }
    float* red_num = &lds_o[0][0];  // [groups][dp] (the per-wave partials are no longer needed)
    float* red_den = &lds_o[2][0];
    __syncthreads();  // (also: every thread has read the maxima and sums it needs)
    red_num[tid] = num;
    red_den[tid] = den;
    // the maxima and sums were read by many threads: put back to "empty" once everybody is past the barrier above
    for (uint32_t s = tid; s < n_split; s += 256u) {
        __hip_atomic_store(base + (uint64_t)s * a.part_stride + d, kAttnEmpty, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(base + (uint64_t)s * a.part_stride + d + 1u, kAttnEmpty, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (tid < d) {
        num = 0.0f;
        den = 0.0f;
        for (uint32_t gg = 0; gg < groups; ++gg) {
            num += red_num[gg * dp + tid];
            den += red_den[gg * dp + tid];
        }
        const float r = PR ? num / den : num * __builtin_amdgcn_rcpf(den);
        if (DT == DT_F32) static_cast<float*>(a.o)[(uint64_t)head * d + tid] = r;
        else {
            float tmp[VEC] = {r};
            static_cast<uint16_t*>(a.o)[(uint64_t)head * d + tid] = (uint16_t)(S::pack(tmp)[0] & 0xffffu);
        }
    }
}

template <int DT, int NV>
__global__ void __launch_bounds__(256) attn_decode_kernel(const AttnArgs a) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    constexpr bool PR = S::PRECISE;
    __shared__ float lds_m[4], lds_l[4];
    __shared__ float lds_o[4][256];  // per-wave partial output, head dimension <= 256
    __shared__ uint32_t s_last;

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63u, wave = tid >> 6;
    const uint32_t lpr = a.lanes_per_row;            // lanes that share one cache row (power of two, <= 64)
    const uint32_t in_row = tid & (lpr - 1u);        // which 16-byte piece of the row
    const uint32_t row_in_step = tid >> a.log2_lpr;  // which row of a step of 256 / lpr rows
    const uint32_t rps = 256u >> a.log2_lpr;
    const uint32_t head = blockIdx.y, split = blockIdx.x;
    const uint32_t row0 = split * (uint32_t)NV * rps;
    const uint32_t d = a.d, t_total = a.t_total;

    const uint64_t head_vec = (uint64_t)head * d + in_row * VEC;  // element offset inside q / k / v / o
    float qf[VEC];
    S::unpack(load_cached(a.q, head_vec * S::ESIZE), qf);

    // ---- every key and value vector of this slice, loaded before anything is used
    u32x4 kraw[NV], vraw[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        load_key_value<DT>(a, head, row0 + (uint32_t)i * rps + row_in_step, in_row, head_vec, kraw[i], vraw[i]);
    }
    // the grown caches, if they are outputs
    if (a.k_out != nullptr || a.v_out != nullptr) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const uint32_t row = row0 + (uint32_t)i * rps + row_in_step;
            if (row < t_total) {
                const uint64_t off = (((uint64_t)head * t_total + row) * d + in_row * VEC) * S::ESIZE;
                if (a.k_out != nullptr) store_stream(a.k_out, off, kraw[i]);
                if (a.v_out != nullptr) store_stream(a.v_out, off, vraw[i]);
            }
        }
    }

    // ---- first product: contract the head dimension (lanes of a row combine by lane permutations)
    float sc[NV];
    float m = -__builtin_inff();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const uint32_t row = row0 + (uint32_t)i * rps + row_in_step;
        float kf[VEC];
        S::unpack(kraw[i], kf);
        float dot = 0.0f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) dot = __builtin_fmaf(kf[e], qf[e], dot);
        for (uint32_t msk = 1; msk < lpr; msk <<= 1) dot += shfl_xor_f(dot, (int)msk);
        sc[i] = row < t_total ? dot * a.scale : -__builtin_inff();
        m = fmaxf(m, sc[i]);
    }
    // the slice's maximum: over the row groups of the wave, then over the four waves
    for (uint32_t msk = lpr; msk < 64u; msk <<= 1) m = fmaxf(m, shfl_xor_f(m, (int)msk));
    if (lane == 0) lds_m[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(lds_m[0], lds_m[1]), fmaxf(lds_m[2], lds_m[3]));

    // ---- softmax numerators and the second product: contract the row dimension (per-lane accumulation)
    float l = 0.0f;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        // exp(-inf - m) = 0 for rows past the end; m is finite because every slice holds at least one row
        const float p = PR ? expf(sc[i] - m) : __builtin_amdgcn_exp2f((sc[i] - m) * kLog2e);
        l += p;
        float vf[VEC];
        S::unpack(vraw[i], vf);
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = __builtin_fmaf(p, vf[e], acc[e]);
    }
    for (uint32_t msk = lpr; msk < 64u; msk <<= 1) {
        l += shfl_xor_f(l, (int)msk);
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] += shfl_xor_f(acc[e], (int)msk);
    }
    if (lane == 0) lds_l[wave] = l;
    if (lane < lpr) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) lds_o[wave][in_row * VEC + e] = acc[e];
    }
    __syncthreads();

    // ---- the slice's partial result
    float o_mine = 0.0f;
    if (tid < d) o_mine = lds_o[0][tid] + lds_o[1][tid] + lds_o[2][tid] + lds_o[3][tid];
    const float l_blk = lds_l[0] + lds_l[1] + lds_l[2] + lds_l[3];
    if (a.polled != 0u && gridDim.x > 1u) finish_slice_polled<DT>(a, head, split, o_mine, m, l_blk, lds_o);
    else finish_slice<DT>(a, head, split, o_mine, m, l_blk, lds_o, &s_last);
}

// Streaming variant: a workgroup walks a longer slice of the head in chunks of NV steps, the loads of the next
// chunk in flight while the current one is consumed (two register buffers).  Every lane keeps its own running
// (maximum, sum of exponentials, weighted value sum) over the rows it has seen -- the mergeable form again, so
// nothing crosses lanes per chunk except the dot products of the lanes that share a row; row groups, waves and
// finally slices are merged once at the end.  Fewer, longer slices mean fewer partial results and fewer
// workgroups that sit through the publish / count / merge tail with nothing in flight.
template <int DT, int NV>
__global__ void __launch_bounds__(256) attn_decode_stream_kernel(const AttnArgs a) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    constexpr bool PR = S::PRECISE;
    __shared__ float lds_m[4], lds_l[4];
    __shared__ float lds_o[4][256];
    __shared__ uint32_t s_last;

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63u, wave = tid >> 6;
    const uint32_t lpr = a.lanes_per_row;
    const uint32_t in_row = tid & (lpr - 1u);
    const uint32_t row_in_step = tid >> a.log2_lpr;
    const uint32_t rps = 256u >> a.log2_lpr;
    const uint32_t head = blockIdx.y, split = blockIdx.x;
    const uint32_t chunk_rows = (uint32_t)NV * rps;
    const uint32_t d = a.d, t_total = a.t_total;
    const uint32_t row_begin = split * a.chunks * chunk_rows;
    const uint32_t row_end = min(t_total, row_begin + a.chunks * chunk_rows);
    const uint32_t n_chunks = (row_end - row_begin + chunk_rows - 1u) / chunk_rows;  // >= 1: the planner leaves no slice empty

    const uint64_t head_vec = (uint64_t)head * d + in_row * VEC;
    float qf[VEC];
    S::unpack(load_cached(a.q, head_vec * S::ESIZE), qf);
    auto neg_exp = [](float x) { return PR ? expf(x) : __builtin_amdgcn_exp2f(x * kLog2e); };

    auto load_chunk = [&](uint32_t c, u32x4 (&kr)[NV], u32x4 (&vr)[NV]) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            load_key_value<DT>(a, head, row_begin + c * chunk_rows + (uint32_t)i * rps + row_in_step, in_row, head_vec, kr[i], vr[i]);
        }
    };
    float m = -__builtin_inff(), l = 0.0f, acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;
    auto consume = [&](uint32_t c, const u32x4 (&kr)[NV], const u32x4 (&vr)[NV]) {
        // the grown caches, if they are outputs
        if (a.k_out != nullptr || a.v_out != nullptr) {
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const uint32_t row = row_begin + c * chunk_rows + (uint32_t)i * rps + row_in_step;
                if (row < t_total) {
                    const uint64_t off = (((uint64_t)head * t_total + row) * d + in_row * VEC) * S::ESIZE;
                    if (a.k_out != nullptr) store_stream(a.k_out, off, kr[i]);
                    if (a.v_out != nullptr) store_stream(a.v_out, off, vr[i]);
                }
            }
        }
        float sc[NV], cm = -__builtin_inff();
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const uint32_t row = row_begin + c * chunk_rows + (uint32_t)i * rps + row_in_step;
            float kf[VEC];
            S::unpack(kr[i], kf);
            float dot = 0.0f;
#pragma unroll
            for (int e = 0; e < VEC; ++e) dot = __builtin_fmaf(kf[e], qf[e], dot);
            for (uint32_t msk = 1; msk < lpr; msk <<= 1) dot += shfl_xor_f(dot, (int)msk);
            sc[i] = row < t_total ? dot * a.scale : -__builtin_inff();
            cm = fmaxf(cm, sc[i]);
        }
        const float m_new = fmaxf(m, cm);
        if (m_new == -__builtin_inff()) return;  // this lane has not seen a row yet
        const float keep = m == -__builtin_inff() ? 0.0f : neg_exp(m - m_new);
        l *= keep;
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] *= keep;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const float p = neg_exp(sc[i] - m_new);  // exp(-inf) = 0 for rows past the end
            l += p;
            float vf[VEC];
            S::unpack(vr[i], vf);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = __builtin_fmaf(p, vf[e], acc[e]);
        }
        m = m_new;
    };

    u32x4 k0[NV], v0[NV], k1[NV], v1[NV];
    load_chunk(0u, k0, v0);
    for (uint32_t c = 0; c < n_chunks; c += 2u) {
        if (c + 1u < n_chunks) load_chunk(c + 1u, k1, v1);
        consume(c, k0, v0);
        if (c + 1u < n_chunks) {
            if (c + 2u < n_chunks) load_chunk(c + 2u, k0, v0);
            consume(c + 1u, k1, v1);
        }
    }

    // ---- merge the row groups of the wave, then the four waves
    auto weight = [&](float mine, float top) { return mine == -__builtin_inff() ? 0.0f : neg_exp(mine - top); };
    for (uint32_t msk = lpr; msk < 64u; msk <<= 1) {
        const float m_o = shfl_xor_f(m, (int)msk), l_o = shfl_xor_f(l, (int)msk);
        const float top = fmaxf(m, m_o);
        const float wa = weight(m, top), wb = weight(m_o, top);
        l = l * wa + l_o * wb;
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = acc[e] * wa + shfl_xor_f(acc[e], (int)msk) * wb;
        m = top;
    }
    if (lane == 0) {
        lds_m[wave] = m;
        lds_l[wave] = l;
    }
    if (lane < lpr) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) lds_o[wave][in_row * VEC + e] = acc[e];
    }
    __syncthreads();
    const float top = fmaxf(fmaxf(lds_m[0], lds_m[1]), fmaxf(lds_m[2], lds_m[3]));
    float o_mine = 0.0f, l_blk = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const float ww = weight(lds_m[w], top);
        l_blk += lds_l[w] * ww;
        if (tid < d) o_mine += lds_o[w][tid] * ww;
    }
    if (a.polled != 0u && gridDim.x > 1u) finish_slice_polled<DT>(a, head, split, o_mine, top, l_blk, lds_o);
    else finish_slice<DT>(a, head, split, o_mine, top, l_blk, lds_o, &s_last);
}

template <int DT>
static hipError_t launch_attn_dt(const AttnArgs& a, int variant, int nv, dim3 grid, hipStream_t st) {
    if (variant == 1) {
        switch (nv) {
            case 2: hipLaunchKernelGGL((attn_decode_stream_kernel<DT, 2>), grid, dim3(256), 0, st, a); break;
            case 4: hipLaunchKernelGGL((attn_decode_stream_kernel<DT, 4>), grid, dim3(256), 0, st, a); break;
            default: return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
    switch (nv) {
        case 1: hipLaunchKernelGGL((attn_decode_kernel<DT, 1>), grid, dim3(256), 0, st, a); break;
        case 2: hipLaunchKernelGGL((attn_decode_kernel<DT, 2>), grid, dim3(256), 0, st, a); break;
        case 4: hipLaunchKernelGGL((attn_decode_kernel<DT, 4>), grid, dim3(256), 0, st, a); break;
        case 8: hipLaunchKernelGGL((attn_decode_kernel<DT, 8>), grid, dim3(256), 0, st, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_attn_decode(int dtype, const AttnArgs& a, int variant, int nv, dim3 grid, hipStream_t st) {
    switch (dtype) {
        case DT_F32: return launch_attn_dt<DT_F32>(a, variant, nv, grid, st);
        case DT_F16: return launch_attn_dt<DT_F16>(a, variant, nv, grid, st);
        case DT_BF16: return launch_attn_dt<DT_BF16>(a, variant, nv, grid, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace pf
