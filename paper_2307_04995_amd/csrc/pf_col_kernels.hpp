// Column family: layer / RMS normalisation over a dimension that is NOT the innermost one.
//
// A channels-first tensor [outer, C, S] (S = everything after the normalised dimension, contiguous) normalised
// over C is usually written as: move C to the end, normalise rows, move it back -- three kernels and three times
// the bytes when each step is a kernel of its own.  The paper's rewriting (section 5: operators swapped across
// data movement until reads and writes of the same slice merge) removes both layout changes: the reduction runs
// over a strided dimension instead.  Here a workgroup owns a slab [C, 8 vectors of S]: lane (row group rg = tid / 8,
// column col = tid % 8) loads the 16-byte vectors of rows rg, rg + 32, ... at column col -- every load instruction
// of a wave reads 8 rows x 128 contiguous bytes, like the tile transposition -- and keeps them in registers (KC
// vectors per lane, so C <= 32 * KC).  The statistics of one position are spread over the 32 row groups: three
// lane exchanges inside a wave (lanes 8, 16, 32 apart hold the same column), then one LDS exchange between the
// four waves (one barrier each).  Mean first (as differences from a pivot row), then centred squares: no cancellation; RMS needs one
// exchange.  Every input
// element is read once and every output element written once; nothing is transposed.
#pragma once
#include "pf_device.hpp"

namespace pf {

template <int VEC>
PF_DEVICE void col_all_reduce(float (&v)[VEC], float* lds, uint32_t wave, uint32_t col, uint32_t lane) {
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
        v[j] += __shfl_xor(v[j], 8, 64);
        v[j] += __shfl_xor(v[j], 16, 64);
        v[j] += __shfl_xor(v[j], 32, 64);
    }
    if (lane < 8u) {  // (each exchange of a kernel has an LDS area of its own: no barrier in front)
#pragma unroll
        for (int j = 0; j < VEC; ++j) lds[(wave * 8u + col) * VEC + j] = v[j];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < VEC; ++j)
        v[j] = (lds[(0u * 8u + col) * VEC + j] + lds[(1u * 8u + col) * VEC + j]) + (lds[(2u * 8u + col) * VEC + j] + lds[(3u * 8u + col) * VEC + j]);
}

// The slab stays in registers in its storage form between the passes: the compiler may not keep the unpacked values
// of one pass alive for the next.
template <int KC>
PF_DEVICE void keep_packed(u32x4 (&raw)[KC]) {
#pragma unroll
    for (int k = 0; k < KC; ++k)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t w = raw[k][i];
            asm volatile("" : "+v"(w));
            raw[k][i] = w;
        }
}

// RAGGED: the extent after the normalised dimension is not a whole number of 16-byte vectors (7 x 7 or 14 x 14
// positions of 16-bit data): rows start at element alignment and the last vector of a row is partial.
template <int DT, int KC, bool RMS, bool RAGGED = false>
__global__ void __launch_bounds__(256) colnorm_kernel(const ColArgs a) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    __shared__ float lds[2][4 * 8 * VEC];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6, col = tid & 7u, rg = tid >> 3;
    const uint32_t o = blockIdx.x / a.tiles_per_outer, t = blockIdx.x - o * a.tiles_per_outer;
    const uint32_t sv = t * 8u + col;
    const bool col_ok = sv < a.s_vecs;
    const uint32_t cnt = RAGGED ? elems_below<VEC>(sv * VEC, a.s) : (uint32_t)VEC;  // elements of this lane's vector inside the row
    const uint64_t base = ((uint64_t)o * a.c) * a.s + (uint64_t)sv * VEC;  // element offset of row 0 at this column

    // Whole vectors are loaded without a branch: a lane whose row or column does not exist reads the last one that does
    // (the line a neighbour reads anyway) and never uses or stores the value.  Behind a guard every load would merge
    // with a fill value at the join, which the compiler resolves by waiting for it: the loads of a lane, all
    // independent, would then go to memory one round trip after the other.
    const uint64_t base_ld = RAGGED ? base : ((uint64_t)o * a.c) * a.s + (uint64_t)min(sv, a.s_vecs - 1u) * VEC;
    // (RAGGED: a lane's vector is whole, partial or absent for all its rows alike, so the three cases are told apart once,
    // outside the loop over the rows, and each runs its loads back to back)
    u32x4 raw[KC];
    if (!RAGGED || cnt == (uint32_t)VEC) {
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            const uint64_t elem = base_ld + (uint64_t)min(rg + 32u * (uint32_t)k, a.c - 1u) * a.s;
            raw[k] = RAGGED ? load_elems<DT>(a.x, elem, (uint32_t)VEC, 0u) : load_stream(a.x, elem * S::ESIZE);
        }
    } else if (cnt != 0u) {
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            // (what follows a partial vector is the next row of the tensor, unless this is its last row)
            const uint32_t c = min(rg + 32u * (uint32_t)k, a.c - 1u);
            raw[k] = load_elems<DT>(a.x, base + (uint64_t)c * a.s, cnt, 0u, c + 1u < a.c || blockIdx.x + a.tiles_per_outer < gridDim.x);
        }
    } else {
#pragma unroll
        for (int k = 0; k < KC; ++k) raw[k] = u32x4{0u, 0u, 0u, 0u};
    }
    // the parameters of the lane's rows, requested behind the slab (they are needed last; fetched where they are used,
    // every row's store would wait for a trip to the cache of its own)
    u32x4 gam_raw[KC], bet_raw[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        const uint64_t off = (uint64_t)min(rg + 32u * (uint32_t)k, a.c - 1u) * S::ESIZE;
        gam_raw[k] = S::splat(static_cast<const char*>(a.gamma) + off);
        // (no beta: gamma's element is read instead and dropped below -- no branch around a load, as above)
        bet_raw[k] = S::splat(static_cast<const char*>(a.beta ? a.beta : a.gamma) + off);
    }
    // mean = piv + mean[]: kept as a pivot (row 0 of the same position) plus the mean of the differences from it, so
    // that a large common offset of the values eats the digits neither of the sum nor of x - mean
    // (every lane fetches the pivot row itself: the 32 row groups of a column read the same 16 bytes, which the cache
    // serves, and no barrier is needed to share them)
    u32x4 piv_raw = u32x4{0u, 0u, 0u, 0u};
    if (!RMS) {
        if (!RAGGED) piv_raw = load_cached(a.x, base_ld * S::ESIZE);
        else if (col_ok) piv_raw = load_elems<DT>(a.x, base, cnt, 0u);
    }
    float piv[VEC], mean[VEC], acc[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) piv[j] = 0.0f, mean[j] = 0.0f, acc[j] = 0.0f;
    if (!RMS) {
        S::unpack(piv_raw, piv);
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            if (rg + 32u * (uint32_t)k < a.c) {
                float x[VEC];
                S::unpack(raw[k], x);
#pragma unroll
                for (int j = 0; j < VEC; ++j) mean[j] += x[j] - piv[j];
            }
        }
        col_all_reduce<VEC>(mean, lds[0], wave, col, lane);
#pragma unroll
        for (int j = 0; j < VEC; ++j) mean[j] *= a.inv_c;
        keep_packed<KC>(raw);
    }
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        const uint32_t c = rg + 32u * (uint32_t)k;
        if (c < a.c) {
            float x[VEC];
            S::unpack(raw[k], x);
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                const float d = (x[j] - piv[j]) - mean[j];
                acc[j] = fmaf(d, d, acc[j]);
            }
        }
    }
    col_all_reduce<VEC>(acc, lds[1], wave, col, lane);
    keep_packed<KC>(raw);
    float rstd[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) rstd[j] = pf_rsqrt<S::PRECISE>(fmaf(acc[j], a.inv_c, a.eps));
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        const uint32_t c = rg + 32u * (uint32_t)k;
        if (!(col_ok && c < a.c)) continue;
        float x[VEC], gam, bet;
        {
            float tmp[VEC];  // one element of the parameter vectors: the same for the whole row
            S::unpack(gam_raw[k], tmp);
            gam = tmp[0];
            S::unpack(bet_raw[k], tmp);
            bet = a.beta ? tmp[0] : 0.0f;
        }
        S::unpack(raw[k], x);
#pragma unroll
        for (int j = 0; j < VEC; ++j) x[j] = fmaf(((x[j] - piv[j]) - mean[j]) * rstd[j], gam, bet);
        if (RAGGED) store_elems<DT>(a.out, base + (uint64_t)c * a.s, cnt, S::pack(x));
        else store_stream(a.out, (base + (uint64_t)c * a.s) * S::ESIZE, S::pack(x));
    }
}

}  // namespace pf
