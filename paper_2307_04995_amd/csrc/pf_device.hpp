// Device-side building blocks shared by every kernel family (gfx950, wave64).
//
//   * 16-byte vector loads/stores and storage <-> fp32 conversion (the DRAM <-> register data-movement
//     steps of a chain; each lane moves 16 contiguous bytes, a wave 1 KB: the paper's rule that a parallel
//     unit reads n x lanes contiguous elements as n elements per lane at lane stride, section 7);
//   * wave-scope all-reduce built on DPP lane permutations (the "parallel unit" synchronisation scope of
//     section 5.1: the exchange stays in registers);
//   * the micro-op interpreter that runs the element-wise part of a chain on a register accumulator
//     (lane scope: read pattern == write pattern, nothing moves).
//
// All control flow inside the interpreter depends only on kernel arguments, so it is wave-uniform and
// costs scalar branches, not divergence.
#pragma once
#ifndef __HIPCC_RTC__  // the run-time compiler brings the HIP device declarations with it
#include <hip/hip_runtime.h>
#endif

#include "pf_common.h"

namespace pf {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

#define PF_DEVICE __device__ __forceinline__

// ---------------------------------------------------------------------------------------------
// storage types
// ---------------------------------------------------------------------------------------------
template <int DT>
struct Storage;

template <>
struct Storage<DT_F32> {
    static constexpr int VEC = 4;      // elements per 16-byte vector
    static constexpr int ESIZE = 4;
    static constexpr bool PRECISE = true;  // fp32 results are held to 1e-5: correctly rounded exp, division, square root (GELU: see pf_gelu_erf)
    static PF_DEVICE void unpack(u32x4 raw, float* out) {
        f32x4 v = __builtin_bit_cast(f32x4, raw);
        out[0] = v[0]; out[1] = v[1]; out[2] = v[2]; out[3] = v[3];
    }
    static PF_DEVICE u32x4 pack(const float* in) {
        f32x4 v = {in[0], in[1], in[2], in[3]};
        return __builtin_bit_cast(u32x4, v);
    }
    static PF_DEVICE u32x4 splat(const void* p) {
        uint32_t b = *reinterpret_cast<const uint32_t*>(p);
        return u32x4{b, b, b, b};
    }
};

template <>
struct Storage<DT_F16> {
    static constexpr int VEC = 8;
    static constexpr int ESIZE = 2;
    static constexpr bool PRECISE = false;
    static PF_DEVICE void unpack(u32x4 raw, float* out) {
        f16x8 h = __builtin_bit_cast(f16x8, raw);
        f32x8 v = __builtin_convertvector(h, f32x8);
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = v[i];
    }
    static PF_DEVICE u32x4 pack(const float* in) {
        f32x8 v = {in[0], in[1], in[2], in[3], in[4], in[5], in[6], in[7]};
        f16x8 h = __builtin_convertvector(v, f16x8);  // round to nearest even
        return __builtin_bit_cast(u32x4, h);
    }
    static PF_DEVICE u32x4 splat(const void* p) {
        uint32_t b = *reinterpret_cast<const uint16_t*>(p);
        b |= b << 16;
        return u32x4{b, b, b, b};
    }
};

template <>
struct Storage<DT_BF16> {
    static constexpr int VEC = 8;
    static constexpr int ESIZE = 2;
    static constexpr bool PRECISE = false;
    static PF_DEVICE void unpack(u32x4 raw, float* out) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __builtin_bit_cast(float, raw[i] << 16);
            out[2 * i + 1] = __builtin_bit_cast(float, raw[i] & 0xffff0000u);
        }
    }
    static PF_DEVICE u32x4 pack(const float* in) {
        f32x8 v = {in[0], in[1], in[2], in[3], in[4], in[5], in[6], in[7]};
        bf16x8 h = __builtin_convertvector(v, bf16x8);  // round to nearest even
        return __builtin_bit_cast(u32x4, h);
    }
    static PF_DEVICE u32x4 splat(const void* p) {
        uint32_t b = *reinterpret_cast<const uint16_t*>(p);
        b |= b << 16;
        return u32x4{b, b, b, b};
    }
};

// Streamed data is touched once: mark it non-temporal so it does not displace the broadcast operands.
PF_DEVICE u32x4 load_stream(const char* base, uint32_t byte_off) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + byte_off));
}
PF_DEVICE void store_stream(char* base, uint32_t byte_off, u32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(base + byte_off));
}
PF_DEVICE u32x4 load_stream(const void* base, uint64_t byte_off) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(static_cast<const char*>(base) + byte_off));
}
PF_DEVICE void store_stream(void* base, uint64_t byte_off, u32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(static_cast<char*>(base) + byte_off));
}
PF_DEVICE u32x4 load_cached(const void* base, uint64_t byte_off) {
    return *reinterpret_cast<const u32x4*>(static_cast<const char*>(base) + byte_off);
}

// Kernel arguments live in memory and the scalar loads that read them are issued where a value is first needed, so a
// kernel whose control flow depends on them pays one memory round trip per dependent step: several in a row before
// the first data load on a workgroup that is alone on its compute unit (a launch of a few hundred workgroups).
// Touching every 64-byte line of the first `BYTES` bytes of the argument block once, up front and in one batch,
// leaves those later loads to the scalar cache.  (Reads only.)
// ALSO: offset of one more argument to touch (the family's geometry, which follows the chain arguments).
template <uint32_t BYTES, uint32_t ALSO>
PF_DEVICE void warm_kernel_arguments() {
    typedef const __attribute__((address_space(4))) uint32_t* karg_ptr;
    karg_ptr k = (karg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
    uint32_t acc = k[ALSO / 4u];
#pragma unroll
    for (uint32_t off = 0; off < BYTES; off += 64u) acc |= k[off / 4u];
    asm volatile("" ::"s"(acc));
}
// for kernels whose arguments are (ChainArgs, geometry): a specialised kernel never reads the two programs
template <class Spec>
PF_DEVICE void warm_chain_arguments() {
    warm_kernel_arguments<Spec::kStatic ? (uint32_t)__builtin_offsetof(ChainArgs, pro) : (uint32_t)sizeof(ChainArgs), (uint32_t)sizeof(ChainArgs)>();
}

// Element-granular access, for rows whose byte length is not a multiple of 16: their vectors are not
// 16-byte aligned and the last one is partial.  The first `count` elements of the vector are touched; the
// others read as the matching half of `fill` and are not stored.
//
// Whole vectors of such a row move as one 16-byte access at element alignment (the device runs with
// unaligned global access enabled, and the compiler emits a single dwordx4 access for this pointer type); only
// the partial vector at the end of a row goes element by element, so nothing outside the row is touched.
typedef u32x4 u32x4_elem_aligned __attribute__((aligned(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x2 u32x2_elem_aligned __attribute__((aligned(2)));
typedef uint32_t u32_elem_aligned __attribute__((aligned(2)));

// `room`: the VEC elements from `elem` on all lie inside the tensor (what follows a partial vector is the start of the
// tensor's next row, say): the partial vector is then read as one whole vector and the slots past `count` replaced by
// the fill value -- one load instead of `count`.
// NT: streamed data (touched once) is loaded with the non-temporal hint; small operands that every row reads again are not.
template <int DT, bool NT = true>
PF_DEVICE u32x4 load_elems(const void* base, uint64_t elem, uint32_t count, uint32_t fill, bool room = false) {
    u32x4 r = {fill, fill, fill, fill};
    if (count == 0u) return r;
    // (whole vectors and partial ones with room behind them take the same load instruction: the lanes of a wave that
    // hold a row's whole vectors and the lane that holds its tail do not part ways)
    if (count == (uint32_t)Storage<DT>::VEC || room) {
        const u32x4_elem_aligned* vp = reinterpret_cast<const u32x4_elem_aligned*>(static_cast<const char*>(base) + elem * Storage<DT>::ESIZE);
        const u32x4 got = NT ? __builtin_nontemporal_load(vp) : *vp;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t w = got[j];
            if (DT == DT_F32) {
                r[j] = (uint32_t)j < count ? w : fill;
            } else {
                const uint32_t lo = (uint32_t)(2 * j) < count ? (w & 0xffffu) : (fill & 0xffffu);
                const uint32_t hi = (uint32_t)(2 * j + 1) < count ? (w & 0xffff0000u) : (fill & 0xffff0000u);
                r[j] = lo | hi;
            }
        }
        return r;
    }
    // A partial vector: every slot reads an element that exists (the last one, for the slots past the end) and the
    // fill value is selected afterwards.  No branch per element: behind one, each load would wait for the one before.
    const uint32_t last = count - 1u;
    if (DT == DT_F32) {
        const uint32_t* p = static_cast<const uint32_t*>(base) + elem;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t got = NT ? __builtin_nontemporal_load(p + min((uint32_t)e, last)) : p[min((uint32_t)e, last)];
            r[e] = (uint32_t)e < count ? got : fill;
        }
    } else {
        const uint16_t* p = static_cast<const uint16_t*>(base) + elem;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t got_lo = NT ? __builtin_nontemporal_load(p + min((uint32_t)(2 * j), last)) : p[min((uint32_t)(2 * j), last)];
            const uint32_t got_hi = NT ? __builtin_nontemporal_load(p + min((uint32_t)(2 * j + 1), last)) : p[min((uint32_t)(2 * j + 1), last)];
            const uint32_t lo = (uint32_t)(2 * j) < count ? got_lo : (fill & 0xffffu);
            const uint32_t hi = (uint32_t)(2 * j + 1) < count ? got_hi : (fill >> 16);
            r[j] = lo | (hi << 16);
        }
    }
    return r;
}
template <int DT>
PF_DEVICE void store_elems(void* base, uint64_t elem, uint32_t count, u32x4 v) {
    if (count == (uint32_t)Storage<DT>::VEC) {
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4_elem_aligned*>(static_cast<char*>(base) + elem * Storage<DT>::ESIZE));
        return;
    }
    // A partial vector goes out in pieces of 8, 4 and 2 bytes (the binary digits of its length), at element alignment:
    // at most three stores, not one per element.
    const uint32_t v0 = v[0], v1 = v[1], v2 = v[2], v3 = v[3];
    if (DT == DT_F32) {
        uint32_t* p = static_cast<uint32_t*>(base) + elem;
        if (count & 2u) __builtin_nontemporal_store(u32x2{v0, v1}, reinterpret_cast<u32x2_elem_aligned*>(p));
        if (count & 1u) __builtin_nontemporal_store((count & 2u) ? v2 : v0, p + (count & 2u));
    } else {
        uint16_t* p = static_cast<uint16_t*>(base) + elem;
        if (count & 4u) __builtin_nontemporal_store(u32x2{v0, v1}, reinterpret_cast<u32x2_elem_aligned*>(p));
        const uint32_t mid = (count & 4u) ? v2 : v0;  // the dword behind the 8-byte piece, if there was one
        if (count & 2u) __builtin_nontemporal_store(mid, reinterpret_cast<u32_elem_aligned*>(p + (count & 4u)));
        const uint32_t last = (count & 4u) ? ((count & 2u) ? v3 : v2) : ((count & 2u) ? v1 : v0);
        if (count & 1u) __builtin_nontemporal_store((uint16_t)(last & 0xffffu), p + (count & 6u));
    }
}
// how many elements of the vector that starts at `col` lie below `limit` (0 .. VEC)
template <int VEC>
PF_DEVICE uint32_t elems_below(uint32_t col, uint32_t limit) {
    return col < limit ? (limit - col < (uint32_t)VEC ? limit - col : (uint32_t)VEC) : 0u;
}

PF_DEVICE uint32_t fast_div(uint32_t n, const FastDiv& f) {
    const uint32_t t = __umulhi(f.m, n);
    return (t + ((n - t) >> f.s1)) >> f.s2;
}

// ---------------------------------------------------------------------------------------------
// wave-scope all-reduce (64 lanes) on DPP permutations; every lane ends with the same bits
// ---------------------------------------------------------------------------------------------
template <int CTRL>
PF_DEVICE float dpp_move(float v) {
    int r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true);
    return __builtin_bit_cast(float, r);
}
PF_DEVICE float read_lane(float v, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// DPP move where the lanes of rows not selected by ROW_MASK receive `old`
template <int CTRL, int ROW_MASK>
PF_DEVICE int dpp_move_rows(int old, int v) {
    return __builtin_amdgcn_update_dpp(old, v, CTRL, ROW_MASK, 0xf, false);
}

// Order-preserving map between fp32 bit patterns and signed integers (its own inverse).  Reducing the
// keys with integer max avoids the NaN-quieting moves a floating-point max needs after every lane
// permutation; a (positive) NaN maps above +inf, so it wins the reduction and poisons the row.
PF_DEVICE int32_t float_to_key(float f) {
    const int32_t b = __builtin_bit_cast(int32_t, f);
    return b ^ ((b >> 31) & 0x7fffffff);
}
PF_DEVICE float key_to_float(int32_t k) { return __builtin_bit_cast(float, k ^ ((k >> 31) & 0x7fffffff)); }

struct OpSum {
    static PF_DEVICE float identity() { return 0.0f; }
    static PF_DEVICE float apply(float a, float b) { return a + b; }
    static PF_DEVICE float wave(float v) {
        v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
        v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
        v += dpp_move<0x141>(v);  // row_half_mirror
        v += dpp_move<0x140>(v);  // row_mirror: every lane holds its 16-lane row's sum
        v += __builtin_bit_cast(float, dpp_move_rows<0x142, 0xa>(0, __builtin_bit_cast(int, v)));  // row_bcast15 -> rows 1, 3
        v += __builtin_bit_cast(float, dpp_move_rows<0x143, 0xc>(0, __builtin_bit_cast(int, v)));  // row_bcast31 -> rows 2, 3
        return read_lane(v, 63);
    }
};
struct OpMax {
    static PF_DEVICE float identity() { return -__builtin_inff(); }
    static PF_DEVICE float apply(float a, float b) { return fmaxf(a, b); }
    static PF_DEVICE float wave(float f) {
        int32_t v = float_to_key(f);
        constexpr int32_t lowest = (int32_t)0x80000000;
        v = max(v, __builtin_amdgcn_update_dpp(lowest, v, 0xB1, 0xf, 0xf, true));
        v = max(v, __builtin_amdgcn_update_dpp(lowest, v, 0x4E, 0xf, 0xf, true));
        v = max(v, __builtin_amdgcn_update_dpp(lowest, v, 0x141, 0xf, 0xf, true));
        v = max(v, __builtin_amdgcn_update_dpp(lowest, v, 0x140, 0xf, 0xf, true));
        v = max(v, dpp_move_rows<0x142, 0xa>(lowest, v));
        v = max(v, dpp_move_rows<0x143, 0xc>(lowest, v));
        return key_to_float(__builtin_amdgcn_readlane(v, 63));
    }
};

template <class Op>
PF_DEVICE float wave_allreduce(float v) {
    return Op::wave(v);
}

// all-reduce over groups of 2^LOG2 adjacent lanes (LOG2 <= 4), result in every lane of the group
template <class Op, int LOG2>
PF_DEVICE float subrow_allreduce(float v) {
    if (LOG2 >= 1) v = Op::apply(v, dpp_move<0xB1>(v));
    if (LOG2 >= 2) v = Op::apply(v, dpp_move<0x4E>(v));
    if (LOG2 >= 3) v = Op::apply(v, dpp_move<0x141>(v));
    if (LOG2 >= 4) v = Op::apply(v, dpp_move<0x140>(v));
    return v;
}

// all-reduce over aligned segments of 2^LOG2 lanes (LOG2 = 6: the whole wave), result in every lane of the segment
template <class Op, int LOG2>
PF_DEVICE float seg_allreduce(float v) {
    if (LOG2 >= 6) return Op::wave(v);
    if (LOG2 == 5) {
        v = subrow_allreduce<Op, 4>(v);
        return Op::apply(v, __shfl_xor(v, 16, 64));
    }
    return subrow_allreduce<Op, LOG2>(v);
}

// ---------------------------------------------------------------------------------------------
// mean / variance statistics as (count, mean, M2) triples
// ---------------------------------------------------------------------------------------------
struct Stat {
    float n, mean, m2;
};

// parallel-variance update; counts are small integers, so the approximate reciprocal is exact enough
PF_DEVICE Stat stat_merge(Stat a, Stat b) {
    const float n = a.n + b.n;
    const float inv = n > 0.0f ? __builtin_amdgcn_rcpf(n) : 0.0f;
    const float delta = b.mean - a.mean;
    Stat r;
    r.n = n;
    // (merging with an empty side must return the other side's mean bit for bit: the reciprocal is approximate, and a
    // group of one element has to come out with zero deviation exactly)
    r.mean = a.n == 0.0f ? b.mean : (b.n == 0.0f ? a.mean : a.mean + delta * (b.n * inv));
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

// A lane's running statistics.  Each vector is reduced on its own (mean of its elements, then squared deviations
// from that mean: everything is in registers, so the two passes cost nothing extra) and merged into the running
// triple with the parallel-variance update.  No step subtracts large nearly-equal sums, so a spread that is
// tiny against the values' offset (a channel that is almost constant) keeps its relative accuracy.
struct LaneAcc {
    float n = 0.0f, mean = 0.0f, m2 = 0.0f;
    template <int VEC>
    PF_DEVICE void add_vector(const float* x) {
        float sv = 0.0f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) sv += x[e];
        const float mv = sv * (1.0f / (float)VEC);
        float m2v = 0.0f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float d = x[e] - mv;
            m2v = __builtin_fmaf(d, d, m2v);
        }
        const float nn = n + (float)VEC;
        const float inv = __builtin_amdgcn_rcpf(nn);
        const float delta = mv - mean;
        mean = __builtin_fmaf(delta, (float)VEC * inv, mean);
        m2 += m2v + delta * delta * (n * (float)VEC * inv);
        n = nn;
    }
    PF_DEVICE Stat finish() const { return Stat{n, mean, m2}; }
};

// ---------------------------------------------------------------------------------------------
// element-wise math
// ---------------------------------------------------------------------------------------------
constexpr float kLog2e = 1.4426950408889634f;

template <bool PRECISE>
PF_DEVICE float pf_exp(float x) {
    if (PRECISE) return expf(x);
    return __builtin_amdgcn_exp2f(x * kLog2e);
}
template <bool PRECISE>
PF_DEVICE float pf_rcp(float x) {
    if (PRECISE) return 1.0f / x;
    return __builtin_amdgcn_rcpf(x);
}
template <bool PRECISE>
PF_DEVICE float pf_div(float a, float b) {
    if (PRECISE) return a / b;
    return a * __builtin_amdgcn_rcpf(b);
}
template <bool PRECISE>
PF_DEVICE float pf_rsqrt(float x) {
    if (PRECISE) return 1.0f / sqrtf(x);
    return __builtin_amdgcn_rsqf(x);
}
template <bool PRECISE>
PF_DEVICE float pf_sigmoid(float x) {
    return pf_rcp<PRECISE>(1.0f + pf_exp<PRECISE>(-x));
}
template <bool PRECISE>
PF_DEVICE float pf_tanh(float x) {
    if (PRECISE) return tanhf(x);
    return 2.0f * pf_sigmoid<false>(2.0f * x) - 1.0f;
}
// GELU(x) = x * Phi(x), Phi(x) = (1 + erf(x / sqrt 2)) / 2.  The tail Q = erfc(|x| / sqrt 2) / 2 comes from the rational
// approximation 7.1.26 of Abramowitz & Stegun's handbook, erfc(z) = (a1 t + ... + a5 t^5) exp(-z^2) with
// t = 1 / (1 + p z), whose absolute error is below 1.5e-7; Phi is Q left of zero and 1 - Q right of it, so the left
// tail has no cancellation.  The result is within 3e-7 * |x| of the exact value (the library erff costs six times the
// instructions and made the fp32 chain arithmetic-bound).
PF_DEVICE float pf_gelu_erf(float x) {
    const float z = __builtin_fabsf(x) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f, z, 1.0f));
    float poly = 1.061405429f;
    poly = __builtin_fmaf(poly, t, -1.453152027f);
    poly = __builtin_fmaf(poly, t, 1.421413741f);
    poly = __builtin_fmaf(poly, t, -0.284496736f);
    poly = __builtin_fmaf(poly, t, 0.254829592f);
    const float q = 0.5f * poly * t * __builtin_amdgcn_exp2f(-z * z * kLog2e);
    return x * (x < 0.0f ? q : 1.0f - q);
}
PF_DEVICE float pf_max_nan(float a, float b) {
    float r = fmaxf(a, b);
    return (a != a || b != b) ? __builtin_nanf("") : r;
}
PF_DEVICE float pf_min_nan(float a, float b) {
    float r = fminf(a, b);
    return (a != a || b != b) ? __builtin_nanf("") : r;
}

// ---------------------------------------------------------------------------------------------
// chain specifications: how a kernel learns what the chain looks like
// ---------------------------------------------------------------------------------------------
// A kernel is instantiated once per "spec".  The generic spec reads operand counts and the micro-programs
// from the kernel arguments at run time (wave-uniform scalar loads and branches).  A static spec fixes
// the structure (operand counts, step codes, operand kinds and slots) at compile time, so the interpreter
// loop unrolls and the switches fold away; immediates (scale factors, eps, mask extent) stay run-time
// values in both cases.  This mirrors the paper's GIR templates (section 6): a graph structure chosen
// ahead of time, with parameters filled in per use.

struct UopC {
    uint8_t code, kind, slot;
};

// run-time program list
struct DynList {
    static constexpr bool kDynamic = true;
    static constexpr int n = 0;
    static constexpr UopC at(int) { return UopC{0, 0, 0}; }
};

template <class L>
struct ProgView {
    const Program& p;
    PF_DEVICE int n() const { return L::kDynamic ? p.n : L::n; }
    PF_DEVICE int code(int i) const { return L::kDynamic ? p.u[i].code : L::at(i).code; }
    PF_DEVICE int kind(int i) const { return L::kDynamic ? p.u[i].kind : L::at(i).kind; }
    PF_DEVICE int slot(int i) const { return L::kDynamic ? p.u[i].slot : L::at(i).slot; }
    PF_DEVICE float imm(int i) const { return p.u[i].imm; }
    PF_DEVICE int32_t ival(int i) const { return p.u[i].ival; }
};

struct GenericSpec {
    static constexpr bool kStatic = false;
    static constexpr bool kBcast = true;  // general broadcasting of operands is a run-time property here
    static constexpr int kVecMode = 3;    // ... and so is a broadcast operand with a single element
    static constexpr int NF = 3, NV = 4, NT = PF_DEV_MAX_TMP;
    using Pro = DynList;
    using Epi = DynList;
    static PF_DEVICE int n_full(const ChainArgs& a) { return a.n_full; }
    static PF_DEVICE int n_vec(const ChainArgs& a) { return a.n_vec; }
    static PF_DEVICE int core(const ChainArgs& a) { return a.core; }
    static PF_DEVICE int gamma(const ChainArgs& a) { return a.core_vec[0]; }
    static PF_DEVICE int beta(const ChainArgs& a) { return a.core_vec[1]; }
};

// FLAGS_: bit 0 = some operand broadcasts the general way (extents of 1 anywhere); bit 1 = some broadcast operand has a
// single element.  Kernels built without a bit carry none of that case's code: the one-element case in particular
// costs more than its branch, because the compiler issues its 2-byte load next to the 16-byte one and waits for both
// before it goes on, which turns the operand loads of a kernel into one memory round trip after the other.
template <int NF_, int NV_, int NT_, int CORE_, int GAMMA_, int BETA_, class ProL, class EpiL, int FLAGS_ = 0>
struct StaticSpec {
    static constexpr bool kStatic = true;
    static constexpr bool kBcast = (FLAGS_ & 1) != 0;
    static constexpr int kVecMode = FLAGS_ & 3;
    static constexpr int NF = NF_, NV = NV_, NT = NT_;
    using Pro = ProL;
    using Epi = EpiL;
    static PF_DEVICE int n_full(const ChainArgs&) { return NF_; }
    static PF_DEVICE int n_vec(const ChainArgs&) { return NV_; }
    static PF_DEVICE int core(const ChainArgs&) { return CORE_; }
    static PF_DEVICE int gamma(const ChainArgs&) { return GAMMA_; }
    static PF_DEVICE int beta(const ChainArgs&) { return BETA_; }
};

constexpr int at_least_1(int n) { return n < 1 ? 1 : n; }

// Facts about a static step list that kernels can use at compile time.
// Which slots of operand kind `kind` the list reads (bit per slot).
template <class L>
constexpr uint32_t list_operand_mask(int kind) {
    uint32_t m = 0;
    for (int i = 0; i < L::n; ++i)
        if (L::at(i).kind == kind) m |= 1u << L::at(i).slot;
    return m;
}
// Whether the list only loads one full operand and applies steps whose results are again exactly representable
// in the storage type (so they can be kept packed without changing any later result).
template <class L>
constexpr bool list_keeps_storage_precision() {
    if (L::kDynamic || L::n < 1) return false;
    for (int i = 0; i < L::n; ++i) {
        const UopC u = L::at(i);
        const bool load = u.code == U_MOV && u.kind == K_FULL && i == 0;
        const bool exact = (u.code == U_RELU || u.code == U_NEG) && i > 0;
        if (!load && !exact) return false;
    }
    return true;
}

// ---------------------------------------------------------------------------------------------
// per-lane state: K 16-byte vectors of every operand, an fp32 accumulator, temporaries
// ---------------------------------------------------------------------------------------------
template <int DT, int K, class Spec>
struct LaneState {
    static constexpr int VEC = Storage<DT>::VEC;
    static constexpr int E = K * VEC;
    u32x4 fraw[at_least_1(Spec::NF)][K];
    u32x4 vraw[at_least_1(Spec::NV)][K];
    float acc[E];
    float tmp[at_least_1(Spec::NT)][E];
    uint32_t row[K];  // row (index over all but the innermost dim) of vector k
    uint32_t col[K];  // column of the first element of vector k
    float rowv[PF_DEV_MAX_ROWV][K];  // per-row values produced by U_RED_* steps (row programs), one per vector: a lane
                                     // may hold vectors of several rows
};

// Where a broadcast operand's 16-byte vector for position (row, col) starts, in elements.
// BC = false: the kernel was built for chains without general broadcasting (the check and its code drop out).
template <bool BC = true>
PF_DEVICE uint32_t vec_offset(const VecArg& va, uint32_t row, uint32_t col, uint32_t n_inner) {
    if (BC && va.n_terms != 0u) {
        uint32_t r = 0;
#pragma unroll
        for (int k = 0; k < PF_DEV_MAX_BCAST_TERMS; ++k)
            if ((uint32_t)k < va.n_terms) {
                const BcastTerm t = va.terms[k];
                const uint32_t q = fast_div(row, t.div);
                r += (q - fast_div(q, t.mod) * t.mod.d) * t.stride;
            }
        return va.col_bcast ? r : r * n_inner + col;
    }
    if (va.numel >= n_inner) {
        const uint32_t r = (va.period_rows == 1) ? 0u : row % va.period_rows;
        return r * n_inner + col;
    }
    return col % va.numel;
}

// VM: which of the cases above the kernel was built for (bit 0: general broadcasting, bit 1: one-element operands)
template <int DT, int VM = 3>
PF_DEVICE u32x4 load_vec_operand(const VecArg& va, uint32_t row, uint32_t col, uint32_t n_inner) {
    constexpr bool BC = (VM & 1) != 0;
    if ((VM & 2) && va.numel == 1) return Storage<DT>::splat(va.ptr);
    const uint32_t off = vec_offset<BC>(va, row, col, n_inner);
    if (BC && va.n_terms != 0u && va.col_bcast) return Storage<DT>::splat(static_cast<const char*>(va.ptr) + (uint64_t)off * Storage<DT>::ESIZE);
    return load_cached(va.ptr, (uint64_t)off * Storage<DT>::ESIZE);
}

// The same for a position whose vector may be unaligned or partial: gathered element by element.
template <int DT, int VM = 3>
PF_DEVICE u32x4 load_vec_operand_elems(const VecArg& va, uint32_t row, uint32_t col, uint32_t n_inner, uint32_t count) {
    using S = Storage<DT>;
    constexpr bool BC = (VM & 1) != 0;
    if ((VM & 2) && va.numel == 1) return S::splat(va.ptr);
    if (BC && va.n_terms != 0u && va.col_bcast) return S::splat(static_cast<const char*>(va.ptr) + (uint64_t)vec_offset<BC>(va, row, col, n_inner) * S::ESIZE);
    u32x4 r = {0u, 0u, 0u, 0u};
    if (count == 0u) return r;
    // An operand whose elements for this vector lie side by side (a vector of the row's length, or one such vector per
    // row): one 16-byte load at element alignment, as for the rows themselves, with the partial vector read whole where
    // the operand continues behind it.
    if (!(BC && va.n_terms != 0u) && va.numel >= n_inner) {
        const uint32_t off = vec_offset<false>(va, row, col, n_inner);
        return load_elems<DT, false>(va.ptr, off, count, 0u, off + (uint32_t)S::VEC <= va.numel);
    }
    // (slots past the end read the last element that exists and are zeroed: no branch per element, see load_elems)
    const uint32_t last = count - 1u;
    if (DT == DT_F32) {
        const uint32_t* p = static_cast<const uint32_t*>(va.ptr);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t got = p[vec_offset<BC>(va, row, col + min((uint32_t)e, last), n_inner)];
            r[e] = (uint32_t)e < count ? got : 0u;
        }
    } else {
        const uint16_t* p = static_cast<const uint16_t*>(va.ptr);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t got_lo = p[vec_offset<BC>(va, row, col + min((uint32_t)(2 * j), last), n_inner)];
            const uint32_t got_hi = p[vec_offset<BC>(va, row, col + min((uint32_t)(2 * j + 1), last), n_inner)];
            const uint32_t lo = (uint32_t)(2 * j) < count ? got_lo : 0u;
            const uint32_t hi = (uint32_t)(2 * j + 1) < count ? got_hi : 0u;
            r[j] = lo | (hi << 16);
        }
    }
    return r;
}

template <int DT, int K>
PF_DEVICE void unpack_slot(const u32x4 (&raw)[K], float* out) {
#pragma unroll
    for (int k = 0; k < K; ++k) Storage<DT>::unpack(raw[k], out + k * Storage<DT>::VEC);
}

// Fetch an operand by slot; the unrolled compare chain keeps every register index static.
template <int DT, int K, class Spec>
PF_DEVICE void fetch_full(const LaneState<DT, K, Spec>& s, int slot, float* b) {
#pragma unroll
    for (int f = 0; f < Spec::NF; ++f)
        if (slot == f) unpack_slot<DT, K>(s.fraw[f], b);
}
template <int DT, int K, class Spec>
PF_DEVICE void fetch_vec(const LaneState<DT, K, Spec>& s, int slot, float* b) {
#pragma unroll
    for (int v = 0; v < Spec::NV; ++v)
        if (slot == v) unpack_slot<DT, K>(s.vraw[v], b);
}

// the KC vectors of a broadcast operand that start at vector k0
template <int DT, int K, int KC, class Spec>
PF_DEVICE void fetch_vec_part(const LaneState<DT, K, Spec>& s, int slot, int k0, float* b) {
#pragma unroll
    for (int v = 0; v < Spec::NV; ++v)
        if (slot == v) {
#pragma unroll
            for (int c = 0; c < KC; ++c) Storage<DT>::unpack(s.vraw[v][k0 + c], b + c * Storage<DT>::VEC);
        }
}

// Secondary-output hook: the families that support U_STORE pass a functor; others pass NoStore.
struct NoStore {
    template <int DT, int K, class Spec>
    PF_DEVICE void operator()(int, const LaneState<DT, K, Spec>&) const {}
};

// Row-reduction hook (U_RED_*): only the row kernel's hook type overloads this; everywhere else the planner
// never emits such a step.
template <class Hook, int DT, int K, class Spec>
PF_DEVICE void hook_reduce(const Hook&, int, int, LaneState<DT, K, Spec>&) {}

template <int DT, int K, class Spec>
PF_DEVICE void apply_uop(int code, int slot, int32_t ival, LaneState<DT, K, Spec>& s, const float* b) {
    constexpr int E = LaneState<DT, K, Spec>::E;
    constexpr int VEC = LaneState<DT, K, Spec>::VEC;
    constexpr bool PR = Storage<DT>::PRECISE;
    switch (code) {
        case U_MOV:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = b[e];
            break;
        case U_ADD:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = s.acc[e] + b[e];
            break;
        case U_SUB:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = s.acc[e] - b[e];
            break;
        case U_RSUB:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = b[e] - s.acc[e];
            break;
        case U_MUL:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = s.acc[e] * b[e];
            break;
        case U_DIV:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = pf_div<PR>(s.acc[e], b[e]);
            break;
        case U_RDIV:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = pf_div<PR>(b[e], s.acc[e]);
            break;
        case U_MAX:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = pf_max_nan(s.acc[e], b[e]);
            break;
        case U_MIN:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = pf_min_nan(s.acc[e], b[e]);
            break;
        case U_NEG:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = -s.acc[e];
            break;
        case U_RELU:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = pf_max_nan(s.acc[e], 0.0f);
            break;
        case U_SIGMOID:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = pf_sigmoid<PR>(s.acc[e]);
            break;
        case U_SILU:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = s.acc[e] * pf_sigmoid<PR>(s.acc[e]);
            break;
        case U_GELU_ERF:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = pf_gelu_erf(s.acc[e]);
            break;
        case U_TANH:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = pf_tanh<PR>(s.acc[e]);
            break;
        case U_EXP:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = pf_exp<PR>(s.acc[e]);
            break;
        case U_RSQRT:
#pragma unroll
            for (int e = 0; e < E; ++e) s.acc[e] = pf_rsqrt<PR>(s.acc[e]);
            break;
        case U_MASK_CAUSAL: {
            const uint32_t si = (uint32_t)ival;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const int32_t last = (int32_t)(s.row[k] % si) - (int32_t)s.col[k];  // last unmasked element of the vector
#pragma unroll
                for (int e = 0; e < VEC; ++e) s.acc[k * VEC + e] = (e > last) ? -__builtin_inff() : s.acc[k * VEC + e];
            }
            break;
        }
        case U_SAVE:
#pragma unroll
            for (int t = 0; t < Spec::NT; ++t)
                if (slot == t) {
#pragma unroll
                    for (int e = 0; e < E; ++e) s.tmp[t][e] = s.acc[e];
                }
            break;
        default: break;
    }
}

// One step of the interpreter.
template <int DT, int K, class Spec, class L, class StoreFn>
PF_DEVICE void run_step(const ProgView<L>& pv, int i, LaneState<DT, K, Spec>& s, const StoreFn& store_fn) {
    constexpr int E = LaneState<DT, K, Spec>::E;
    constexpr int VEC = LaneState<DT, K, Spec>::VEC;
    const int kind = pv.kind(i), code = pv.code(i), slot = pv.slot(i);
    float b[E];
    switch (kind) {
        case K_IMM: {
            const float imm = pv.imm(i);
#pragma unroll
            for (int e = 0; e < E; ++e) b[e] = imm;
            break;
        }
        case K_FULL: fetch_full<DT, K, Spec>(s, slot, b); break;
        case K_VEC: fetch_vec<DT, K, Spec>(s, slot, b); break;
        case K_TMP:
#pragma unroll
            for (int t = 0; t < Spec::NT; ++t)
                if (slot == t) {
#pragma unroll
                    for (int e = 0; e < E; ++e) b[e] = s.tmp[t][e];
                }
            break;
        case K_ROW:
#pragma unroll
            for (int t = 0; t < PF_DEV_MAX_ROWV; ++t)
                if (slot == t) {
#pragma unroll
                    for (int e = 0; e < E; ++e) b[e] = s.rowv[t][e / VEC];
                }
            break;
        default:
#pragma unroll
            for (int e = 0; e < E; ++e) b[e] = 0.0f;
            break;
    }
    if (code == U_STORE) store_fn(slot, s);
    else if (code == U_RED_SUM || code == U_RED_MAX || code == U_RED_MEAN) hook_reduce(store_fn, code, slot, s);
    else apply_uop<DT, K, Spec>(code, slot, pv.ival(i), s, b);
}

// The micro-op interpreter.  With a static list the loop bound and every code / kind / slot are compile
// time constants: the loop unrolls and only the selected arithmetic remains.
template <int DT, int K, class Spec, class L, class StoreFn>
PF_DEVICE void run_program(const ProgView<L> pv, LaneState<DT, K, Spec>& s, const StoreFn& store_fn) {
    if (L::kDynamic) {
        const int n = pv.n();
        for (int i = 0; i < n; ++i) run_step<DT, K, Spec, L, StoreFn>(pv, i, s, store_fn);
    } else {
#pragma unroll
        for (int i = 0; i < L::n; ++i) run_step<DT, K, Spec, L, StoreFn>(pv, i, s, store_fn);
    }
}

}  // namespace pf
