// Transpose family: prologue -> permutation of dimensions -> epilogue in one kernel.
//
// A layout change is a synchronisation step whose read and write slice patterns differ (paper section 4,
// synchronisation gOperators).  Element-wise steps commute with it (section 5.1, gOperator swapping), so
// the prologue runs on values addressed in the input layout, the epilogue on values addressed in the
// output layout, and the permuted tensor itself never exists in HBM twice.
//
// Variants for permutations that keep the innermost dimension (every 16-byte vector moves intact):
//   T_ROWS      each lane re-addresses its vector: one side of the transfer is contiguous per wave, the
//               other side is contiguous in runs of the innermost extent;
//   T_LDS_ROWS  a workgroup stages a [tile_a x tile_b] block of innermost rows in LDS between a read phase
//               and a write phase, so both sides are walked in long contiguous runs.
// Variant for permutations that change the innermost dimension:
//   T_TILE      a wave owns a square tile; each lane transposes a VEC x VEC block of elements in registers.
#pragma once
#include "pf_row_kernels.hpp"

namespace pf {

struct NoStoreT {
    template <int DT, int K, class Spec>
    PF_DEVICE void operator()(int, const LaneState<DT, K, Spec>&) const {}
};

// Split a vector index of the iteration space into element offsets on both sides.
PF_DEVICE void perm_offsets(const PermGeom& g, uint32_t v, uint32_t vec, uint32_t* in_off, uint32_t* out_off) {
    uint32_t io = 0, oo = 0, rem = v;
#pragma unroll
    for (int q = PF_DEV_MAX_RANK - 1; q >= 0; --q) {
        if (q < g.rank) {
            const uint32_t quo = (q == 0) ? 0u : fast_div(rem, g.div[q]);
            const uint32_t idx = (q == 0) ? rem : rem - quo * g.extent[q];
            const uint32_t scale = (q == g.rank - 1) ? vec : 1u;
            io += idx * scale * g.in_stride[q];
            oo += idx * scale * g.out_stride[q];
            rem = quo;
        }
    }
    *in_off = io;
    *out_off = oo;
}

// Geometry as a compile-time fact.  Splitting an index over up to six dimensions whose extents are kernel arguments
// costs a lane a dozen 32-bit multiplications per vector, more instructions than the rest of a permutation kernel
// together.  For large tensors the planner therefore hands the run-time compiler a type that holds the geometry as
// constants (same members as below, kConst = true, plus what it knows about the broadcast operands): divisions by
// powers of two become shifts, the others multiplications by constants, and nothing is loaded or branched on.
// RuntimePermGeom stands for "read the PermGeom argument".
struct RuntimePermGeom {
    static constexpr bool kConst = false;
};

template <class CG>
PF_DEVICE void perm_offsets_t(const PermGeom& g, uint32_t v, uint32_t vec, uint32_t* in_off, uint32_t* out_off) {
    if constexpr (!CG::kConst) {
        perm_offsets(g, v, vec, in_off, out_off);
    } else {
        uint32_t io = 0, oo = 0, rem = v;
#pragma unroll
        for (int q = CG::rank - 1; q >= 0; --q) {
            const uint32_t quo = (q == 0) ? 0u : rem / CG::extent[q];
            const uint32_t idx = (q == 0) ? rem : rem - quo * CG::extent[q];
            const uint32_t scale = (q == CG::rank - 1) ? vec : 1u;
            io += idx * (scale * CG::in_stride[q]);
            oo += idx * (scale * CG::out_stride[q]);
            rem = quo;
        }
        *in_off = io;
        *out_off = oo;
    }
}

// SIDES: 3 = operands of both programs, 1 = prologue operands only (input layout), 2 = epilogue operands only
// RAGGED: vectors may start at any element and hold fewer than VEC elements (cnt[k] of them; 0 = none)
template <int DT, int K, class Spec, int SIDES = 3, bool RAGGED = false, class CG = RuntimePermGeom>
PF_DEVICE void perm_load_operands(const ChainArgs& a, const PermGeom& g, LaneState<DT, K, Spec>& s, const uint32_t* in_off,
                                  const uint32_t* out_off, const bool* valid, const uint32_t* cnt = nullptr) {
    using S = Storage<DT>;
    if constexpr (CG::kConst && !RAGGED && (Spec::kVecMode & 1) == 0) {
        // every mask, extent and operand length is a constant: plain address arithmetic, no division at run time
#pragma unroll
        for (int f = 0; f < Spec::NF; ++f) {
            const bool epi = (CG::epi_full_mask >> f) & 1u;
            if ((epi && !(SIDES & 2)) || (!epi && !(SIDES & 1))) continue;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                s.fraw[f][k] = u32x4{0u, 0u, 0u, 0u};
                if (valid[k]) s.fraw[f][k] = load_stream(a.full[f], (uint64_t)(epi ? out_off[k] : in_off[k]) * S::ESIZE);
            }
        }
#pragma unroll
        for (int v = 0; v < Spec::NV; ++v) {
            const bool epi = (CG::epi_vec_mask >> v) & 1u;
            if ((epi && !(SIDES & 2)) || (!epi && !(SIDES & 1))) continue;
            constexpr uint32_t in_inner = CG::in_n_inner, out_inner = CG::out_n_inner;
            const uint32_t inner = epi ? out_inner : in_inner;
            const uint32_t numel = CG::vec_numel[v], period = CG::vec_period[v];
#pragma unroll
            for (int k = 0; k < K; ++k) {
                s.vraw[v][k] = u32x4{0u, 0u, 0u, 0u};
                if (!valid[k]) continue;
                const uint32_t off = epi ? out_off[k] : in_off[k];
                if ((Spec::kVecMode & 2) && numel == 1u) {
                    s.vraw[v][k] = S::splat(a.vec[v].ptr);
                    continue;
                }
                const uint32_t row = epi ? off / out_inner : off / in_inner;
                const uint32_t col = off - row * inner;
                const uint32_t o = numel >= inner ? (period == 1u ? 0u : row % period) * inner + col : col % numel;
                s.vraw[v][k] = load_cached(a.vec[v].ptr, (uint64_t)o * S::ESIZE);
            }
        }
        return;
    }
#pragma unroll
    for (int f = 0; f < Spec::NF; ++f) {
        if (f < Spec::n_full(a)) {
            const bool epi = (g.epi_full_mask >> f) & 1u;
            if ((epi && !(SIDES & 2)) || (!epi && !(SIDES & 1))) continue;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                s.fraw[f][k] = u32x4{0u, 0u, 0u, 0u};
                if (!valid[k]) continue;
                if (RAGGED) s.fraw[f][k] = load_elems<DT>(a.full[f], epi ? out_off[k] : in_off[k], cnt[k], 0u);
                else s.fraw[f][k] = load_stream(a.full[f], (uint64_t)(epi ? out_off[k] : in_off[k]) * S::ESIZE);
            }
        }
    }
#pragma unroll
    for (int v = 0; v < Spec::NV; ++v) {
        if (v < Spec::n_vec(a)) {
            const bool epi = (g.epi_vec_mask >> v) & 1u;
            if ((epi && !(SIDES & 2)) || (!epi && !(SIDES & 1))) continue;
            const uint32_t inner = epi ? g.out_n_inner : g.in_n_inner;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                s.vraw[v][k] = u32x4{0u, 0u, 0u, 0u};
                if (valid[k]) {
                    const uint32_t off = epi ? out_off[k] : in_off[k];
                    const uint32_t row = fast_div(off, epi ? g.div_out_inner : g.div_in_inner);
                    if (RAGGED) s.vraw[v][k] = load_vec_operand_elems<DT, Spec::kVecMode>(a.vec[v], row, off - row * inner, inner, cnt[k]);
                    else s.vraw[v][k] = load_vec_operand<DT, Spec::kVecMode>(a.vec[v], row, off - row * inner, inner);
                }
            }
        }
    }
}

template <int DT, int K, class Spec>
PF_DEVICE void set_positions(LaneState<DT, K, Spec>& s, const uint32_t* off, const FastDiv& d, uint32_t inner) {
#pragma unroll
    for (int k = 0; k < K; ++k) {
        s.row[k] = fast_div(off[k], d);
        s.col[k] = off[k] - s.row[k] * inner;
    }
}

template <int DT, int K, class Spec, uint32_t INNER>
PF_DEVICE void set_positions_c(LaneState<DT, K, Spec>& s, const uint32_t* off) {
#pragma unroll
    for (int k = 0; k < K; ++k) {
        s.row[k] = off[k] / INNER;
        s.col[k] = off[k] - s.row[k] * INNER;
    }
}

// RAGGED: the innermost extent (kept by the permutation) is not a whole number of vectors; the last vector of
// every innermost run is partial and all of them start at element alignment.
// CG: RuntimePermGeom, or a type that holds this launch's geometry as constants (see above).
template <int DT, int K, class Spec, bool RAGGED = false, class CG = RuntimePermGeom>
__global__ void __launch_bounds__(256) perm_rows_kernel(const ChainArgs a, const PermGeom g) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    static_assert(!(CG::kConst && RAGGED), "constant geometry is for whole vectors");
    LaneState<DT, K, Spec> s;
    uint32_t in_off[K], out_off[K], cnt[K];
    bool valid[K];
    const uint32_t base = blockIdx.x * (256u * K) + threadIdx.x;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t v = base + 256u * k;
        if constexpr (CG::kConst) valid[k] = v < CG::total_vecs;
        else valid[k] = v < g.total_vecs;
        perm_offsets_t<CG>(g, valid[k] ? v : 0u, VEC, &in_off[k], &out_off[k]);
        cnt[k] = (uint32_t)VEC;
        if (RAGGED) {
            // position inside the innermost run (tile_a elements long here): the last iteration dimension counts its vectors
            const uint32_t vv = valid[k] ? v : 0u;
            const uint32_t iv = vv - fast_div(vv, g.div[g.rank - 1]) * g.extent[g.rank - 1];
            cnt[k] = elems_below<VEC>(iv * (uint32_t)VEC, g.tile_a);
        }
    }
    perm_load_operands<DT, K, Spec, 3, RAGGED, CG>(a, g, s, in_off, out_off, valid, cnt);
    auto store = [&](int k, u32x4 v) {
        if (RAGGED) store_elems<DT>(a.out[0], out_off[k], cnt[k], v);
        else store_stream(a.out[0], (uint64_t)out_off[k] * S::ESIZE, v);
    };
    if (a.raw_copy) {
        // layout-only chain: the bits travel untouched (no fp32 round trip, NaN payloads survive)
#pragma unroll
        for (int k = 0; k < K; ++k)
            if (valid[k]) store(k, s.fraw[0][k]);
        return;
    }
    if constexpr (CG::kConst) set_positions_c<DT, K, Spec, CG::in_n_inner>(s, in_off);
    else set_positions<DT, K, Spec>(s, in_off, g.div_in_inner, g.in_n_inner);
    run_program<DT, K, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStoreT{});
    if constexpr (CG::kConst) set_positions_c<DT, K, Spec, CG::out_n_inner>(s, out_off);
    else set_positions<DT, K, Spec>(s, out_off, g.div_out_inner, g.out_n_inner);
    run_program<DT, K, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, NoStoreT{});
#pragma unroll
    for (int k = 0; k < K; ++k)
        if (valid[k]) store(k, S::pack(s.acc + k * VEC));
}

// LDS-staged variant for permutations that keep the innermost dimension and swap two outer dims A and B
// (input order ... A, B, inner; output order ... B, A, inner).  A workgroup owns a tile of tile_a x tile_b
// inner rows: it reads tile_a runs of tile_b * inner contiguous elements, runs the prologue, parks the
// fp32 -> storage converted vectors in LDS, and after one barrier writes tile_b runs of tile_a * inner
// contiguous elements, running the epilogue on the way out.  LDS traffic is 16 bytes per lane both ways:
// consecutive lanes fill consecutive 16-byte slots in the staging phase; in the read-out phase a group of
// lanes reads one inner row (inner * element size contiguous bytes) and the next group the inner row one
// staged line further.  The staged line pitch is padded so that this step advances the bank index by
// exactly one inner row: the groups that are served together then tile the 256 bytes of bank space
// side by side instead of landing on top of each other.
template <int DT, class Spec>
__global__ void __launch_bounds__(256) perm_lds_rows_kernel(const ChainArgs a, const PermGeom g) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    extern __shared__ u32x4 tile[];
    // iteration dims: [rank-3] = outer (merged batch), [rank-2]... are described by the host as:
    //   extent[0] = batch, extent[1] = A tiles, extent[2] = B tiles; inner vectors = extent[3]
    const uint32_t inner_v = g.extent[3];
    const uint32_t ta = g.tile_a, tb = g.tile_b;
    uint32_t blk = blockIdx.x;
    const uint32_t bt = blk % g.extent[2];
    blk /= g.extent[2];
    const uint32_t at = blk % g.extent[1];
    const uint32_t batch = blk / g.extent[1];
    // element offsets of the tile origin on both sides
    const uint32_t in_base = batch * g.in_stride[0] + at * ta * g.in_stride[1] + bt * tb * g.in_stride[2];
    const uint32_t out_base = batch * g.out_stride[0] + at * ta * g.out_stride[1] + bt * tb * g.out_stride[2];
    const uint32_t row_v = tb * inner_v;           // vectors per staged input run
    const uint32_t pitch = g.lds_pitch;            // padded LDS pitch in vectors (chosen by the planner)
    const uint32_t tile_v = ta * row_v;
    LaneState<DT, 1, Spec> s;
    // ---- read phase: input-contiguous
    for (uint32_t v = threadIdx.x; v < tile_v; v += 256u) {
        const uint32_t ai = v / row_v, r = v - ai * row_v;  // r = bi * inner_v + iv
        const uint32_t in_off = in_base + ai * g.in_stride[1] + r * VEC;   // B and inner are contiguous in the input
        const uint32_t bi = r / inner_v, iv = r - bi * inner_v;
        const uint32_t out_off = out_base + bi * g.out_stride[2] + ai * g.out_stride[1] + iv * VEC;
        const bool valid = true;
        perm_load_operands<DT, 1, Spec>(a, g, s, &in_off, &out_off, &valid);
        if (a.raw_copy) {
            tile[ai * pitch + r] = s.fraw[0][0];
            continue;
        }
        set_positions<DT, 1, Spec>(s, &in_off, g.div_in_inner, g.in_n_inner);
        run_program<DT, 1, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStoreT{});
        set_positions<DT, 1, Spec>(s, &out_off, g.div_out_inner, g.out_n_inner);
        run_program<DT, 1, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, NoStoreT{});
        tile[ai * pitch + r] = S::pack(s.acc);
    }
    __syncthreads();
    // ---- write phase: output-contiguous (for each b: ta runs of inner)
    const uint32_t orow_v = ta * inner_v;
    for (uint32_t v = threadIdx.x; v < tile_v; v += 256u) {
        const uint32_t bi = v / orow_v, r = v - bi * orow_v;  // r = ai * inner_v + iv
        const uint32_t ai = r / inner_v, iv = r - ai * inner_v;
        const uint32_t out_off = out_base + bi * g.out_stride[2] + r * VEC;  // A and inner are contiguous in the output
        store_stream(a.out[0], (uint64_t)out_off * S::ESIZE, tile[ai * pitch + bi * inner_v + iv]);
    }
}

// Variant for permutations that change the innermost dimension.  Let I be the input's innermost dim and O
// the output's.  A wave owns a square tile of 8 x 8 lanes; lane (ti, to) loads VEC vectors -- rows
// o = to * VEC + r of the tile, columns i = ti * VEC .. + VEC - 1 -- so every load instruction of the wave
// reads 8 runs of 8 * 16 = 128 contiguous bytes.  The lane transposes its VEC x VEC block of elements in
// registers (byte permutes for 16-bit types, pure renaming for fp32) and stores VEC vectors -- rows
// i = ti * VEC + c, columns o = to * VEC .. -- so every store instruction writes 8 runs of 128 contiguous
// bytes as well.  Both sides move whole 128-byte lines and nothing passes through LDS: the exchange the
// layout change needs fits inside one lane's registers (lane scope in the paper's terms) once the tile is
// cut this way.  Element-wise steps run on the side whose layout their operands have; to keep a single
// rounding, 16-bit chains may compute on one side only (the planner enforces it).
template <int DT>
PF_DEVICE void transpose_block(const u32x4 (&in)[Storage<DT>::VEC], u32x4 (&out)[Storage<DT>::VEC]) {
    if (DT == DT_F32) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) out[c][r] = in[r][c];
    } else {
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // output vector c, dword j = elements (row 2j, column c) and (row 2j + 1, column c)
                const uint32_t lo = in[2 * j][c / 2], hi = in[2 * j + 1][c / 2];
                out[c][j] = (c & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
            }
    }
}

// RAGGED: the two transposed extents need not be whole vectors: a lane's block is ni x no elements (0 .. VEC
// each), rows and columns beyond that are neither loaded nor stored, and every access is element-aligned.
// (Left to itself the compiler interleaves the eight rows' conversions of a specialised fp16 chain and ends up at 234
// registers, two waves per SIMD and 2.9 TB/s; held to four waves per SIMD it needs 93 and no scratch.)
template <int DT, class Spec, bool RAGGED = false>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(Spec::kStatic ? 4 : 2))) perm_tile_kernel(const ChainArgs a, const PermGeom g) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    constexpr uint32_t TE = 8u * VEC;  // tile edge in elements
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t tile = blockIdx.x * 4u + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (tile >= g.total_vecs) return;  // total_vecs counts tiles in this variant; wave-uniform exit
    uint32_t in_base, out_base;
    perm_offsets(g, tile, 1u, &in_base, &out_base);
    const uint32_t q_o = fast_div(tile, g.div[g.rank - 1]);
    const uint32_t ot = tile - q_o * g.extent[g.rank - 1];
    const uint32_t it = q_o - fast_div(q_o, g.div[g.rank - 2]) * g.extent[g.rank - 2];
    const uint32_t ti = lane & 7u, to = lane >> 3;
    // elements of this lane's block along the input's innermost dimension (ni) and the output's (no)
    const uint32_t ni = elems_below<VEC>(it * TE + ti * VEC, g.tile_a), no = elems_below<VEC>(ot * TE + to * VEC, g.tile_b);
    const bool valid = ni != 0u && no != 0u;

    LaneState<DT, 1, Spec> s;
    u32x4 blk[VEC], outv[VEC];
    // nothing but the load / nothing after the transposition: known when the kernel is compiled for a static chain
    using ProL = typename Spec::Pro;
    using EpiL = typename Spec::Epi;
    const bool pro_trivial = ProL::kDynamic ? a.pro.n == 1 : ProL::n == 1;
    const bool has_epi = EpiL::kDynamic ? a.epi.n != 0 : EpiL::n != 0;
    // Whole-vector tiles load without a branch: a lane outside the tensor (a partial tile at an edge) reads the tile's
    // first vector instead and stores nothing.  Behind a guard every load merges with a fill value at the join, which
    // the compiler resolves by waiting for it -- the eight rows' operands were then fetched one round trip after the
    // other, each waiting for the whole block as well.
    uint32_t in_off[VEC];
#pragma unroll
    for (int r = 0; r < VEC; ++r) {
        in_off[r] = in_base + (to * VEC + r) * g.t_in_stride_o + ti * VEC;
        if (RAGGED) {
            blk[r] = u32x4{0u, 0u, 0u, 0u};
        } else {
            in_off[r] = valid ? in_off[r] : in_base;
            blk[r] = load_stream(a.full[0], (uint64_t)in_off[r] * S::ESIZE);
        }
    }
    if (RAGGED && valid) {
        // The block's rows without a branch per row: a row past the block's end (r >= no) reads the last one that exists
        // and is not stored; whether the vectors are whole (ni == VEC) is the same for all rows and told apart once.  A
        // partial vector is read whole where the tensor continues behind it (see load_elems).
        const uint32_t last_row = in_base + (to * VEC + (no - 1u)) * g.t_in_stride_o + ti * VEC;
        const bool room = (uint64_t)last_row + (uint64_t)VEC <= a.rows * a.n_inner;
        if (ni == (uint32_t)VEC) {
#pragma unroll
            for (int r = 0; r < VEC; ++r)
                blk[r] = load_elems<DT>(a.full[0], in_base + (to * VEC + min((uint32_t)r, no - 1u)) * g.t_in_stride_o + ti * VEC, (uint32_t)VEC, 0u);
        } else {
#pragma unroll
            for (int r = 0; r < VEC; ++r)
                blk[r] = load_elems<DT>(a.full[0], in_base + (to * VEC + min((uint32_t)r, no - 1u)) * g.t_in_stride_o + ti * VEC, ni, 0u, room);
        }
    }
    // A specialised chain with one or two operands beside the block asks for the operands of all its rows right behind
    // the block (they arrive together with it) and keeps them in registers; fetched row by row, in front of each row's
    // program, every row would cost the wave a trip to the cache of its own -- and a launch of this kernel is a single
    // round of resident waves, so a wave's latency is the kernel's.
    constexpr bool kBatchOperands = Spec::kStatic && !RAGGED && (Spec::NF - 1) + Spec::NV <= 2;
    if (!pro_trivial && kBatchOperands) {
        u32x4 fop[Spec::NF][VEC], vop[Spec::NV > 0 ? Spec::NV : 1][VEC];
        const uint32_t zero = 0u;
        const bool row_ok = true;
#pragma unroll
        for (int r = 0; r < VEC; ++r) {
            perm_load_operands<DT, 1, Spec, 1, RAGGED>(a, g, s, &in_off[r], &zero, &row_ok, &ni);
#pragma unroll
            for (int f = 1; f < Spec::NF; ++f) fop[f][r] = s.fraw[f][0];
#pragma unroll
            for (int v = 0; v < Spec::NV; ++v) vop[v][r] = s.vraw[v][0];
        }
#pragma unroll
        for (int r = 0; r < VEC; ++r) {
#pragma unroll
            for (int f = 1; f < Spec::NF; ++f) s.fraw[f][0] = fop[f][r];
#pragma unroll
            for (int v = 0; v < Spec::NV; ++v) s.vraw[v][0] = vop[v][r];
            s.fraw[0][0] = blk[r];
            set_positions<DT, 1, Spec>(s, &in_off[r], g.div_in_inner, g.in_n_inner);
            run_program<DT, 1, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStoreT{});
            blk[r] = S::pack(s.acc);
        }
    } else if (!pro_trivial) {
#pragma unroll
        for (int r = 0; r < VEC; ++r) {
            const uint32_t zero = 0u;
            const bool row_ok = RAGGED ? valid && (uint32_t)r < no : true;
            perm_load_operands<DT, 1, Spec, 1, RAGGED>(a, g, s, &in_off[r], &zero, &row_ok, &ni);
            s.fraw[0][0] = blk[r];
            set_positions<DT, 1, Spec>(s, &in_off[r], g.div_in_inner, g.in_n_inner);
            run_program<DT, 1, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStoreT{});
            blk[r] = S::pack(s.acc);
        }
    }
    transpose_block<DT>(blk, outv);
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
        const uint32_t out_off_real = out_base + (ti * VEC + c) * g.t_out_stride_i + to * VEC;
        const uint32_t out_off = RAGGED || valid ? out_off_real : out_base;  // (as above)
        const bool row_ok = valid && (!RAGGED || (uint32_t)c < ni);
        if (has_epi) {
            const uint32_t zero = 0u;
            const bool load_ok = RAGGED ? row_ok : true;
            perm_load_operands<DT, 1, Spec, 2, RAGGED>(a, g, s, &zero, &out_off, &load_ok, &no);
            S::unpack(outv[c], s.acc);
            set_positions<DT, 1, Spec>(s, &out_off, g.div_out_inner, g.out_n_inner);
            run_program<DT, 1, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, NoStoreT{});
            outv[c] = S::pack(s.acc);
        }
        if (RAGGED) {
            if (row_ok) store_elems<DT>(a.out[0], out_off, no, outv[c]);
        } else if (valid) {
            store_stream(a.out[0], (uint64_t)out_off * S::ESIZE, outv[c]);
        }
    }
}

}  // namespace pf
