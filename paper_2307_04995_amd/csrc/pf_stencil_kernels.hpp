// Stencil family: prologue -> depthwise 3 x 3 or 5 x 5 convolution (channels-last, stride 1, zero "same" padding)
// -> epilogue, one kernel.
//
// The depthwise convolution of the paper's EfficientNet fragment (section 6, preprocessing of the computation
// graph) does 9 multiply-adds per element it reads and writes: memory-intensive, so it is expressed with the
// same building blocks as the other chains and fused with the activation in front of it.  In GIR terms the
// nine taps are nine reads of overlapping slices of one tensor; the read-after-read merging rule (section 5.1)
// keeps the overlap on chip: a lane owns 8 channels of one image column and walks down a strip of rows with a
// 3 x 3 window of activated values in registers, so a value enters the window once per strip; the columns to
// its left and right are the neighbouring lanes' columns and come from the first-level cache.  HBM sees every
// input element about once (plus the two halo rows per strip) and every output element once.
//
// The prologue runs on every value as it enters the window (zero padding is applied after it, as the operator
// order says); the epilogue runs on the finished sum.
#pragma once
#include "pf_row_kernels.hpp"

namespace pf {

// Memory access of the family.  ragged (a compile-time fact of the kernel: a run-time test at every load costs the
// aligned kernels a third of their speed): the channel count is not a whole number of vectors, so a position starts at
// element alignment and its last vector holds `cnt` channels; the rest of that vector reads as zero (and contributes
// zero to every tap) and is not stored.
// total: elements of the tensor read from, when known (0 = not): a partial vector is then read as a whole one wherever
// 16 bytes from its start still lie inside the tensor (they belong to the next position) -- see load_elems.
template <int DT>
PF_DEVICE u32x4 stencil_load(const void* base, uint64_t elem, bool ragged, uint32_t cnt, uint64_t total = 0) {
    return ragged ? load_elems<DT>(base, elem, cnt, 0u, elem + (uint64_t)Storage<DT>::VEC <= total) : load_cached(base, elem * Storage<DT>::ESIZE);
}
template <int DT>
PF_DEVICE void stencil_store(void* base, uint64_t elem, bool ragged, uint32_t cnt, u32x4 v) {
    if (ragged) store_elems<DT>(base, elem, cnt, v);
    else store_stream(base, elem * Storage<DT>::ESIZE, v);
}
template <int DT, int VM>
PF_DEVICE u32x4 stencil_load_vec(const VecArg& va, uint32_t row, uint32_t col, uint32_t n, bool ragged, uint32_t cnt) {
    return ragged ? load_vec_operand_elems<DT, VM>(va, row, col, n, cnt) : load_vec_operand<DT, VM>(va, row, col, n);
}

constexpr int kStencilRows = 6;   // output rows per strip, 3 x 3 kernels (8 input rows are read for them)
constexpr int kStencilRows5 = 4;  // output rows per strip, 5 x 5 kernels (staged variant only; 8 input rows as well)

template <int DT, class Spec, bool RAGGED = false>
__global__ void __launch_bounds__(256) dwconv3x3_kernel(const ChainArgs a, const StencilGeom g) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;  // (column, channel vector) of this lane, channel fastest
    if (t >= g.row_vecs) return;
    const uint32_t wcol = fast_div(t, g.div_cv);
    const uint32_t cvi = t - wcol * g.cv;
    constexpr bool ragged = RAGGED;
    const uint32_t cnt = ragged ? elems_below<Storage<DT>::VEC>(cvi * (uint32_t)Storage<DT>::VEC, g.c) : (uint32_t)Storage<DT>::VEC;
    const uint32_t sample = blockIdx.z;
    const uint32_t h0 = blockIdx.y * (uint32_t)kStencilRows;
    const int wslot = Spec::gamma(a);  // broadcast slot that holds the kernels [3, 3, channels]

    // the nine kernel vectors of this lane's channels, kept packed
    u32x4 wraw[9];
#pragma unroll
    for (int k = 0; k < 9; ++k)
        wraw[k] = stencil_load<DT>(a.vec[wslot].ptr, (uint64_t)k * g.c + cvi * VEC, ragged, cnt);

    // which operands each side of the convolution reads: known at compile time for a specialised kernel
    const uint32_t pro_full = Spec::kStatic ? list_operand_mask<typename Spec::Pro>(K_FULL) : ~g.epi_full_mask;
    const uint32_t pro_vec = Spec::kStatic ? list_operand_mask<typename Spec::Pro>(K_VEC) : ~g.epi_vec_mask;
    const uint32_t epi_full = Spec::kStatic ? list_operand_mask<typename Spec::Epi>(K_FULL) : g.epi_full_mask;
    const uint32_t epi_vec = Spec::kStatic ? list_operand_mask<typename Spec::Epi>(K_VEC) : g.epi_vec_mask;
    // When the prologue only loads and applies steps that stay exact in the storage type (RELU in front of the
    // convolution is the standard case), the window holds the activated values packed: half the registers.
    constexpr bool kPacked = DT != DT_F32 && list_keeps_storage_precision<typename Spec::Pro>();
    constexpr int WE = kPacked ? 4 : VEC;  // 32-bit words per window entry

    LaneState<DT, 1, Spec> s;
    s.col[0] = cvi * VEC;
    // the epilogue's operands, read at the output position
    auto load_epilogue_operands = [&](uint32_t pos) {
        s.row[0] = pos;
#pragma unroll
        for (int f = 0; f < Spec::NF; ++f)
            if (f < Spec::n_full(a) && ((epi_full >> f) & 1u))
                s.fraw[f][0] = stencil_load<DT>(a.full[f], (uint64_t)pos * g.c + cvi * VEC, ragged, cnt);
#pragma unroll
        for (int v = 0; v < Spec::NV; ++v)
            if (v < Spec::n_vec(a) && v != wslot && ((epi_vec >> v) & 1u))
                s.vraw[v][0] = stencil_load_vec<DT, Spec::kVecMode>(a.vec[v], pos, s.col[0], g.c, ragged, cnt);
    };

    uint32_t win[3][3][WE];  // activated values (fp32 bits, or packed): window row (input row mod 3), column -1 / 0 / +1
    // An input row enters the window in two steps so that its loads are in flight while the previous output
    // row is computed: fetch_row issues the loads of the three columns, admit_row runs the prologue on them.
    u32x4 pend_f[3][at_least_1(Spec::NF)], pend_v[3][at_least_1(Spec::NV)];
    auto inside_image = [&](int r, int dw) {
        const int col = (int)wcol + dw - 1;
        return r >= 0 && r < (int)g.h && col >= 0 && col < (int)g.w;
    };
    auto fetch_row = [&](int r) {
#pragma unroll
        for (int dw = 0; dw < 3; ++dw) {
            if (!inside_image(r, dw)) continue;
            const uint32_t pos = (sample * g.h + (uint32_t)r) * g.w + (uint32_t)((int)wcol + dw - 1);
#pragma unroll
            for (int f = 0; f < Spec::NF; ++f)
                if (f < Spec::n_full(a) && ((pro_full >> f) & 1u))
                    pend_f[dw][f] = stencil_load<DT>(a.full[f], (uint64_t)pos * g.c + cvi * VEC, ragged, cnt, (uint64_t)g.n * g.h * g.w * g.c);
#pragma unroll
            for (int v = 0; v < Spec::NV; ++v)
                if (v < Spec::n_vec(a) && v != wslot && ((pro_vec >> v) & 1u))
                    pend_v[dw][v] = stencil_load_vec<DT, Spec::kVecMode>(a.vec[v], pos, s.col[0], g.c, ragged, cnt);
        }
    };
    auto admit_row = [&](int r, int slot) {
#pragma unroll
        for (int dw = 0; dw < 3; ++dw) {
            const bool inside = inside_image(r, dw);
            if (inside) {
                s.row[0] = (sample * g.h + (uint32_t)r) * g.w + (uint32_t)((int)wcol + dw - 1);
#pragma unroll
                for (int f = 0; f < Spec::NF; ++f)
                    if (f < Spec::n_full(a) && ((pro_full >> f) & 1u)) s.fraw[f][0] = pend_f[dw][f];
#pragma unroll
                for (int v = 0; v < Spec::NV; ++v)
                    if (v < Spec::n_vec(a) && v != wslot && ((pro_vec >> v) & 1u)) s.vraw[v][0] = pend_v[dw][v];
                run_program<DT, 1, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStore{});
            }
            if (kPacked) {
                const u32x4 packed = S::pack(s.acc);
#pragma unroll
                for (int e = 0; e < 4; ++e) win[slot][dw][e] = inside ? packed[e] : 0u;
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) win[slot][dw][e % WE] = inside ? __builtin_bit_cast(uint32_t, s.acc[e]) : 0u;
            }
        }
    };

    // relative numbering: input row h0 + k lives in window row k mod 3 (k = -1 -> 2)
    fetch_row((int)h0 - 1);
    admit_row((int)h0 - 1, 2);
    fetch_row((int)h0);
    admit_row((int)h0, 0);
    fetch_row((int)h0 + 1);
#pragma unroll
    for (int i = 0; i < kStencilRows; ++i) {
        const uint32_t row = h0 + (uint32_t)i;
        if (row >= g.h) break;
        admit_row((int)row + 1, (i + 1) % 3);
        if (i + 1 < kStencilRows) fetch_row((int)row + 2);  // in flight during this row's arithmetic
        float acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;
#pragma unroll
        for (int dh = 0; dh < 3; ++dh) {
            const int slot = (i + dh + 2) % 3;  // input row row + dh - 1 = h0 + (i + dh - 1)
#pragma unroll
            for (int dw = 0; dw < 3; ++dw) {
                float wf[VEC], xf[VEC];
                S::unpack(wraw[dh * 3 + dw], wf);
                if (kPacked) {
                    S::unpack(u32x4{win[slot][dw][0], win[slot][dw][1 % WE], win[slot][dw][2 % WE], win[slot][dw][3 % WE]}, xf);
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) xf[e] = __builtin_bit_cast(float, win[slot][dw][e % WE]);
                }
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = __builtin_fmaf(wf[e], xf[e], acc[e]);
            }
        }
        const uint32_t pos = (sample * g.h + row) * g.w + wcol;
        load_epilogue_operands(pos);
#pragma unroll
        for (int e = 0; e < VEC; ++e) s.acc[e] = acc[e];
        run_program<DT, 1, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, NoStore{});
        stencil_store<DT>(a.out[0], (uint64_t)pos * g.c + cvi * VEC, ragged, cnt, S::pack(s.acc));
    }
}

// Staged variant: the workgroup activates every input value of its tile ONCE and shares it through LDS.
//
// The direct variant above runs the prologue on each of the three columns a lane reads per input row, i.e.
// three times per input value, and its neighbouring columns come from the cache.  Here a workgroup first
// brings the eight input rows of its strip, for its 256 lanes plus a halo of one image column on either side,
// through the prologue and into an LDS tile (one barrier), then every lane reads its nine taps per output row
// from the tile.  The prologue runs about 1.3 times per input value (halo rows and columns), the loads of a
// whole strip are in flight together, and no window lives in registers.
//
// LDS layout: tile[input row 0..7][staging lane 0 .. 256 + 2 cv), entries of 16 bytes (packed storage type, when
// the prologue keeps storage precision) or 32 bytes (fp32).  Lanes read consecutive entries: no bank conflicts.
template <int DT, class Spec, int KS, bool RAGGED = false>
__global__ void __launch_bounds__(256) dwconv_staged_kernel(const ChainArgs a, const StencilGeom g) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    constexpr bool kPacked = DT != DT_F32 && list_keeps_storage_precision<typename Spec::Pro>();
    constexpr int EV = (kPacked || DT == DT_F32) ? 1 : 2;  // 16-byte vectors per tile entry
    static_assert(KS == 3 || KS == 5, "kernel extents 3 and 5");
    constexpr int R = KS / 2;                      // halo rows above and below, halo image columns left and right
    constexpr int kOut = KS == 3 ? kStencilRows : kStencilRows5;  // output rows per strip
    constexpr int kRows = kOut + KS - 1;           // input rows of a strip: eight for both kernel extents
    extern __shared__ u32x4 tile[];

    // Tile of this workgroup.  Workgroups are dealt to the eight compute dies round-robin by their linear index,
    // and each die has its own L2.  Tiles that share halo rows and columns are therefore numbered so that
    // neighbours fall on the same die (tile = (index mod 8) * tiles_per_die + index / 8): a halo fetched by one
    // workgroup is an L2 hit for the next instead of a second trip to HBM.
    const uint32_t tile_id = (blockIdx.x & 7u) * g.tiles_per_die + (blockIdx.x >> 3);
    if (tile_id >= g.tiles) return;  // (the grid is rounded up to a multiple of eight)
    const uint32_t tx = tile_id % g.tiles_x;
    const uint32_t ty = (tile_id / g.tiles_x) % g.tiles_y;
    const uint32_t t0 = tx * 256u;  // first (column, channel vector) lane of this workgroup
    const uint32_t sample = tile_id / (g.tiles_x * g.tiles_y);
    const uint32_t h0 = ty * (uint32_t)kOut;
    const int wslot = Spec::gamma(a);
    const uint32_t cv = g.cv;
    const uint32_t tw = 256u + 2u * R * cv;  // staging lanes per row
    const uint32_t pro_full = Spec::kStatic ? list_operand_mask<typename Spec::Pro>(K_FULL) : ~g.epi_full_mask;
    const uint32_t pro_vec = Spec::kStatic ? list_operand_mask<typename Spec::Pro>(K_VEC) : ~g.epi_vec_mask;
    const uint32_t epi_full = Spec::kStatic ? list_operand_mask<typename Spec::Epi>(K_FULL) : g.epi_full_mask;
    const uint32_t epi_vec = Spec::kStatic ? list_operand_mask<typename Spec::Epi>(K_VEC) : g.epi_vec_mask;

    LaneState<DT, 1, Spec> s;

    // ---- stage: staging lane j of input row h0 - R + r holds image lane t0 - R * cv + j
    for (uint32_t j = threadIdx.x; j < tw; j += 256u) {
        const int64_t lane_pos = (int64_t)t0 - (int64_t)R * cv + j;
        const bool lane_ok = lane_pos >= 0 && lane_pos < (int64_t)g.row_vecs;
        const uint32_t lp = lane_ok ? (uint32_t)lane_pos : 0u;
        const uint32_t wcol = fast_div(lp, g.div_cv);
        const uint32_t cvi = lp - wcol * cv;
        constexpr bool ragged = RAGGED;
        const uint32_t cnt = ragged ? elems_below<Storage<DT>::VEC>(cvi * (uint32_t)Storage<DT>::VEC, g.c) : (uint32_t)Storage<DT>::VEC;
        s.col[0] = cvi * VEC;
        u32x4 pend_f[kRows][at_least_1(Spec::NF)];
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const int row = (int)h0 - R + r;
            const bool ok = lane_ok && row >= 0 && row < (int)g.h;
            const uint32_t pos = (sample * g.h + (uint32_t)(ok ? row : 0)) * g.w + wcol;
#pragma unroll
            for (int f = 0; f < Spec::NF; ++f) {
                pend_f[r][f] = u32x4{0u, 0u, 0u, 0u};
                if (f < Spec::n_full(a) && ((pro_full >> f) & 1u) && ok)
                    pend_f[r][f] = stencil_load<DT>(a.full[f], (uint64_t)pos * g.c + cvi * VEC, ragged, cnt, (uint64_t)g.n * g.h * g.w * g.c);
            }
        }
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const int row = (int)h0 - R + r;
            const bool ok = lane_ok && row >= 0 && row < (int)g.h;
            if (ok) {
                s.row[0] = (sample * g.h + (uint32_t)row) * g.w + wcol;
#pragma unroll
                for (int f = 0; f < Spec::NF; ++f)
                    if (f < Spec::n_full(a) && ((pro_full >> f) & 1u)) s.fraw[f][0] = pend_f[r][f];
#pragma unroll
                for (int v = 0; v < Spec::NV; ++v)
                    if (v < Spec::n_vec(a) && v != wslot && ((pro_vec >> v) & 1u))
                        s.vraw[v][0] = stencil_load_vec<DT, Spec::kVecMode>(a.vec[v], s.row[0], s.col[0], g.c, ragged, cnt);
                run_program<DT, 1, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStore{});
            }
            u32x4* dst = tile + ((uint32_t)r * tw + j) * EV;
            if (kPacked) {
                dst[0] = ok ? S::pack(s.acc) : u32x4{0u, 0u, 0u, 0u};
            } else {
#pragma unroll
                for (int q = 0; q < EV; ++q) {
                    u32x4 w4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w4[e] = ok ? __builtin_bit_cast(uint32_t, s.acc[(q * 4 + e) % VEC]) : 0u;
                    dst[q] = w4;
                }
            }
        }
    }
    __syncthreads();

    // ---- compute: lane t0 + tid, six output rows, nine taps each from the tile
    const uint32_t t = t0 + threadIdx.x;
    if (t >= g.row_vecs) return;
    const uint32_t wcol = fast_div(t, g.div_cv);
    const uint32_t cvi = t - wcol * cv;
    constexpr bool ragged = RAGGED;
    const uint32_t cnt = ragged ? elems_below<Storage<DT>::VEC>(cvi * (uint32_t)Storage<DT>::VEC, g.c) : (uint32_t)Storage<DT>::VEC;
    s.col[0] = cvi * VEC;
    // fp16 tile entries meet fp16 kernels: the multiply-add takes both halves of the packed registers directly
    // (v_fma_mix_f32 widens them on the fly), so nothing is unpacked in the inner loop
    constexpr bool kMix = kPacked && DT == DT_F16;
    // 3 x 3: the nine kernel vectors live in registers; 5 x 5: they are read where they are used (first-level cache)
    constexpr bool kKeepW = KS == 3;
    constexpr int NW = kKeepW ? KS * KS : 1;
    u32x4 wraw[NW];
    float wf[(kMix || !kKeepW) ? 1 : NW][VEC];
    auto load_w = [&](int k) { return stencil_load<DT>(a.vec[wslot].ptr, (uint64_t)k * g.c + cvi * VEC, ragged, cnt); };
    if (kKeepW) {
#pragma unroll
        for (int k = 0; k < NW; ++k) {
            wraw[k] = load_w(k);
            if (!kMix) S::unpack(wraw[k], wf[k % ((kMix || !kKeepW) ? 1 : NW)]);
        }
    }
    // 5 x 5: the kernel vectors do not fit the registers beside the window, so the loops are turned inside out: a kernel
    // row's five vectors are fetched together (one trip to the cache per kernel row, not one per tap and output row) and
    // applied to every output row of the strip before the next kernel row is fetched.
    float acc_all[kKeepW ? 1 : kOut][VEC];
    if (!kKeepW) {
#pragma unroll
        for (int i = 0; i < kOut; ++i)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc_all[i % (kKeepW ? 1 : kOut)][e] = 0.0f;
#pragma unroll
        for (int dh = 0; dh < KS; ++dh) {
            u32x4 wrow[KS];
#pragma unroll
            for (int dw = 0; dw < KS; ++dw) wrow[dw] = load_w(dh * KS + dw);
#pragma unroll
            for (int i = 0; i < kOut; ++i) {
                float(&acc)[VEC] = acc_all[i % (kKeepW ? 1 : kOut)];
#pragma unroll
                for (int dw = 0; dw < KS; ++dw) {
                    // (rows of the window past the image's end hold zeros or halo values; their outputs are not stored)
                    const u32x4* src = tile + ((uint32_t)(i + dh) * tw + threadIdx.x + (uint32_t)dw * cv) * EV;
                    const u32x4 wv = wrow[dw];
                    if (kMix) {
                        const u32x4 xv = src[0];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const uint32_t xp = xv[j], wp = wv[j];
                            asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[0,0,0] op_sel_hi:[1,1,0]" : "+v"(acc[(2 * j) % VEC]) : "v"(xp), "v"(wp));
                            asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[1,1,0] op_sel_hi:[1,1,0]" : "+v"(acc[(2 * j + 1) % VEC]) : "v"(xp), "v"(wp));
                        }
                        continue;
                    }
                    float xf[VEC], wu[VEC];
                    S::unpack(wv, wu);
                    if (kPacked) {
                        S::unpack(src[0], xf);
                    } else {
#pragma unroll
                        for (int q = 0; q < EV; ++q) {
                            const u32x4 w4 = src[q];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const uint32_t bits = w4[e];  // (a bit cast applied directly to a vector element is miscompiled)
                                if (q * 4 + e < VEC) xf[(q * 4 + e) % VEC] = __builtin_bit_cast(float, bits);
                            }
                        }
                    }
#pragma unroll
                    for (int e = 0; e < VEC; ++e) acc[e] = __builtin_fmaf(wu[e], xf[e], acc[e]);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < kOut; ++i) {
        const uint32_t row = h0 + (uint32_t)i;
        if (row >= g.h) break;
        float acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = kKeepW ? 0.0f : acc_all[i % (kKeepW ? 1 : kOut)][e];
#pragma unroll
        for (int dh = 0; dh < (kKeepW ? KS : 0); ++dh)
#pragma unroll
            for (int dw = 0; dw < KS; ++dw) {
                const u32x4* src = tile + ((uint32_t)(i + dh) * tw + threadIdx.x + (uint32_t)dw * cv) * EV;
                const u32x4 wv = kKeepW ? wraw[(dh * KS + dw) % NW] : load_w(dh * KS + dw);
                if (kMix) {
                    const u32x4 xv = src[0];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t xp = xv[j], wp = wv[j];
                        asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[0,0,0] op_sel_hi:[1,1,0]" : "+v"(acc[(2 * j) % VEC]) : "v"(xp), "v"(wp));
                        asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[1,1,0] op_sel_hi:[1,1,0]" : "+v"(acc[(2 * j + 1) % VEC]) : "v"(xp), "v"(wp));
                    }
                    continue;
                }
                float xf[VEC], wu[VEC];
                if (kKeepW) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) wu[e] = wf[(dh * KS + dw) % ((kMix || !kKeepW) ? 1 : NW)][e];
                } else {
                    S::unpack(wv, wu);
                }
                if (kPacked) {
                    S::unpack(src[0], xf);
                } else {
#pragma unroll
                    for (int q = 0; q < EV; ++q) {
                        const u32x4 w4 = src[q];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const uint32_t bits = w4[e];  // (a bit cast applied directly to a vector element is miscompiled)
                            if (q * 4 + e < VEC) xf[(q * 4 + e) % VEC] = __builtin_bit_cast(float, bits);
                        }
                    }
                }
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = __builtin_fmaf(wu[e], xf[e], acc[e]);
            }
        const uint32_t pos = (sample * g.h + row) * g.w + wcol;
        s.row[0] = pos;
#pragma unroll
        for (int f = 0; f < Spec::NF; ++f)
            if (f < Spec::n_full(a) && ((epi_full >> f) & 1u))
                s.fraw[f][0] = stencil_load<DT>(a.full[f], (uint64_t)pos * g.c + cvi * VEC, ragged, cnt);
#pragma unroll
        for (int v = 0; v < Spec::NV; ++v)
            if (v < Spec::n_vec(a) && v != wslot && ((epi_vec >> v) & 1u))
                s.vraw[v][0] = stencil_load_vec<DT, Spec::kVecMode>(a.vec[v], pos, s.col[0], g.c, ragged, cnt);
#pragma unroll
        for (int e = 0; e < VEC; ++e) s.acc[e] = acc[e];
        run_program<DT, 1, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, NoStore{});
        stencil_store<DT>(a.out[0], (uint64_t)pos * g.c + cvi * VEC, ragged, cnt, S::pack(s.acc));
    }
}

// Strided variant (stride >= 2 along both axes, as in the down-sampling blocks of the network the paper's fragment
// comes from): a lane owns 8 channels of one OUTPUT column and walks down a strip of output rows.  Consecutive
// outputs share at most one input row and one input column, so there is no window worth keeping: the KS x KS
// taps of an output are loaded where they are used, one kernel row's loads in flight together, and what
// neighbouring lanes and rows read twice comes from the first-level cache.  The prologue runs on every tap.

template <int DT, class Spec, int KS, bool RAGGED = false>
__global__ void __launch_bounds__(256) dwconv_strided_kernel(const ChainArgs a, const StencilGeom g) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    constexpr int R = KS / 2;
    static_assert(KS == 3 || KS == 5, "kernel extents 3 and 5");
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;  // (output column, channel vector), channel fastest
    if (t >= g.out_row_vecs) return;
    const uint32_t ocol = fast_div(t, g.div_cv);
    const uint32_t cvi = t - ocol * g.cv;
    constexpr bool ragged = RAGGED;
    const uint32_t cnt = ragged ? elems_below<Storage<DT>::VEC>(cvi * (uint32_t)Storage<DT>::VEC, g.c) : (uint32_t)Storage<DT>::VEC;
    const uint32_t sample = blockIdx.z;
    const uint32_t i0 = blockIdx.y * g.strip_rows;  // strip_rows output rows per workgroup (the planner keeps the grid large)
    const int wslot = Spec::gamma(a);
    const uint32_t pro_full = Spec::kStatic ? list_operand_mask<typename Spec::Pro>(K_FULL) : ~g.epi_full_mask;
    const uint32_t pro_vec = Spec::kStatic ? list_operand_mask<typename Spec::Pro>(K_VEC) : ~g.epi_vec_mask;
    const uint32_t epi_full = Spec::kStatic ? list_operand_mask<typename Spec::Epi>(K_FULL) : g.epi_full_mask;
    const uint32_t epi_vec = Spec::kStatic ? list_operand_mask<typename Spec::Epi>(K_VEC) : g.epi_vec_mask;
    auto load_w = [&](int k) { return stencil_load<DT>(a.vec[wslot].ptr, (uint64_t)k * g.c + cvi * VEC, ragged, cnt); };
    // 3 x 3: the nine kernel vectors stay in registers; 5 x 5: read where they are used (first-level cache)
    constexpr bool kKeepW = KS == 3;
    u32x4 wraw[kKeepW ? KS * KS : 1];
    if (kKeepW) {
#pragma unroll
        for (int k = 0; k < KS * KS; ++k) wraw[k % (kKeepW ? KS * KS : 1)] = load_w(k);
    }

    LaneState<DT, 1, Spec> s;
    s.col[0] = cvi * VEC;
#pragma unroll 1
    for (uint32_t r = 0; r < g.strip_rows; ++r) {
        const uint32_t orow = i0 + r;
        if (orow >= g.oh) break;
        float acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;
#pragma unroll
        for (int dh = 0; dh < KS; ++dh) {
            const int ii = (int)(orow * g.stride) + dh - R;
            u32x4 pend_f[KS][at_least_1(Spec::NF)], pend_v[KS][at_least_1(Spec::NV)];
            bool ok[KS];
            uint32_t pos[KS];
            // (5 x 5: the kernel row's vectors are asked for together with its taps, not one by one where they are used)
            u32x4 wrow[kKeepW ? 1 : KS];
            if (!kKeepW) {
#pragma unroll
                for (int dw = 0; dw < KS; ++dw) wrow[dw % (kKeepW ? 1 : KS)] = load_w(dh * KS + dw);
            }
#pragma unroll
            for (int dw = 0; dw < KS; ++dw) {
                const int jj = (int)(ocol * g.stride) + dw - R;
                ok[dw] = ii >= 0 && ii < (int)g.h && jj >= 0 && jj < (int)g.w;
                pos[dw] = ok[dw] ? (sample * g.h + (uint32_t)ii) * g.w + (uint32_t)jj : 0u;
                // (no branch around the loads: a tap in the padding reads position 0 and is skipped below; behind a guard
                // every tap's load would wait for the one before)
#pragma unroll
                for (int f = 0; f < Spec::NF; ++f)
                    if (f < Spec::n_full(a) && ((pro_full >> f) & 1u))
                        pend_f[dw][f] = stencil_load<DT>(a.full[f], (uint64_t)pos[dw] * g.c + cvi * VEC, ragged, cnt, (uint64_t)g.n * g.h * g.w * g.c);
#pragma unroll
                for (int v = 0; v < Spec::NV; ++v)
                    if (v < Spec::n_vec(a) && v != wslot && ((pro_vec >> v) & 1u))
                        pend_v[dw][v] = stencil_load_vec<DT, Spec::kVecMode>(a.vec[v], pos[dw], s.col[0], g.c, ragged, cnt);
            }
#pragma unroll
            for (int dw = 0; dw < KS; ++dw) {
                if (!ok[dw]) continue;  // zero padding: the tap contributes nothing (the prologue is not applied to it)
                s.row[0] = pos[dw];
#pragma unroll
                for (int f = 0; f < Spec::NF; ++f)
                    if (f < Spec::n_full(a) && ((pro_full >> f) & 1u)) s.fraw[f][0] = pend_f[dw][f];
#pragma unroll
                for (int v = 0; v < Spec::NV; ++v)
                    if (v < Spec::n_vec(a) && v != wslot && ((pro_vec >> v) & 1u)) s.vraw[v][0] = pend_v[dw][v];
                run_program<DT, 1, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStore{});
                float wf[VEC];
                S::unpack(kKeepW ? wraw[(dh * KS + dw) % (kKeepW ? KS * KS : 1)] : wrow[dw % (kKeepW ? 1 : KS)], wf);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = __builtin_fmaf(wf[e], s.acc[e], acc[e]);
            }
        }
        const uint32_t opos = (sample * g.oh + orow) * g.ow + ocol;
        s.row[0] = opos;
#pragma unroll
        for (int f = 0; f < Spec::NF; ++f)
            if (f < Spec::n_full(a) && ((epi_full >> f) & 1u))
                s.fraw[f][0] = stencil_load<DT>(a.full[f], (uint64_t)opos * g.c + cvi * VEC, ragged, cnt);
#pragma unroll
        for (int v = 0; v < Spec::NV; ++v)
            if (v < Spec::n_vec(a) && v != wslot && ((epi_vec >> v) & 1u))
                s.vraw[v][0] = stencil_load_vec<DT, Spec::kVecMode>(a.vec[v], opos, s.col[0], g.c, ragged, cnt);
#pragma unroll
        for (int e = 0; e < VEC; ++e) s.acc[e] = acc[e];
        run_program<DT, 1, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, NoStore{});
        stencil_store<DT>(a.out[0], (uint64_t)opos * g.c + cvi * VEC, ragged, cnt, S::pack(s.acc));
    }
}

}  // namespace pf
