// Stencil family: prologue -> depthwise 3 x 3 convolution (channels-last, stride 1, zero "same" padding) ->
// epilogue, one kernel.
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

constexpr int kStencilRows = 6;  // output rows per strip (8 input rows are read for them)

template <int DT, class Spec>
__global__ void __launch_bounds__(256) dwconv3x3_kernel(const ChainArgs a, const StencilGeom g) {
    using S = Storage<DT>;
    constexpr int VEC = S::VEC;
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;  // (column, channel vector) of this lane, channel fastest
    if (t >= g.row_vecs) return;
    const uint32_t wcol = fast_div(t, g.div_cv);
    const uint32_t cvi = t - wcol * g.cv;
    const uint32_t sample = blockIdx.z;
    const uint32_t h0 = blockIdx.y * (uint32_t)kStencilRows;
    const int wslot = Spec::gamma(a);  // broadcast slot that holds the kernels [3, 3, channels]

    // the nine kernel vectors of this lane's channels, kept packed
    u32x4 wraw[9];
#pragma unroll
    for (int k = 0; k < 9; ++k)
        wraw[k] = load_cached(a.vec[wslot].ptr, ((uint64_t)k * g.c + cvi * VEC) * S::ESIZE);

    LaneState<DT, 1, Spec> s;
    s.col[0] = cvi * VEC;
    // operands of one position: prologue side (is_epi = false) or epilogue side
    auto load_operands = [&](uint32_t pos, bool is_epi) {
        s.row[0] = pos;
        const uint32_t fmask = is_epi ? g.epi_full_mask : ~g.epi_full_mask;
        const uint32_t vmask = is_epi ? g.epi_vec_mask : ~g.epi_vec_mask;
#pragma unroll
        for (int f = 0; f < Spec::NF; ++f)
            if (f < Spec::n_full(a) && ((fmask >> f) & 1u))
                s.fraw[f][0] = load_cached(a.full[f], ((uint64_t)pos * g.c + cvi * VEC) * S::ESIZE);
#pragma unroll
        for (int v = 0; v < Spec::NV; ++v)
            if (v < Spec::n_vec(a) && v != wslot && ((vmask >> v) & 1u))
                s.vraw[v][0] = load_vec_operand<DT>(a.vec[v], pos, s.col[0], g.c);
    };

    float win[3][3][VEC];  // activated values: window row (input row mod 3), column offset -1 / 0 / +1
    // bring input row r (may lie outside the image) into its window row
    auto load_row = [&](int r, int slot) {
#pragma unroll
        for (int dw = 0; dw < 3; ++dw) {
            const int col = (int)wcol + dw - 1;
            const bool inside = r >= 0 && r < (int)g.h && col >= 0 && col < (int)g.w;
            if (inside) {
                load_operands((sample * g.h + (uint32_t)r) * g.w + (uint32_t)col, false);
                run_program<DT, 1, Spec>(ProgView<typename Spec::Pro>{a.pro}, s, NoStore{});
            }
#pragma unroll
            for (int e = 0; e < VEC; ++e) win[slot][dw][e] = inside ? s.acc[e] : 0.0f;
        }
    };

    load_row((int)h0 - 1, 2);  // input row h0 - 1 sits in slot (h0 - 1 + 3) mod 3 relative to h0: see below
    load_row((int)h0, 0);
    // relative numbering: input row h0 + k lives in slot k mod 3 (k = -1 -> slot 2)
#pragma unroll
    for (int i = 0; i < kStencilRows; ++i) {
        const uint32_t row = h0 + (uint32_t)i;
        if (row >= g.h) break;
        load_row((int)row + 1, (i + 1) % 3);
        float acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;
#pragma unroll
        for (int dh = 0; dh < 3; ++dh) {
            const int slot = (i + dh + 2) % 3;  // input row row + dh - 1 = h0 + (i + dh - 1)
#pragma unroll
            for (int dw = 0; dw < 3; ++dw) {
                float wf[VEC];
                S::unpack(wraw[dh * 3 + dw], wf);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = __builtin_fmaf(wf[e], win[slot][dw][e], acc[e]);
            }
        }
        const uint32_t pos = (sample * g.h + row) * g.w + wcol;
        load_operands(pos, true);
#pragma unroll
        for (int e = 0; e < VEC; ++e) s.acc[e] = acc[e];
        run_program<DT, 1, Spec>(ProgView<typename Spec::Epi>{a.epi}, s, NoStore{});
        store_stream(a.out[0], ((uint64_t)pos * g.c + cvi * VEC) * S::ESIZE, S::pack(s.acc));
    }
}

}  // namespace pf
