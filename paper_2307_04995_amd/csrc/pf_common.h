// Structures shared by the host planner and the device kernels of the fused-chain library.
//
// A planned chain reaches the device as
//   * up to PF_DEV_MAX_FULL "full" operands: tensors with the shape of the value being computed, each read
//     from HBM exactly once as 16-byte vectors (the DRAM -> register data-movement step of the chain);
//   * up to PF_DEV_MAX_VEC "vec" operands: lower-rank tensors broadcast over the leading dimensions
//     (bias, gamma, beta); they are a few KB and served from cache after first touch;
//   * two micro-programs (prologue, epilogue) of element-wise steps on an accumulator held in registers;
//   * one core step between them (nothing, a row reduction + broadcast, a group normalisation, a
//     permutation).
// The micro-programs are what is left of the chain's element-wise operators after the planner has applied
// by hand the two merging rules of the paper (section 5.1): every write-then-read pair between operators
// collapsed into a register, every repeated read of an input served by the same load.
#pragma once
#ifndef __HIPCC_RTC__
#include <stdint.h>
#else  // the run-time compiler has no C library headers
typedef unsigned char uint8_t;
typedef unsigned short uint16_t;
typedef unsigned int uint32_t;
typedef int int32_t;
typedef unsigned long uint64_t;
typedef long int64_t;
#endif

#define PF_DEV_MAX_FULL 3
#define PF_DEV_MAX_VEC 4
#define PF_DEV_MAX_UOPS 24
#define PF_DEV_MAX_TMP 2
#define PF_DEV_MAX_ROWV 4
#define PF_DEV_MAX_OUT 2
#define PF_DEV_MAX_RANK 6

namespace pf {

// micro-op codes: acc = f(acc, operand) unless noted
enum UopCode : uint8_t {
    U_MOV = 0,     // acc = operand
    U_ADD, U_SUB,  // acc - operand
    U_RSUB,        // operand - acc
    U_MUL, U_DIV,  // acc / operand
    U_RDIV,        // operand / acc
    U_MAX, U_MIN,
    U_NEG, U_RELU, U_SIGMOID, U_SILU, U_GELU_ERF, U_TANH, U_EXP, U_RSQRT,
    U_MASK_CAUSAL, // acc = (col > row % ival) ? -inf : acc ; ival = extent of the second-to-last dim
    U_SAVE,        // tmp[slot] = acc
    U_STORE,       // write acc to output[slot] at the current position (secondary outputs)
    U_RED_SUM,     // rowv[slot] = sum over the row of acc      (row programs: reductions inside the step list; the
    U_RED_MAX,     // rowv[slot] = max over the row of acc       accumulator is left as it is)
    U_RED_MEAN,    // rowv[slot] = mean over the row of acc
    U_COUNT_
};

// K_ROW: a per-row value (the result of a U_RED_* step), the same for every element of the row
enum OperandKind : uint8_t { K_NONE = 0, K_IMM = 1, K_FULL = 2, K_VEC = 3, K_TMP = 4, K_ROW = 5 };

struct Uop {
    uint8_t code;  // UopCode
    uint8_t kind;  // OperandKind
    uint8_t slot;  // full / vec / tmp / output slot
    uint8_t pad;
    union {
        float imm;
        int32_t ival;
    };
};

struct Program {
    int32_t n;
    Uop u[PF_DEV_MAX_UOPS];
};

enum DType : int32_t { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2 };

// Division of a 32-bit index by a run-time constant without a divide instruction: q = n / d for every
// 32-bit n (multiply-high, one correction add, two shifts).  Built on the host by make_fastdiv().
struct FastDiv {
    uint32_t m, s1, s2, d;
};

// A broadcast operand with `numel` elements laid over a value whose innermost extent is n_inner:
//   numel >= n_inner (numel = m * n_inner): element (row, col) reads vec[(row % m) * n_inner + col]
//   numel <  n_inner (n_inner % numel == 0): reads vec[col % numel]; numel == 1 is a scalar.
// General broadcasting (operand dimensions of extent 1 anywhere, numpy style): the operand's row for row r of
// the value is sum_k ((r / div_k) mod mod_k) * stride_k over n_terms terms, one per run of kept dimensions.
#define PF_DEV_MAX_BCAST_TERMS 3
struct BcastTerm {
    FastDiv div, mod;  // mod.d is the modulus
    uint32_t stride;   // in operand rows
    uint32_t pad[3];
};

struct VecArg {
    const void* ptr;
    uint32_t numel;
    uint32_t period_rows;  // m above (1 when numel <= n_inner)
    int32_t dtype;         // DType of the storage; may differ from the chain's main dtype only as f32
    uint32_t n_terms;      // > 0: general broadcasting, described by terms[0 .. n_terms)
    uint32_t col_bcast;    // general broadcasting: the operand's innermost extent is 1 (one value per operand row)
    uint32_t pad;
    const BcastTerm* terms;  // device memory owned by the plan (kept out of the kernel arguments, which every launch copies)
};

enum CoreKind : int32_t {
    CORE_NONE = 0,
    CORE_SOFTMAX = 1,
    CORE_LAYERNORM = 2,
    CORE_RMSNORM = 3,
    CORE_REDUCE_SUM = 4,
    CORE_REDUCE_MAX = 5,
    CORE_REDUCE_MEAN = 6,
    CORE_GROUPNORM = 7,
    CORE_PERMUTE = 8,
    CORE_COLNORM = 14,      // layer / RMS normalisation over a dimension that is not the innermost (column family)
    CORE_POOL = 13,         // reduction over the positions of a channels-last tensor (pool family)
    CORE_DWCONV = 12,       // depthwise convolution (stencil family); core_vec[0] = slot of the kernels
    CORE_GATHER = 11,       // layout-only chain with concatenations / slices
    CORE_ATTN_DECODE = 10,  // concat -> matrix-vector -> softmax -> concat -> vector-matrix (one-token attention)
    CORE_ROWPROG = 9   // no fixed core: the prologue itself holds row reductions (U_RED_*) and their broadcasts
};

// Arguments common to all families.
struct ChainArgs {
    const void* full[PF_DEV_MAX_FULL];
    VecArg vec[PF_DEV_MAX_VEC];
    void* out[PF_DEV_MAX_OUT];
    int32_t n_full, n_vec;
    int32_t core;            // CoreKind
    int32_t core_vec[2];     // vec slots of gamma / beta (-1 = absent)
    float eps;
    uint32_t n_inner;        // innermost extent (elements) of the value the programs run on
    uint32_t mask_si;        // > 0: the prologue masks columns > row % mask_si and loads may skip them
    uint32_t raw_copy;       // 1: the chain only moves data; kernels forward the raw bits unconverted
    float core_scale;        // softmax: the input is multiplied by this (> 0) inside the core (folded SCALE step)
    uint32_t core_mask;      // softmax: the causal mask (extent mask_si) is applied inside the core; 1 = element by
                             // element, 2 = skipped vectors read as -inf and only the diagonal vector is masked
    uint32_t vec_plain_all;  // 1: every broadcast operand is one vector of n_inner elements, indexed by column alone
    FastDiv mask_div;        // division by mask_si
    uint64_t rows;           // number of rows (product of the other extents)
    Program pro, epi;
};

// Row family geometry.
struct RowGeom {
    uint32_t waves_per_row;  // 1 = a wave owns a row; > 1 = a workgroup of that many waves owns a row
    uint32_t rows_per_block; // row slots per workgroup (a slot is rows_per_wave rows when a wave owns its rows)
    uint32_t rows_per_wave;  // rows each wave processes at once (1 unless a wave owns its rows)
};

// Group family (channels-last GroupNorm) geometry.
struct GroupGeom {
    uint32_t samples, hw, channels, groups;
    uint32_t cv;                 // 16-byte vectors per position (channels / VEC)
    uint32_t vpg;                // vectors per group (power of two)
    uint32_t log2_vpg;
    uint32_t pos_per_step;       // positions a workgroup covers per step (blockDim / cv)
    uint32_t pos_per_block;      // positions one workgroup owns (a tile)
    uint32_t lanes_per_group;    // lanes that share a group when a sample's partials are merged (power of two)
    uint32_t vec_per_channel;    // 1: every broadcast operand is indexed by channel only
    uint32_t blocks_per_sample;
    float* ws_partial;           // two-launch variant: [samples][blocks_per_sample][groups][4] = (count, mean, M2, -)
    uint64_t* ws_gather;         // resident variant: [2][samples][groups][blocks_per_sample] (mean, M2) words per launch
                                 // parity; all-ones = not written yet
    uint32_t epoch;              // launch number (its parity selects the half of ws_gather in use)
    uint32_t spin_limit;         // resident variant: bounded wait, then the error flag is raised
    uint32_t* ws_error;          // resident variant: set to 1 if a wait ran out
    FastDiv div_cv;
    // groups of any width (GEN kernels): channels per group, its divider, and the most groups one vector touches
    uint32_t cpg, parts;
    FastDiv div_cpg;
    uint32_t ragged;             // 1: channels is not a whole number of 16-byte vectors (general kernels only): positions
                                 // are not vector-aligned and the last vector of each is partial
};

// Pool family (reduction over the positions of a channels-last tensor) geometry.
struct PoolGeom {
    uint32_t samples, hw, channels;
    uint32_t cv;                 // 16-byte vectors per position (channels / VEC)
    uint32_t pos_per_step;       // positions a workgroup covers per step (512 / cv)
    uint32_t pos_per_block;      // positions one workgroup owns
    uint32_t blocks_per_sample;
    uint32_t chunks;             // chunks (of NV position steps) a workgroup walks
    uint32_t epi_full_mask, epi_vec_mask;  // operands that belong to the epilogue (read in the result's layout)
    float inv_hw;                // 1 / positions (mean)
    uint32_t* ws_partial;        // [samples][blocks_per_sample][channels] partial results as words, all-ones = not published
                                 // (more than one block per sample; the merger puts them back to all-ones)
    uint32_t* ws_error;          // set to 1 if a wait ran out
    uint32_t spin_limit;         // re-reads before a wait gives up
    uint32_t merge_rows;         // row groups of threads the merger splits the slices over (512 / channels, at least 1)
    uint32_t ragged;             // the channel count is not a whole number of vectors (cv rounds up; RAGGED kernels)
    FastDiv div_cv;
};

// Column family: normalisation of [outer, c, s] over c (s contiguous); all tensors of one storage type.
struct ColArgs {
    const void* x;
    void* out;
    const void* gamma;        // [c]
    const void* beta;         // [c], or null (RMS normalisation)
    uint32_t c, s;            // normalised extent; elements after it
    uint32_t s_vecs;          // s in 16-byte vectors
    uint32_t tiles_per_outer; // workgroups per outer index: ceil(s_vecs / 8)
    float inv_c, eps;
};

// Attention family (one new token against cached keys and values); all tensors of one storage type.
struct AttnArgs {
    const void* q;        // [heads, d]
    const void* k_new;    // [heads, d] row appended to the keys, or null when the cache already holds it
    const void* v_new;
    const void* k_cache;  // [heads, t, d]
    const void* v_cache;
    void* o;              // [heads, d]
    void* k_out;          // [heads, t_total, d] grown caches, or null when they are not outputs
    void* v_out;
    float* ws_partial;    // [heads][splits][part_stride]: weighted value sum (d), maximum, sum of exponentials
    uint32_t* ws_counter; // [heads] arrivals of the current launch (re-armed by the last arrival)
    uint32_t t, t_total;  // cached rows; rows after the concatenation (t or t + 1)
    uint32_t d;           // head dimension (elements), at most 256
    uint32_t lanes_per_row, log2_lpr;
    float scale;
    uint32_t chunks;      // streaming variant: chunks (of NV steps of 256 / lanes_per_row rows) a workgroup walks
    uint32_t part_stride; // floats between the partial results of two slices: d + 2 rounded up to whole 128-byte lines, so
                          // that no two workgroups publish (device-coherent stores) into one memory line
    // Polled merge (plans that own a workspace; 0 / null = the counted, wait-free merge): the partial results are
    // published as self-describing words (all-ones = not written in this launch) and the head's last slice waits for them.
    uint32_t polled;
    uint32_t spin_limit;  // re-reads before the wait gives up
    uint32_t* ws_error;   // set to 1 if it did
};

// Stencil family (depthwise 3 x 3 convolution on a channels-last tensor) geometry.
struct StencilGeom {
    uint32_t n, h, w, c;
    uint32_t cv;        // 16-byte vectors per position (c / VEC)
    uint32_t row_vecs;  // w * cv: lanes needed for one image row
    uint32_t epi_full_mask, epi_vec_mask;  // operands that belong to the epilogue (read at the output position)
    uint32_t tiles_x, tiles_y, tiles;      // staged variant: tiles per image row, strips per image, tiles in all
    uint32_t tiles_per_die;                // ceil(tiles / 8)
    FastDiv div_cv;
    uint32_t stride, oh, ow, out_row_vecs; // strided variant: stride along both axes, output extents, ow * cv
    uint32_t strip_rows;                   // strided variant: output rows per workgroup
    uint32_t ragged;                       // 1: c is not a whole number of 16-byte vectors (cv counts the partial one)
};

// Gather family: layout-only chains as a copy of contiguous runs.  Run k of the table moves run_elems elements
// from input src_id at element src_off to output dst_id at element dst_off.
struct GatherRun {
    uint32_t src_off, dst_off;
    uint8_t src_id, dst_id;
    uint16_t pad;
};
struct GatherArgs {
    const void* in[8];
    void* out[3];
    const GatherRun* table;
    uint32_t n_runs, run_elems, vec_per_run;
    FastDiv div_vpr;
};

// Transpose family geometry.  The iteration space lists the merged dims from outermost to innermost in
// the order of the side that is walked contiguously; both sides' strides are given per iteration dim.
struct PermGeom {
    int32_t rank;                               // iteration dims used (<= PF_DEV_MAX_RANK)
    uint32_t extent[PF_DEV_MAX_RANK];           // extents, innermost counted in 16-byte vectors
    uint32_t in_stride[PF_DEV_MAX_RANK];        // input stride in elements of each iteration dim
    uint32_t out_stride[PF_DEV_MAX_RANK];       // output stride in elements
    FastDiv div[PF_DEV_MAX_RANK];
    uint32_t in_n_inner, out_n_inner;           // innermost extents (elements) of the two layouts
    FastDiv div_in_inner, div_out_inner;
    uint32_t total_vecs;
    uint32_t epi_full_mask, epi_vec_mask;       // operands addressed in the output layout
    // LDS-staged variant (innermost dim kept): a workgroup moves a [tile_a x tile_b] block of inner rows.
    // Tile variant (innermost dim changes): tile_a / tile_b = extents of the input's / output's innermost dim.
    uint32_t tile_a, tile_b;
    uint32_t lds_pitch;       // LDS-staged variant: pitch of a staged line in 16-byte vectors
    uint32_t t_in_stride_o;   // tile variant: input stride (elements) of the output's innermost dim
    uint32_t t_out_stride_i;  // tile variant: output stride (elements) of the input's innermost dim
};

}  // namespace pf
