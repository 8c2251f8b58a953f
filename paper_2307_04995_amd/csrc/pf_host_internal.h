// Declarations shared by the host-side translation units of the fused-chain library: description checking
// (pf_check.cpp), recomposition of basic operators (pf_recompose.cpp), lowering to micro-programs (pf_lower.cpp),
// kernel-family planning (pf_plan.cpp) and the C ABI with the launch path (pf_host.cpp).
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "../../include/pf_chain.h"
#include "pf_common.h"
#include "pf_jit.h"
#include "pf_launch.h"

namespace pfh {

// ---- errors: the message is kept per thread for pf_last_error ----
pf_status fail(pf_status s, const char* fmt, ...);
const char* last_error();

// ---- operator table and shapes ----
enum OpClass { OC_BINARY, OC_UNARY, OC_MASK, OC_REDUCE, OC_SOFTMAX, OC_LAYERNORM, OC_RMSNORM, OC_GROUPNORM, OC_PERMUTE, OC_RESHAPE,
               OC_CONCAT_ROWS, OC_MATVEC, OC_VECMAT, OC_CONCAT, OC_SLICE, OC_DWCONV };

struct OpTraits {
    OpClass cls;
    int arity;
    const char* name;
};

extern const OpTraits kOps[PF_OP_COUNT_];

inline bool is_elementwise(OpClass c) { return c == OC_BINARY || c == OC_UNARY || c == OC_MASK; }

typedef std::vector<int64_t> Shape;

int64_t numel(const Shape& s);
bool is_trailing(const Shape& small_in, const Shape& big);
bool is_row_value_of(const Shape& small, const Shape& big);
bool broadcasts_onto(const Shape& small, const Shape& big);
inline int dtype_size(int dt) { return dt == PF_F32 ? 4 : 2; }

// A REDUCE_* operator with integer attributes names the dimensions it reduces; without, or with just the last
// dimension, it is the row reduction.
inline bool reduces_other_dims(const pf_op_desc& o, size_t rank) { return o.n_i > 1 || (o.n_i == 1 && o.i[0] != (int64_t)rank - 1); }

struct Checked {
    std::vector<Shape> shape;  // per value id
};

// Full structural and shape check of a chain description; fills the shape of every value.
pf_status check_desc(const pf_chain_desc* d, Checked* out);

// Rewrites sub-graphs of basic operators that spell a softmax, a layer normalisation or an RMS normalisation over the
// last dimension into that operator.  Returns false (out untouched or partial) when nothing matched.
bool recompose_chain(const pf_chain_desc* d, const Checked& c, pf_chain_desc* out);

// ---- lowering ----
struct Lowered {
    int main_dtype = PF_F32;
    int core_op = -1;         // index into desc->ops, -1 = none
    int pool_op = 0;          // CORE_POOL: 0 sum, 1 maximum, 2 mean
    int core = pf::CORE_NONE;
    float eps = 0.0f;
    int n_full = 0, n_vec = 0, n_tmp = 0;
    int full_input[PF_DEV_MAX_FULL];  // chain input index per full slot
    bool full_is_epi[PF_DEV_MAX_FULL];
    int vec_input[PF_DEV_MAX_VEC];
    bool vec_is_epi[PF_DEV_MAX_VEC];
    bool general_bcast = false;         // some broadcast input needs the general (term-based) addressing
    bool scalar_vec = false;            // some broadcast input has a single element
    Shape vec_partner[PF_DEV_MAX_VEC];  // shape of the value the operand is broadcast against (where it is first used)
    int core_vec[2] = {-1, -1};
    pf::Program pro, epi;
    uint32_t mask_si = 0;     // load skipping allowed for a causal mask of this extent
    uint32_t core_mask = 0;   // the mask is applied inside the softmax core
    float core_scale = 1.0f;  // scale folded into the softmax core
    int out_slot_to_user[PF_MAX_OUTPUTS];  // args.out[slot] <- user outputs[...]
    int n_out = 1;
    Shape pre_shape;          // shape of the value entering the core (or the final value if no core)
    Shape post_shape;         // shape of the value leaving the core
    int64_t groups = 0;
    int perm[PF_MAX_RANK];
    // one-token attention: chain input index of q, new key row, new value row, key cache, value cache (-1: the
    // caches already hold the new rows); user output index of o, grown key cache, grown value cache (-1: not an output)
    int attn_in[5] = {-1, -1, -1, -1, -1};
    int attn_out[3] = {-1, -1, -1};
    float attn_scale = 1.0f;
    // column family: chain input index of x, gamma, beta (-1: RMS normalisation); [outer, c, s] view of x
    int col_in[3] = {-1, -1, -1};
    int64_t col_outer = 0, col_c = 0, col_s = 0;
};

// Lowers a checked chain: prologue and epilogue micro-programs around at most one core, operand slots, output slots.
pf_status lower_chain(const pf_chain_desc* d, const Checked& c, Lowered* L);

}  // namespace pfh

// ---------------------------------------------------------------------------------------------
// the plan
// ---------------------------------------------------------------------------------------------
struct pf_plan_s {
    pf_chain_desc desc;
    pfh::Lowered low;
    int device = 0;
    int family = 0, variant = 0;
    int spec_id = 0;          // 0 = generic interpreter
    int k = 1;                // 16-byte vectors per lane
    bool reduce_only = false;
    hipFunction_t jit_fn2 = nullptr; // second launch of a two-launch plan
    hipFunction_t jit_fn = nullptr;  // kernel specialised for this chain's structure when the plan was made (spec_id == kSpecJit)
    bool ragged = false;      // rows or broadcast operands that are not whole 16-byte vectors: element-granular kernels
    pf::ChainArgs args;       // pointers are filled per run
    pf::RowGeom row;
    pf::GroupGeom group;
    pf::PermGeom permg;
    pf::AttnArgs attn;
    pf::GatherArgs gather;
    pf::StencilGeom stencil;
    pf::PoolGeom pool;
    pf::ColArgs col;
    int stencil_ks = 3;       // kernel extent of the depthwise convolution
    int row_log2l = 6;        // row family: log2 of the lanes of a wave that share a row
    pf::BcastTerm bcast_host[PF_DEV_MAX_VEC][PF_DEV_MAX_BCAST_TERMS];  // general broadcasting terms, staged on the host
    void* bcast_dev = nullptr;  // ... and their copy in device memory
    bool group_general = false; // group family: groups of any width (general kernels)
    bool interpreter_fallback = false;  // a specialised kernel was wanted and could not be produced: the interpreter runs
    std::string fallback_reason;
    uint32_t dyn_lds = 0;     // group family: dynamic LDS bytes of each launch
    uint32_t ew_total_vecs = 0, ew_vecs_per_row = 0;
    dim3 grid, block;
    dim3 grid2, block2;       // second launch (two-pass group variant)
    uint32_t lds_bytes = 0;
    void* workspace = nullptr;
    bool workspace_borrowed = false;  // the workspace lies in the library's static scratch array: nothing to free
    struct Fill {                     // ... and these parts of it must hold `byte` when the kernels start
        void* ptr;
        uint64_t bytes;
        int byte;
    };
    std::vector<Fill> fills;
    uint32_t* ws_error = nullptr;  // device word a kernel sets when one of its bounded waits ran out
    uint64_t workspace_bytes = 0;
    uint64_t in_bytes[PF_MAX_INPUTS];
    uint64_t out_bytes[PF_MAX_OUTPUTS];
    pfh::Shape out_shape[PF_MAX_OUTPUTS];
    int n_launches = 1;
    mutable uint32_t epoch = 0;
    // a chain split into several kernels: one plan per kernel, run in order on the caller's stream
    struct Part {
        pf_plan_s* plan = nullptr;
        int n_in = 0, n_out = 0;
        int in_kind[PF_MAX_INPUTS], in_index[PF_MAX_INPUTS];     // kind 0: the caller's input, 1: the caller's output, 2: tensor in the arena
        int out_kind[PF_MAX_OUTPUTS], out_index[PF_MAX_OUTPUTS];
    };
    // a chain of several kernels on 16-bit storage runs in fp32 between its first load and its last store: inputs are
    // widened into the arena before the first kernel, outputs rounded from the arena after the last
    struct Cast {
        int user = 0;          // index of the caller's input / output
        int slot = 0;          // index into arena_offset
        uint64_t numel = 0;
    };
    std::vector<Cast> widen_in, round_out;
    int storage_dtype = PF_F32;
    bool composite = false;
    std::vector<Part> parts;
    pf_partition partition;               // the cut points in use (composite plans)
    void* arena = nullptr;                // tensors that cross from one kernel to the next
    uint64_t arena_bytes = 0;
    std::vector<uint64_t> arena_offset;
};

namespace pfh {

// ---- planning ----
int env_int(const char* name, int dflt);
void note_interpreter_fallback(pf_plan_s* p, const std::string& why);

// Where a plan's device memory comes from.  Ordinary plans allocate it.  While pf_chain_run_static plans (tls_scratch is
// set on that thread) it is carved out of the library's static scratch array instead, nothing is allocated, compiled
// or uploaded, and whatever must start at a given value is recorded in the plan (pf_plan_s::fills) for a fill kernel
// on the caller's stream.
struct ScratchArena {
    char* base;
    uint64_t cap, used;
};
extern thread_local ScratchArena* tls_scratch;
inline bool planning_static() { return tls_scratch != nullptr; }
// `bytes` of device memory for the plan's workspace (p->workspace, p->workspace_bytes); the device must be current.
pf_status plan_workspace_alloc(pf_plan_s* p, uint64_t bytes, const char* what);
// Sets `bytes` bytes at `ptr` to `byte`.  must_hold: the kernels rely on the value (flags, counters, error words);
// otherwise the clear is hygiene and a plan on the static scratch array skips it.
pf_status plan_workspace_fill(pf_plan_s* p, void* ptr, int byte, uint64_t bytes, bool must_hold);
pf::FastDiv make_fastdiv(uint32_t d);
// Checks, lowers and plans one description as it stands (no recomposition).
pf_status plan_checked_desc(const pf_chain_desc* desc, int32_t device, int32_t variant, pf_plan** out);
// One kernel for the whole chain: as its composite operators when it spells them in basic operators, else as written.
pf_status plan_one_kernel(const pf_chain_desc* desc, int32_t device, int32_t variant, pf_plan** out);

// ---- chains of several kernels (pf_partition.cpp) ----
// Modelled time and bytes of operators [first, last) run as one kernel; an error status when they are not one kernel.
pf_status segment_cost(const pf_chain_desc* d, int first, int last, double* us, uint64_t* bytes);
// The cheapest split under the model that uses no segment of `blocked`.
pf_status partition_chain(const pf_chain_desc* d, const Checked& c, const std::vector<std::pair<int, int>>& blocked, pf_partition* out);
// A plan of several kernels for a chain that is not one kernel.
pf_status plan_partitioned(const pf_chain_desc* d, int32_t device, pf_plan** out);

}  // namespace pfh
