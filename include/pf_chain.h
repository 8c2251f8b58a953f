/*
 * pf_chain.h -- C ABI of the fused-chain executor for AMD Instinct MI355X (gfx950).
 *
 * The library runs one already-isolated subgraph of memory-intensive operators (a "chain") as a single
 * HIP kernel: every input is read from HBM once, every output is written once, all intermediates live in
 * registers and LDS.  This is the run-time half of the method of arXiv 2307.04995: what its optimised
 * GIR-Graph does on the device after synchronisation insertion, gOperator merging and swapping have
 * removed the DRAM round trips between operators (sections 4 and 5.1).  The search and the code
 * generator of the paper are not part of this library; a chain is mapped onto one of a few hand-written
 * kernel families instead.
 *
 * All functions are thread-safe with respect to distinct plans.  No function throws or aborts; every
 * failure is a pf_status and a thread-local detail string (pf_last_error).  "Device pointer" always
 * means memory of the plan's device; "host pointer" means ordinary process memory.
 */
#ifndef PF_CHAIN_H
#define PF_CHAIN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PF_CHAIN_VERSION 1u
#define PF_MAX_RANK 6
#define PF_MAX_INPUTS 8
#define PF_MAX_OPS 32
#define PF_MAX_OUTPUTS 3

typedef enum {
    PF_OK = 0,
    PF_ERR_INVALID_ARG = 1, /* null pointer, bad struct_size/version, value id out of range, bad attribute */
    PF_ERR_SHAPE = 2,       /* shapes do not fit the operator (broadcast, parameter length, permutation)   */
    PF_ERR_DTYPE = 3,       /* unknown dtype, or a dtype mix the kernels do not implement                  */
    PF_ERR_UNSUPPORTED = 4, /* valid chain that fits no kernel family; there is no unfused fallback        */
    PF_ERR_ALIGNMENT = 5,   /* pointer not 16-byte aligned, or an extent that the family needs as a whole number
                               of 16-byte vectors (attention head dimension, tiled transposes)            */
    PF_ERR_ALIAS = 6,       /* an output overlaps an input in a family that cannot run in place            */
    PF_ERR_NOMEM = 7,       /* host or device allocation failed                                            */
    PF_ERR_HIP = 8,         /* a HIP runtime call failed; pf_last_error holds hipGetErrorString            */
    PF_STATUS_FORCE_INT32_ = 0x7fffffff /* (any non-negative int is a representable value: pf_status_str takes what it is given) */
} pf_status;

typedef enum { PF_F32 = 0, PF_F16 = 1, PF_BF16 = 2 } pf_dtype;

/*
 * The fixed operator set: the four basic operator kinds a memory-intensive subgraph is split into
 * (element-wise, broadcast, reduce, transpose: section 6, "GIR-Graph generation"), plus the usual
 * composites, which the library treats as one reduce-then-broadcast step.
 *
 * Element-wise binary operators take two values; if their shapes differ, one operand must have the result's
 * shape and the other is broadcast to it: the two shapes are aligned at the innermost dimension and every
 * extent of the smaller operand equals the other's or is 1 (a bias [D] or a mask [S, S] over leading dimensions,
 * an attention mask [B, 1, 1, S] under scores [B, H, S, S], a per-sample bias [N, 1, 1, C], one value per row
 * [..., 1]).  At most three separate runs of kept dimensions above the innermost one.  Operand order is kept
 * (SUB = src0 - src1, DIV = src0 / src1).  MAX, MIN and RELU return NaN when an operand is NaN.
 * All arithmetic is done in fp32 whatever the storage type; results are rounded to the output type once,
 * on the final store (round to nearest even).
 */
typedef enum {
    /* element-wise, two operands */
    PF_ADD = 0, PF_SUB = 1, PF_MUL = 2, PF_DIV = 3, PF_MAX = 4, PF_MIN = 5,
    /* element-wise, one operand */
    PF_SCALE = 6,       /* x * f[0]                                   */
    PF_ADDC = 7,        /* x + f[0]                                   */
    PF_NEG = 8,
    PF_RELU = 9,
    PF_SIGMOID = 10,    /* 1 / (1 + exp(-x))                          */
    PF_SILU = 11,       /* x * sigmoid(x)   (section 6: sigmoid, then multiply) */
    PF_GELU_ERF = 12,   /* x/2 * (1 + erf(x / sqrt 2))                */
    PF_TANH = 13,
    PF_EXP = 14,
    PF_RSQRT = 15,      /* 1 / sqrt(x)                                */
    PF_CAUSAL_MASK = 16,/* last two dims (i, j): j > i -> -inf, else x; the mask is implicit, never stored */
    /* reduce; the result keeps every reduced dimension with extent 1.  n_i = 0: over the last dimension.
       n_i >= 1: over the dimensions i[0] < i[1] < ...; implemented besides {last}: every dimension between the
       first and the last (global pooling of a channels-last tensor [n, spatial.., c] into [n, 1.., c])       */
    PF_REDUCE_SUM = 17, PF_REDUCE_MAX = 18, PF_REDUCE_MEAN = 19,
    /* reduce-then-broadcast composites over the last dimension */
    PF_SOFTMAX = 20,    /* exp(x - max) / sum exp(x - max); exp(-inf) = 0; an all -inf row gives NaN        */
    PF_LAYERNORM = 21,  /* src = x, gamma, beta; f[0] = eps; biased variance; (x-mu)/sqrt(var+eps)*g+b      */
    PF_RMSNORM = 22,    /* src = x, gamma;       f[0] = eps; x / sqrt(mean(x^2)+eps) * gamma                */
    PF_GROUPNORM = 23,  /* channels-last x [N, spatial.., C]; src = x, gamma, beta; i[0] = groups; f[0]=eps */
    /* layout */
    PF_PERMUTE = 24,    /* i[0..rank-1] = perm; output dim k is input dim perm[k].  A permutation that only moves
                           extents of 1 is lowered as a reshape; "move a dimension to the end -> LAYERNORM / RMSNORM
                           -> move it back" on chain inputs is one kernel without a layout change (column family) */
    PF_RESHAPE = 25,    /* i[0..n_i-1] = new shape with the same element count; contiguous data is
                           reinterpreted, nothing moves                                                     */
    /* one-token attention against cached keys and values (section 8, GPT-2 case study).  These three are
       accepted only in the arrangement  o = VECMAT(SOFTMAX([SCALE](MATVEC(K', q))), V')  with K' and V' either
       chain inputs or CONCAT_ROWS(cache, new row); outputs: o, and optionally K' and V'.                    */
    PF_CONCAT_ROWS = 26,/* src0 [..., t, d], src1 [..., d] -> [..., t+1, d]: src1 appended as the last row  */
    PF_MATVEC = 27,     /* src0 [..., t, d], src1 [..., d] -> [..., t]:   y_j = sum_c a_jc x_c              */
    PF_VECMAT = 28,     /* src0 [..., t],    src1 [..., t, d] -> [..., d]: y_c = sum_j p_j a_jc              */
    /* layout only (with PERMUTE and RESHAPE): chains made of nothing but these four move every element exactly
       once and are run as one index-map copy with any number of inputs (<= PF_MAX_INPUTS) and outputs          */
    PF_CONCAT = 29,     /* src0, src1 joined along axis i[0] (all other extents equal)                          */
    PF_SLICE = 30,      /* elements [i[1], i[1] + i[2]) of src0 along axis i[0]                                  */
    /* depthwise convolution (section 6, the EfficientNet fragment): src0 x [n, h, w, c] channels-last, src1
       kernels [kh, kw, c] (a chain input); cross-correlation, zero padding of kh/2 rows and kw/2 columns on every
       side; n_i = 0: stride 1 (h and w are kept); n_i = 1: stride i[0] (1 .. 8) along both axes, the result is
       [n, (h - 1) / stride + 1, (w - 1) / stride + 1, c].  Implemented for kh = kw = 3 and kh = kw = 5.  Element-wise
       operators may precede it (they run before the padding) and follow it (on the result's shape).           */
    PF_DWCONV2D = 31,
    PF_OP_COUNT_ = 32
} pf_op;

/* A contiguous row-major tensor. */
typedef struct {
    int32_t dtype; /* pf_dtype */
    int32_t rank;  /* 1..PF_MAX_RANK */
    int64_t shape[PF_MAX_RANK];
} pf_tensor_desc;

/*
 * One operator.  Value ids: 0..n_inputs-1 are the chain's inputs, n_inputs+k is the result of ops[k];
 * an operator may only use ids smaller than its own.
 */
typedef struct {
    int32_t op;     /* pf_op */
    int32_t n_src;  /* must equal the operator's arity */
    int32_t src[3];
    float f[2];
    int64_t i[PF_MAX_RANK];
    int32_t n_i;    /* number of meaningful entries of i (rank for PERMUTE / RESHAPE, 1 for GROUPNORM)      */
} pf_op_desc;

/*
 * The chain: plain data, owned by the caller, copied by pf_chain_plan.  struct_size must be
 * sizeof(pf_chain_desc) and version PF_CHAIN_VERSION.
 */
typedef struct {
    uint32_t struct_size, version;
    int32_t n_inputs;
    pf_tensor_desc inputs[PF_MAX_INPUTS];
    int32_t n_ops;
    pf_op_desc ops[PF_MAX_OPS];
    int32_t n_outputs;                   /* 1..PF_MAX_OUTPUTS */
    int32_t out_value[PF_MAX_OUTPUTS];   /* value id of each output (must be an operator result) */
    int32_t out_dtype[PF_MAX_OUTPUTS];   /* pf_dtype each output is stored in */
} pf_chain_desc;

/* Kernel family a plan was mapped to.  Families follow the widest synchronisation scope the chain needs
 * (section 5.1, synchronisation insertion: lane / parallel unit / block / device). */
typedef enum {
    PF_FAMILY_ELEMENTWISE = 0, /* lane scope only: values never leave their register                        */
    PF_FAMILY_ROW = 1,         /* row reduction then broadcast: wave shuffle, LDS when a row spans waves     */
    PF_FAMILY_GROUP = 2,       /* GroupNorm: a group spans workgroups, partial statistics cross the device   */
    PF_FAMILY_TRANSPOSE = 3,   /* layout change staged through an LDS tile                                   */
    PF_FAMILY_STENCIL = 6,     /* depthwise convolution: overlapping reads kept on chip in a register window         */
    PF_FAMILY_GATHER = 5,      /* layout-only chains (concat / slice / permute / reshape): a copy driven by a table
                                  of contiguous runs computed when the plan is made                          */
    PF_FAMILY_POOL = 7,        /* reduction over the positions of a channels-last tensor (global pooling): partial
                                  results per workgroup, merged by the last workgroup of a sample to arrive      */
    PF_FAMILY_COLUMN = 8,      /* layer / RMS normalisation over a dimension that is not the innermost (move it to the
                                  end, normalise, move it back: the two layout changes cancel): a workgroup keeps a slab
                                  [c, 64 positions] in registers, statistics cross lanes and waves, nothing is transposed */
    PF_FAMILY_ATTENTION = 4    /* one-token attention: a head's rows span workgroups, partial results are
                                  merged by the last workgroup to arrive                                     */
} pf_family;

typedef struct {
    int32_t family;   /* pf_family */
    int32_t variant;  /* family-specific: see the PF_VARIANT_* constants */
    uint32_t grid[3], block[3];
    uint32_t lds_bytes;
    uint64_t workspace_bytes;          /* device memory the plan owns */
    uint64_t compulsory_read_bytes;    /* every input once */
    uint64_t compulsory_write_bytes;   /* every output once */
    int32_t n_launches;                /* kernels enqueued per pf_chain_run */
    int32_t n_micro_ops;               /* element-wise steps the kernel executes per element */
    int32_t spec_id;                   /* 0: run-time interpreted kernel; 1..254: built-in catalogue entry;
                                          PF_SPEC_JIT: specialised for this chain when the plan was made      */
    int32_t vectors_per_lane;          /* 16-byte vectors each lane keeps in registers */
    int32_t n_kernels;                 /* 1, or the number of kernels a chain was split into (pf_chain_partition);
                                          family, variant, grid, block, spec_id and vectors_per_lane are then the
                                          first kernel's, workspace_bytes includes the tensors between kernels    */
    int32_t interpreter_fallback;      /* 1: a kernel specialised for this chain was wanted when the plan was made and
                                          could not be produced (kernel headers or run-time compiler missing, compile
                                          error): the run-time-interpreted kernels run instead, correct but several
                                          times slower.  pf_chain_plan still returns PF_OK; pf_last_error holds the
                                          reason right after it.  0 also when PF_JIT=0 asked for the interpreter.   */
} pf_plan_info;

/* A split of a chain into kernels: kernel k runs ops[first_op[k]] .. ops[first_op[k + 1] - 1]. */
typedef struct {
    int32_t n_parts;
    int32_t first_op[PF_MAX_OPS + 1];
    double predicted_us[PF_MAX_OPS]; /* the performance model's time for each kernel, microseconds */
    uint64_t bytes[PF_MAX_OPS];      /* bytes each kernel reads and writes                           */
} pf_partition;

#define PF_VARIANT_EW_FLAT 0          /* element-wise: one 16-byte vector per lane per step                  */
#define PF_SPEC_JIT 255               /* pf_plan_info.spec_id of a plan-time specialised kernel                */
#define PF_VARIANT_ATTN_ONE_PASS 0    /* attention family: a workgroup's slice of the cache in registers at once       */
#define PF_VARIANT_ATTN_STREAM 1      /* attention family: longer slices walked in chunks, next chunk's loads in flight */
#define PF_VARIANT_STENCIL_DIRECT 0   /* stencil family: a register window per lane, neighbours through the cache */
#define PF_VARIANT_STENCIL_STAGED 1   /* stencil family: the workgroup's tile is activated once and shared in LDS  */
#define PF_VARIANT_STENCIL_STRIDED 2  /* stencil family: strides above 1, taps loaded where they are used             */
#define PF_VARIANT_ROW_WAVE 0         /* row family: one 64-lane wave owns a row                             */
#define PF_VARIANT_ROW_BLOCK 1        /* row family: one workgroup owns a row                                */
#define PF_VARIANT_ROW_STREAM 2       /* row family: a workgroup walks a long row twice in chunks            */
#define PF_VARIANT_GROUP_TWO_PASS 0   /* group family: statistics pass, then normalise pass (re-reads x)     */
#define PF_VARIANT_GROUP_RESIDENT 1   /* group family: x held in registers across a device-scope exchange    */
#define PF_VARIANT_T_ROWS 0           /* transpose family: innermost dim kept, 16-byte vectors re-addressed  */
#define PF_VARIANT_T_LDS_ROWS 1       /* transpose family: innermost dim kept, LDS tile makes both sides long*/
#define PF_VARIANT_T_TILE 2           /* transpose family: innermost dim changes, square tiles, blocks of elements
                                         transposed in registers                                               */

/* Opaque plan object, owned by the library.  (Not called pf_chain_plan: in C a typedef and the function of that
 * name cannot coexist.) */
typedef struct pf_plan_s pf_plan;

/*
 * Check a chain description on the host (no GPU needed): structure, value ids, arities, attributes,
 * shape compatibility of every operator.  Returns PF_OK or the first problem found.
 * The rules are those of the four basic operator kinds the method splits a subgraph into (section 6, "GIR-Graph
 * generation": element-wise, broadcast, reduce, transpose) and of the composites built from them.
 */
pf_status pf_chain_validate(const pf_chain_desc *desc);

/*
 * Shape and (for inputs) dtype of any value of the chain (host only).  `value` is a value id.  For
 * operator results the dtype field is PF_F32, the type intermediates are computed in.  `out` is written
 * only on success.  (Section 6: every basic operator kind fixes the shape of its result from its operands' --
 * element-wise keeps it, broadcast extends it, reduce keeps reduced extents as 1, transpose permutes it.)
 */
pf_status pf_chain_infer_shape(const pf_chain_desc *desc, int32_t value, pf_tensor_desc *out);

/*
 * Rewrite sub-graphs of basic operators that spell out a composite operator over the last dimension into that
 * operator (host only).  The paper splits operators into the four basic kinds before it optimises (section 6);
 * a chain that arrives in that form gets the tuned kernel of the composite this way.  Recognised:
 *   exp(x - reduce_max x) / reduce_sum(exp(x - reduce_max x))                          -> softmax(x)
 *   ((h - reduce_mean h) * rsqrt(reduce_mean((h - mean)^2) + eps)) * gamma + beta      -> layernorm(h, gamma, beta)
 *   (x * rsqrt(reduce_mean(x * x) + eps)) * gamma                                      -> rmsnorm(x, gamma)
 * with multiplication and addition in either operand order, gamma and beta chain inputs of shape [n], and no
 * interior value used anywhere else.  `out` receives the rewritten chain (inputs and outputs unchanged, value
 * ids renumbered), or a copy of `desc` when nothing matched; *changed (may be null) says which.
 * pf_chain_plan applies the same rewrite by itself (and keeps the original chain when the rewritten one
 * cannot be planned); PF_RECOMPOSE=0 in the environment switches that off.
 */
pf_status pf_chain_recompose(const pf_chain_desc *desc, pf_chain_desc *out, int32_t *changed);

/*
 * Merge plan of a chain (host only; section 6, graph merging with a performance model).  One kernel holds one
 * exchange wider than a lane; a chain with several (a layout change, then a normalisation, then another layout
 * change; a normalisation followed by a pooling) runs as several kernels, and the element-wise operators between
 * two exchanges can go with either neighbour.  The model prices a kernel at a launch cost plus the bytes it reads
 * and writes over the rate its kernel family reaches; pf_chain_partition returns the split with the smallest
 * total, pf_chain_segment_cost the price of operators first_op .. last_op - 1 as one kernel (an error status when
 * they are not one kernel; us and bytes may be NULL).  Values that cross from one kernel to the next are stored in
 * fp32 whatever the storage type, so that a chain of several kernels still computes in fp32 from its first load to
 * its last store and rounds once: on 16-bit storage its inputs are widened and its outputs rounded by conversion
 * copies around the kernels, priced with the first and the last kernel.  pf_chain_plan applies the split by itself
 * when a chain is not one kernel (PF_PARTITION=0 in the environment: PF_ERR_UNSUPPORTED instead); such a plan owns
 * the tensors between its kernels, must not run on two streams at the same time, and returns PF_ERR_ALIAS when an
 * output overlaps an input.
 */
pf_status pf_chain_partition(const pf_chain_desc *desc, pf_partition *out);
pf_status pf_chain_segment_cost(const pf_chain_desc *desc, int32_t first_op, int32_t last_op, double *us, uint64_t *bytes);

/*
 * Map the chain onto a kernel family and fix launch geometry (section 6: the parallelism and tile size of
 * a GIR template are parameters chosen before code is produced; here they are chosen once per plan).
 * `device` is a HIP device ordinal.  May allocate plan-owned device workspace; launches no kernel.
 * On success *out is a new plan the caller must release with pf_chain_plan_destroy.
 * Limits of the kernels (PF_ERR_UNSUPPORTED beyond them): a chain outside the layout-only family reads at most 3
 * inputs of the full shape and 4 broadcast inputs, keeps at most 2 intermediate values alive besides the one being
 * computed (4 per-row values in chains with in-line reductions), runs at most 24 element-wise steps on either side
 * of its reduce / normalise / permute step, and holds one such step.
 * The environment variable PF_FORCE_VARIANT=<int> overrides the variant choice where that variant is
 * legal for the chain (for A/B measurements); PF_LOG=1 prints the decision to stderr.
 */
pf_status pf_chain_plan(const pf_chain_desc *desc, int32_t device, pf_plan **out);

/* Same as pf_chain_plan but with an explicit variant (-1 = choose automatically). */
pf_status pf_chain_plan_variant(const pf_chain_desc *desc, int32_t device, int32_t variant, pf_plan **out);

/*
 * What the planner decided: kernel family (the synchronisation scope of section 5.1 the chain needs), variant,
 * launch geometry, LDS and workspace sizes, the bytes the chain has to move (every input and output once: what is
 * left after the merging rules of section 5.1 have removed every DRAM round trip between operators), launches per
 * run.  `info` is written only on success; PF_ERR_INVALID_ARG for null arguments.
 */
pf_status pf_chain_plan_get_info(const pf_plan *plan, pf_plan_info *info);

/*
 * The split a plan runs with: one part for a chain that is one kernel, else the cut points pf_chain_plan settled
 * on (those of pf_chain_partition unless the device-side planning refused one of its segments and the search ran
 * again without it).  predicted_us and bytes are the model's figures for the parts.
 */
pf_status pf_chain_plan_get_partition(const pf_plan *plan, pf_partition *out);

/*
 * Run the chain: the device side of the optimised GIR-Graph (section 4: data-movement gOperators DRAM -> registers,
 * computation gOperators in registers, at most one synchronisation whose scope picked the kernel family, data movement
 * registers -> DRAM), launched with the parameters fixed when the plan was made (section 7, code generation).
 * Enqueue the fused kernel on `stream` (a hipStream_t, passed as void*; NULL = the default stream) and
 * return without waiting.  inputs[k] / outputs[k] are device pointers to contiguous tensors of exactly
 * the shapes and dtypes of the description, 16-byte aligned, owned by the caller and not retained.
 * No allocation, no host synchronisation, no host work proportional to tensor size.
 * An output may be the same buffer as an input of identical shape and dtype in the element-wise, row, group and
 * column families (each element is read before it is written, by the same lane or workgroup); the other families
 * return PF_ERR_ALIAS for any overlap.  A plan with workspace (group, attention, pool families) must not run on
 * two streams at the same time.
 * The launches may be recorded into a HIP graph (stream capture) and replayed, except those of the one-launch
 * GroupNorm variant (PF_ERR_UNSUPPORTED while the stream is capturing; plan PF_VARIANT_GROUP_TWO_PASS instead).
 */
pf_status pf_chain_run(const pf_plan *plan, const void *const *inputs, void *const *outputs, void *stream);

/*
 * Kernels that wait for other workgroups (the fused GroupNorm variant, the merging workgroup of a pooling, the merging
 * slice of a one-token attention head) bound every wait; when a wait runs
 * out they set an error word in the plan's workspace and carry on, so a launch always terminates.  This call
 * synchronises with the device (hipMemcpy), stores the word in *flag (0 = no wait gave up since the last poll)
 * and clears it.  A non-zero flag means that the outputs of the plan's launches since the last poll are invalid;
 * the call then also puts the plan's exchange words back into their initial state, so the caller must have
 * synchronised with every stream the plan ran on.  Plans without workspace always report 0.
 * Such waits end because the workgroups waited for are running: the grids are sized to what an otherwise idle
 * device holds at once.  A plan of the one-launch GroupNorm variant should therefore not share the device with other
 * long-running kernels (plan PF_VARIANT_GROUP_TWO_PASS where streams run concurrently).  The merging workgroups of
 * the pool and attention families wait only for workgroups dispatched before them, which wait for nobody: those waits
 * end whatever else runs.
 */
pf_status pf_chain_plan_poll_error(const pf_plan *plan, int32_t *flag);

/*
 * pf_chain_plan + pf_chain_run + pf_chain_plan_destroy in one call that allocates nothing on the device.  For
 * callers that cannot call hipMalloc where they run a chain: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  The device memory a chain's kernels need beyond its inputs and outputs (partial
 * GroupNorm statistics per workgroup; partial results and arrival counters of the one-token attention) comes from a
 * static device array of PF_STATIC_SCRATCH_BYTES that every device the library runs on holds until the process
 * ends.  A chain that needs more returns PF_ERR_NOMEM and nothing is launched.
 * Also refused, with PF_ERR_UNSUPPORTED (all of these need memory or code put on the device when a plan is made):
 * chains that run as several kernels, layout-only chains with CONCAT / SLICE, broadcast inputs with extents of 1
 * inside their shape, poolings split over several workgroups per sample.  Kernels are the library's built-in ones
 * (nothing is compiled: a chain outside the catalogue runs on the run-time-interpreted kernels), GroupNorm runs as
 * its two-launch variant, which waits for no other workgroup.
 * desc, inputs, outputs, stream: as for pf_chain_plan and pf_chain_run; `device` is made current for the call and the
 * caller's current device restored.  The parts of the array that must start at a value are rewritten by a small fill
 * kernel enqueued on `stream` ahead of the chain's kernels (no memset, so the launches can be recorded into a graph).
 * All calls on one device share the array: calls that overlap in time on one device (two streams, two threads)
 * race; order them on one stream or with events.
 */
#define PF_STATIC_SCRATCH_BYTES (2u << 20)
pf_status pf_chain_run_static(const pf_chain_desc *desc, int32_t device, const void *const *inputs, void *const *outputs, void *stream);

/*
 * Release a plan and the device memory it owns (workspace, tables, tensors between the kernels of a split chain).
 * The caller makes sure no launch of the plan is still running.  NULL is ignored.  (Section 6: a generated kernel
 * lives as long as the subgraph it was made for; here that lifetime is the caller's.)
 */
void pf_chain_plan_destroy(pf_plan *plan);

/*
 * Error reporting of the boundary: every entry point returns a pf_status; these turn it into text.  The paper's
 * system hands what it does not optimise to the vendor's DNN library (section 6, compute-bound operators); this
 * library has no such fallback, so a chain it cannot run as fused kernels is an explicit PF_ERR_UNSUPPORTED with the
 * reason here.
 * pf_status_str: the name of a status code (static storage).  pf_last_error: detail of the last failing call on the
 * calling thread (thread-local storage, valid until that thread's next failing call; empty string if none).
 */
const char *pf_status_str(pf_status s);
const char *pf_last_error(void);

/*
 * Measurement aid, not part of a chain: a plain 16-byte-per-lane device copy of `bytes` bytes
 * (multiple of 16) from src to dst on `stream`, used to calibrate achievable HBM bandwidth and the
 * hardware traffic counters against a transfer of known size.
 */
pf_status pf_copy_probe(const void *src, void *dst, uint64_t bytes, int32_t variant, void *stream);

/*
 * Diagnostic: how many kernels this process has specialised at plan time so far.  A chain whose structure
 * (operand counts, steps, core; not shapes or constants) is not in the built-in catalogue has the library's
 * kernel templates instantiated for it when its plan is made -- the counterpart of the paper's per-subgraph
 * code generation from GIR templates (section 6) -- and later plans of the same structure reuse the kernel.
 * PF_JIT=0 in the environment switches this off (such chains then run on the run-time-interpreted kernels).
 */
uint64_t pf_jit_compile_count(void);

/*
 * Diagnostic: how many of this process's plan-time kernels came from disk instead of the compiler.  With
 * PF_JIT_CACHE=<directory> in the environment (the directory must exist and be writable; off by default) every kernel
 * compiled at plan time is also kept there, and a later process that plans the same chain loads it instead of
 * compiling it (a plan then takes milliseconds rather than seconds).  A file's name is a digest of everything its code
 * depends on (generated source, template-id, compiler options and version, the contents of the kernel headers), so a
 * new build of the library never picks up an old kernel; a file that does not load is compiled over.  For callers that
 * start often (section 7 of the paper compiles per model as well, ahead of time).
 */
uint64_t pf_jit_cache_hits(void);

#ifdef __cplusplus
}
#endif
#endif /* PF_CHAIN_H */
