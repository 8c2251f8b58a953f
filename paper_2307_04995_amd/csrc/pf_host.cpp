// Host side of the fused-chain library: description checking, shape inference, lowering of a chain to
// micro-programs, kernel-family choice, launch geometry, and the C ABI of include/pf_chain.h.
//
// Lowering applies, once and by hand, what the paper's rewriting does on a merged GIR-Graph (section 5):
//   * every value produced by one element-wise operator and consumed by the next stays in a register
//     (write-then-read merging; lane-scope synchronisation is a no-op);
//   * an input used by several operators is loaded once (read-after-read merging);
//   * element-wise operators are moved across the layout change so they run where the data already is
//     (gOperator swapping): the prologue of a permutation runs on the input layout, its epilogue on the
//     output layout;
//   * the one remaining exchange (row reduction, group statistics, tile transpose) decides the kernel
//     family by its synchronisation scope.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/pf_chain.h"
#include "pf_common.h"
#include "pf_jit.h"
#include "pf_launch.h"
#include "pf_specs.h"

namespace {

thread_local std::string g_last_error;

pf_status fail(pf_status s, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return s;
}

enum OpClass { OC_BINARY, OC_UNARY, OC_MASK, OC_REDUCE, OC_SOFTMAX, OC_LAYERNORM, OC_RMSNORM, OC_GROUPNORM, OC_PERMUTE, OC_RESHAPE,
               OC_CONCAT_ROWS, OC_MATVEC, OC_VECMAT, OC_CONCAT, OC_SLICE, OC_DWCONV };

struct OpTraits {
    OpClass cls;
    int arity;
    const char* name;
};

const OpTraits kOps[PF_OP_COUNT_] = {
    {OC_BINARY, 2, "add"},      {OC_BINARY, 2, "sub"},      {OC_BINARY, 2, "mul"},      {OC_BINARY, 2, "div"},
    {OC_BINARY, 2, "max"},      {OC_BINARY, 2, "min"},      {OC_UNARY, 1, "scale"},     {OC_UNARY, 1, "addc"},
    {OC_UNARY, 1, "neg"},       {OC_UNARY, 1, "relu"},      {OC_UNARY, 1, "sigmoid"},   {OC_UNARY, 1, "silu"},
    {OC_UNARY, 1, "gelu_erf"},  {OC_UNARY, 1, "tanh"},      {OC_UNARY, 1, "exp"},       {OC_UNARY, 1, "rsqrt"},
    {OC_MASK, 1, "causal_mask"}, {OC_REDUCE, 1, "reduce_sum"}, {OC_REDUCE, 1, "reduce_max"}, {OC_REDUCE, 1, "reduce_mean"},
    {OC_SOFTMAX, 1, "softmax"}, {OC_LAYERNORM, 3, "layernorm"}, {OC_RMSNORM, 2, "rmsnorm"}, {OC_GROUPNORM, 3, "groupnorm"},
    {OC_PERMUTE, 1, "permute"}, {OC_RESHAPE, 1, "reshape"},
    {OC_CONCAT_ROWS, 2, "concat_rows"}, {OC_MATVEC, 2, "matvec"}, {OC_VECMAT, 2, "vecmat"},
    {OC_CONCAT, 2, "concat"}, {OC_SLICE, 1, "slice"}, {OC_DWCONV, 2, "dwconv2d"},
};

bool is_elementwise(OpClass c) { return c == OC_BINARY || c == OC_UNARY || c == OC_MASK; }

typedef std::vector<int64_t> Shape;

int64_t numel(const Shape& s) {
    int64_t n = 1;
    for (int64_t d : s) n *= d;
    return n;
}

// lower-rank operand equals the trailing dims of the other (leading extents of 1 are ignored)
bool is_trailing(const Shape& small_in, const Shape& big) {
    size_t lead = 0;
    while (lead + 1 < small_in.size() && small_in[lead] == 1) ++lead;
    Shape small(small_in.begin() + lead, small_in.end());
    if (small.size() > big.size()) return false;
    return std::equal(small.begin(), small.end(), big.end() - small.size());
}

// `small` is `big` with the last extent collapsed to 1 (the shape a keep-dim reduction over the last dim gives)
bool is_row_value_of(const Shape& small, const Shape& big) {
    if (small.size() != big.size() || small.size() < 1 || small.back() != 1 || big.back() == 1) return false;
    return std::equal(small.begin(), small.end() - 1, big.begin());
}

// `small` broadcasts onto `big` the numpy way: aligned at the innermost dimension, every extent equal or 1
bool broadcasts_onto(const Shape& small, const Shape& big) {
    if (small.size() > big.size()) return false;
    const size_t off = big.size() - small.size();
    for (size_t i = 0; i < small.size(); ++i)
        if (small[i] != big[off + i] && small[i] != 1) return false;
    return true;
}

int dtype_size(int dt) { return dt == PF_F32 ? 4 : 2; }

// A REDUCE_* operator with integer attributes names the dimensions it reduces; without, or with just the last
// dimension, it is the row reduction.
bool reduces_other_dims(const pf_op_desc& o, size_t rank) { return o.n_i > 1 || (o.n_i == 1 && o.i[0] != (int64_t)rank - 1); }

struct Checked {
    std::vector<Shape> shape;  // per value id
};

// Full structural + shape check.  Fills per-value shapes.
pf_status check_desc(const pf_chain_desc* d, Checked* out) {
    if (!d) return fail(PF_ERR_INVALID_ARG, "desc is null");
    if (d->struct_size != sizeof(pf_chain_desc))
        return fail(PF_ERR_INVALID_ARG, "struct_size %u != %zu", d->struct_size, sizeof(pf_chain_desc));
    if (d->version != PF_CHAIN_VERSION) return fail(PF_ERR_INVALID_ARG, "version %u unsupported", d->version);
    if (d->n_inputs < 1 || d->n_inputs > PF_MAX_INPUTS) return fail(PF_ERR_INVALID_ARG, "n_inputs %d out of range", d->n_inputs);
    if (d->n_ops < 1 || d->n_ops > PF_MAX_OPS) return fail(PF_ERR_INVALID_ARG, "n_ops %d out of range", d->n_ops);
    if (d->n_outputs < 1 || d->n_outputs > PF_MAX_OUTPUTS) return fail(PF_ERR_INVALID_ARG, "n_outputs %d out of range", d->n_outputs);
    std::vector<Shape>& sh = out->shape;
    sh.clear();
    for (int k = 0; k < d->n_inputs; ++k) {
        const pf_tensor_desc& t = d->inputs[k];
        if (t.dtype < PF_F32 || t.dtype > PF_BF16) return fail(PF_ERR_DTYPE, "input %d: unknown dtype %d", k, t.dtype);
        if (t.rank < 1 || t.rank > PF_MAX_RANK) return fail(PF_ERR_INVALID_ARG, "input %d: rank %d out of range", k, t.rank);
        Shape s(t.shape, t.shape + t.rank);
        for (int64_t e : s)
            if (e <= 0) return fail(PF_ERR_SHAPE, "input %d: non-positive extent", k);
        sh.push_back(s);
    }
    for (int k = 0; k < d->n_ops; ++k) {
        const pf_op_desc& o = d->ops[k];
        const int id = d->n_inputs + k;
        if (o.op < 0 || o.op >= PF_OP_COUNT_) return fail(PF_ERR_INVALID_ARG, "op %d: unknown operator %d", k, o.op);
        const OpTraits& tr = kOps[o.op];
        if (o.n_src != tr.arity) return fail(PF_ERR_INVALID_ARG, "op %d (%s): n_src %d, expected %d", k, tr.name, o.n_src, tr.arity);
        for (int s = 0; s < o.n_src; ++s)
            if (o.src[s] < 0 || o.src[s] >= id) return fail(PF_ERR_INVALID_ARG, "op %d (%s): operand id %d out of range", k, tr.name, o.src[s]);
        const Shape& a = sh[o.src[0]];
        Shape r;
        switch (tr.cls) {
            case OC_BINARY: {
                const Shape& b = sh[o.src[1]];
                if (a == b) r = a;
                else if (is_row_value_of(b, a)) r = a;  // a keep-dim reduction result broadcast back over its row
                else if (is_row_value_of(a, b)) r = b;
                else if (numel(a) == numel(b) && b.size() > a.size() && is_trailing(a, b)) r = b;  // [n] with [1, n]: the higher rank
                else if (numel(a) >= numel(b) && is_trailing(b, a)) r = a;
                else if (numel(b) > numel(a) && is_trailing(a, b)) r = b;
                else if (broadcasts_onto(b, a)) r = a;  // extents of 1 anywhere (an attention mask [B, 1, 1, S], a per-sample bias)
                else if (broadcasts_onto(a, b)) r = b;
                else return fail(PF_ERR_SHAPE, "op %d (%s): operand shapes do not broadcast", k, tr.name);
                break;
            }
            case OC_UNARY:
                if ((o.op == PF_SCALE || o.op == PF_ADDC) && !std::isfinite(o.f[0]))
                    return fail(PF_ERR_INVALID_ARG, "op %d (%s): constant is not finite", k, tr.name);
                r = a;
                break;
            case OC_MASK:
                if (a.size() < 2) return fail(PF_ERR_SHAPE, "op %d (causal_mask): rank < 2", k);
                r = a;
                break;
            case OC_REDUCE: {
                r = a;
                if (o.n_i == 0) {
                    r.back() = 1;
                    break;
                }
                if (o.n_i > (int)a.size()) return fail(PF_ERR_INVALID_ARG, "op %d (%s): more dimensions named than the operand has", k, tr.name);
                for (int q = 0; q < o.n_i; ++q) {
                    if (o.i[q] < 0 || o.i[q] >= (int64_t)a.size() || (q > 0 && o.i[q] <= o.i[q - 1]))
                        return fail(PF_ERR_INVALID_ARG, "op %d (%s): i = the dimensions to reduce, ascending", k, tr.name);
                    r[o.i[q]] = 1;
                }
                break;
            }
            case OC_SOFTMAX: r = a; break;
            case OC_LAYERNORM:
            case OC_RMSNORM:
            case OC_GROUPNORM: {
                if (!(o.f[0] >= 0.0f) || !std::isfinite(o.f[0])) return fail(PF_ERR_INVALID_ARG, "op %d (%s): eps must be finite and >= 0", k, tr.name);
                if (tr.cls == OC_GROUPNORM) {
                    if (a.size() < 2) return fail(PF_ERR_SHAPE, "op %d (groupnorm): rank < 2", k);
                    if (o.n_i != 1 || o.i[0] < 1 || a.back() % o.i[0] != 0)
                        return fail(PF_ERR_INVALID_ARG, "op %d (groupnorm): groups must divide the channel count", k);
                }
                for (int s = 1; s < o.n_src; ++s) {
                    const Shape& p = sh[o.src[s]];
                    if (p.size() != 1 || p[0] != a.back())
                        return fail(PF_ERR_SHAPE, "op %d (%s): parameter %d must have shape [%lld]", k, tr.name, s, (long long)a.back());
                }
                r = a;
                break;
            }
            case OC_PERMUTE: {
                const int rank = (int)a.size();
                if (o.n_i != rank) return fail(PF_ERR_INVALID_ARG, "op %d (permute): n_i %d != rank %d", k, o.n_i, rank);
                bool seen[PF_MAX_RANK] = {false};
                r.resize(rank);
                for (int q = 0; q < rank; ++q) {
                    const int64_t p = o.i[q];
                    if (p < 0 || p >= rank || seen[p]) return fail(PF_ERR_INVALID_ARG, "op %d (permute): not a permutation", k);
                    seen[p] = true;
                    r[q] = a[p];
                }
                break;
            }
            case OC_CONCAT_ROWS:
            case OC_MATVEC: {
                // a [..., t, d] with b [..., d]
                const Shape& b = sh[o.src[1]];
                if (a.size() < 2 || b.size() != a.size() - 1 || !std::equal(a.begin(), a.end() - 2, b.begin()) || b.back() != a.back())
                    return fail(PF_ERR_SHAPE, "op %d (%s): needs [..., t, d] and [..., d]", k, tr.name);
                r = a;
                if (tr.cls == OC_CONCAT_ROWS) r[r.size() - 2] += 1;
                else r.pop_back();
                break;
            }
            case OC_DWCONV: {
                const Shape& b = sh[o.src[1]];
                if (a.size() != 4 || b.size() != 3 || b[2] != a[3]) return fail(PF_ERR_SHAPE, "op %d (dwconv2d): needs x [n, h, w, c] and kernels [kh, kw, c]", k);
                if (b[0] % 2 == 0 || b[1] % 2 == 0) return fail(PF_ERR_SHAPE, "op %d (dwconv2d): kernel extents must be odd", k);
                if (o.n_i > 1 || (o.n_i == 1 && (o.i[0] < 1 || o.i[0] > 8)))
                    return fail(PF_ERR_INVALID_ARG, "op %d (dwconv2d): i[0] is the stride (1 .. 8), at most one integer attribute", k);
                r = a;
                if (o.n_i == 1) {
                    r[1] = (a[1] - 1) / o.i[0] + 1;
                    r[2] = (a[2] - 1) / o.i[0] + 1;
                }
                break;
            }
            case OC_CONCAT: {
                const Shape& b = sh[o.src[1]];
                const int64_t ax = o.n_i == 1 ? o.i[0] : -1;
                if (ax < 0 || ax >= (int64_t)a.size() || b.size() != a.size())
                    return fail(PF_ERR_INVALID_ARG, "op %d (concat): i[0] must name an axis of both operands", k);
                for (size_t q = 0; q < a.size(); ++q)
                    if ((int64_t)q != ax && a[q] != b[q]) return fail(PF_ERR_SHAPE, "op %d (concat): operands differ outside the axis", k);
                r = a;
                r[ax] += b[ax];
                break;
            }
            case OC_SLICE: {
                const int64_t ax = o.n_i == 3 ? o.i[0] : -1;
                if (ax < 0 || ax >= (int64_t)a.size()) return fail(PF_ERR_INVALID_ARG, "op %d (slice): i = {axis, start, length}", k);
                if (o.i[1] < 0 || o.i[2] < 1 || o.i[1] + o.i[2] > a[ax]) return fail(PF_ERR_SHAPE, "op %d (slice): range outside the axis", k);
                r = a;
                r[ax] = o.i[2];
                break;
            }
            case OC_VECMAT: {
                // a [..., t] with b [..., t, d]
                const Shape& b = sh[o.src[1]];
                if (b.size() < 2 || a.size() != b.size() - 1 || !std::equal(a.begin(), a.end(), b.begin()))
                    return fail(PF_ERR_SHAPE, "op %d (vecmat): needs [..., t] and [..., t, d]", k);
                r.assign(b.begin(), b.end() - 2);
                r.push_back(b.back());
                break;
            }
            case OC_RESHAPE: {
                if (o.n_i < 1 || o.n_i > PF_MAX_RANK) return fail(PF_ERR_INVALID_ARG, "op %d (reshape): n_i out of range", k);
                r.assign(o.i, o.i + o.n_i);
                for (int64_t e : r)
                    if (e <= 0) return fail(PF_ERR_SHAPE, "op %d (reshape): non-positive extent", k);
                if (numel(r) != numel(a)) return fail(PF_ERR_SHAPE, "op %d (reshape): element count changes", k);
                break;
            }
        }
        sh.push_back(r);
    }
    for (int k = 0; k < d->n_outputs; ++k) {
        if (d->out_value[k] < d->n_inputs || d->out_value[k] >= d->n_inputs + d->n_ops)
            return fail(PF_ERR_INVALID_ARG, "output %d: value id %d is not an operator result", k, d->out_value[k]);
        if (d->out_dtype[k] < PF_F32 || d->out_dtype[k] > PF_BF16) return fail(PF_ERR_DTYPE, "output %d: unknown dtype", k);
        for (int j = 0; j < k; ++j)
            if (d->out_value[j] == d->out_value[k]) return fail(PF_ERR_INVALID_ARG, "outputs %d and %d name the same value", j, k);
    }
    return PF_OK;
}

// ---------------------------------------------------------------------------------------------
// lowering
// ---------------------------------------------------------------------------------------------
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
};

struct Lowerer {
    const pf_chain_desc* d;
    const Checked* c;
    Lowered* L;
    std::vector<int> alias;      // value id -> root value id (reshape chains collapse)
    std::vector<int> uses;       // remaining uses per root value
    enum LocKind { LOC_NONE, LOC_ACC, LOC_TMP, LOC_FULL, LOC_VEC, LOC_ROW };
    struct Loc {
        LocKind kind = LOC_NONE;
        int slot = -1;
    };
    std::vector<Loc> loc;
    bool tmp_busy[PF_DEV_MAX_TMP] = {false, false};
    bool row_busy[PF_DEV_MAX_ROWV] = {false, false, false, false};
    bool row_prog = false;       // reductions are lowered as steps of the program (CORE_ROWPROG)
    int acc_val = -1;
    pf::Program* prog = nullptr;
    bool in_epi = false;
    int64_t region_numel = 0;
    pf_status status = PF_OK;

    int root(int v) const { return alias[v]; }

    bool emit(uint8_t code, uint8_t kind, uint8_t slot, float imm = 0.0f, int32_t ival = 0, bool use_ival = false) {
        if (prog->n >= PF_DEV_MAX_UOPS) {
            status = fail(PF_ERR_UNSUPPORTED, "chain needs more than %d element-wise steps", PF_DEV_MAX_UOPS);
            return false;
        }
        pf::Uop& u = prog->u[prog->n++];
        u.code = code;
        u.kind = kind;
        u.slot = slot;
        u.pad = 0;
        if (use_ival) u.ival = ival;
        else u.imm = imm;
        return true;
    }

    // location of a raw input operand (assigning a slot on first use)
    Shape cur_result_shape;  // result shape of the operator being lowered (what a broadcast input is broadcast against)

    // force_vec: classify the input as a broadcast operand even if it has as many elements as the value (a
    // normalisation parameter of a single-row tensor)
    bool input_loc(int v, Loc* out, bool force_vec = false) {
        if (loc[v].kind == LOC_FULL || loc[v].kind == LOC_VEC) {
            // an input used on both sides of a layout change would need two layouts
            const bool was_epi = loc[v].kind == LOC_FULL ? L->full_is_epi[loc[v].slot] : L->vec_is_epi[loc[v].slot];
            if (was_epi != in_epi && L->core == pf::CORE_PERMUTE) {
                status = fail(PF_ERR_UNSUPPORTED, "input %d is used before and after the permutation", v);
                return false;
            }
            *out = loc[v];
            return true;
        }
        const int64_t n = numel(c->shape[v]);
        if (d->inputs[v].dtype != L->main_dtype) {
            status = fail(PF_ERR_DTYPE, "input %d: dtype differs from the chain's main dtype", v);
            return false;
        }
        if (n == region_numel && !force_vec) {
            if (L->n_full >= PF_DEV_MAX_FULL) {
                status = fail(PF_ERR_UNSUPPORTED, "more than %d full-shape inputs", PF_DEV_MAX_FULL);
                return false;
            }
            L->full_input[L->n_full] = v;
            L->full_is_epi[L->n_full] = in_epi;
            loc[v].kind = LOC_FULL;
            loc[v].slot = L->n_full++;
        } else {
            if (L->n_vec >= PF_DEV_MAX_VEC) {
                status = fail(PF_ERR_UNSUPPORTED, "more than %d broadcast inputs", PF_DEV_MAX_VEC);
                return false;
            }
            L->vec_input[L->n_vec] = v;
            L->vec_is_epi[L->n_vec] = in_epi;
            L->vec_partner[L->n_vec] = cur_result_shape;
            loc[v].kind = LOC_VEC;
            loc[v].slot = L->n_vec++;
        }
        *out = loc[v];
        return true;
    }

    bool operand_of(int v, uint8_t* kind, uint8_t* slot) {
        Loc l;
        if (v < d->n_inputs) {
            if (!input_loc(v, &l)) return false;
        } else {
            l = loc[v];
        }
        switch (l.kind) {
            case LOC_FULL: *kind = pf::K_FULL; break;
            case LOC_VEC: *kind = pf::K_VEC; break;
            case LOC_TMP: *kind = pf::K_TMP; break;
            case LOC_ROW: *kind = pf::K_ROW; break;
            default:
                status = fail(PF_ERR_UNSUPPORTED, "value %d is not available where it is used (crosses the core step?)", v);
                return false;
        }
        *slot = (uint8_t)l.slot;
        return true;
    }

    // keep the accumulator's value if something still needs it
    bool spill_acc_if_live(int consumed_now) {
        if (acc_val < 0) return true;
        if (acc_val < d->n_inputs) return true;  // an input can always be fetched again from its operand slot
        if (loc[acc_val].kind == LOC_ROW) return true;  // so can a row value
        if (uses[acc_val] - consumed_now <= 0) return true;
        if (loc[acc_val].kind == LOC_TMP) return true;
        for (int t = 0; t < PF_DEV_MAX_TMP; ++t)
            if (!tmp_busy[t]) {
                tmp_busy[t] = true;
                if (t + 1 > L->n_tmp) L->n_tmp = t + 1;
                if (!emit(pf::U_SAVE, pf::K_NONE, (uint8_t)t)) return false;
                loc[acc_val].kind = LOC_TMP;
                loc[acc_val].slot = t;
                return true;
            }
        status = fail(PF_ERR_UNSUPPORTED, "chain keeps more than %d intermediate values alive", PF_DEV_MAX_TMP);
        return false;
    }

    void consume(int v) {
        if (--uses[v] != 0) return;
        if (loc[v].kind == LOC_TMP) {
            tmp_busy[loc[v].slot] = false;
            loc[v].kind = LOC_NONE;
        } else if (loc[v].kind == LOC_ROW) {
            row_busy[loc[v].slot] = false;
            loc[v].kind = LOC_NONE;
        }
    }

    bool load_acc(int v) {
        if (acc_val == v) return true;
        if (!spill_acc_if_live(0)) return false;
        uint8_t kind, slot;
        if (!operand_of(v, &kind, &slot)) return false;
        if (!emit(pf::U_MOV, kind, slot)) return false;
        if (acc_val >= 0 && loc[acc_val].kind == LOC_ACC) loc[acc_val].kind = LOC_NONE;
        acc_val = v;
        return true;
    }

    void set_acc(int v) {
        if (acc_val >= 0 && loc[acc_val].kind == LOC_ACC) loc[acc_val].kind = LOC_NONE;
        acc_val = v;
        if (loc[v].kind == LOC_NONE) loc[v].kind = LOC_ACC;
    }

    // secondary outputs: store a value the moment it sits in the accumulator
    bool maybe_store_output(int v) {
        if (v == final_value) return true;  // the kernel's last store writes it
        for (int o = 0; o < d->n_outputs; ++o) {
            if (root(d->out_value[o]) != v) continue;
            if (numel(c->shape[v]) != region_numel) {
                status = fail(PF_ERR_UNSUPPORTED, "output %d: only full-shape values can be secondary outputs", o);
                return false;
            }
            L->out_slot_to_user[1] = o;
            L->n_out = 2;
            if (!emit(pf::U_STORE, pf::K_NONE, 1)) return false;
            consume(v);
        }
        return true;
    }

    int final_value = -1;

    bool lower_elementwise_op(int k) {
        const pf_op_desc& o = d->ops[k];
        const int id = d->n_inputs + k;
        cur_result_shape = c->shape[id];
        const OpTraits& tr = kOps[o.op];
        if (tr.cls == OC_RESHAPE) return true;  // alias only
        if (tr.cls == OC_REDUCE) {
            // row program: the reduction is a step; the accumulator keeps the reduced value's source
            const int a = root(o.src[0]);
            if (!row_prog || numel(c->shape[o.src[0]]) != region_numel) {
                status = fail(PF_ERR_UNSUPPORTED, "op %d (%s): reductions inside a chain reduce full-shape values over the last dimension", k, tr.name);
                return false;
            }
            if (!load_acc(a)) return false;
            int r = -1;
            for (int t = 0; t < PF_DEV_MAX_ROWV && r < 0; ++t)
                if (!row_busy[t]) r = t;
            if (r < 0) {
                status = fail(PF_ERR_UNSUPPORTED, "chain keeps more than %d per-row values alive", PF_DEV_MAX_ROWV);
                return false;
            }
            row_busy[r] = true;
            const uint8_t code = o.op == PF_REDUCE_SUM ? pf::U_RED_SUM : (o.op == PF_REDUCE_MAX ? pf::U_RED_MAX : pf::U_RED_MEAN);
            if (!emit(code, pf::K_NONE, (uint8_t)r)) return false;
            loc[id].kind = LOC_ROW;
            loc[id].slot = r;
            consume(a);  // a stays in the accumulator if something else still needs it
            if (uses[id] == 0) {  // a reduction nobody reads
                row_busy[r] = false;
                loc[id].kind = LOC_NONE;
            }
            return true;
        }
        if (tr.cls == OC_UNARY || tr.cls == OC_MASK) {
            const int a = root(o.src[0]);
            if (tr.cls == OC_MASK && numel(c->shape[o.src[0]]) != region_numel) {
                status = fail(PF_ERR_UNSUPPORTED, "op %d (causal_mask): needs a full-shape value", k);
                return false;
            }
            if (!load_acc(a)) return false;
            if (!spill_acc_if_live(1)) return false;
            consume(a);
            bool ok = true;
            switch (o.op) {
                case PF_SCALE: ok = emit(pf::U_MUL, pf::K_IMM, 0, o.f[0]); break;
                case PF_ADDC: ok = emit(pf::U_ADD, pf::K_IMM, 0, o.f[0]); break;
                case PF_NEG: ok = emit(pf::U_NEG, pf::K_NONE, 0); break;
                case PF_RELU: ok = emit(pf::U_RELU, pf::K_NONE, 0); break;
                case PF_SIGMOID: ok = emit(pf::U_SIGMOID, pf::K_NONE, 0); break;
                case PF_SILU: ok = emit(pf::U_SILU, pf::K_NONE, 0); break;
                case PF_GELU_ERF: ok = emit(pf::U_GELU_ERF, pf::K_NONE, 0); break;
                case PF_TANH: ok = emit(pf::U_TANH, pf::K_NONE, 0); break;
                case PF_EXP: ok = emit(pf::U_EXP, pf::K_NONE, 0); break;
                case PF_RSQRT: ok = emit(pf::U_RSQRT, pf::K_NONE, 0); break;
                case PF_CAUSAL_MASK: {
                    const Shape& s = c->shape[o.src[0]];
                    const int64_t si = s[s.size() - 2], sj = s.back();
                    if (sj != region_inner) {
                        status = fail(PF_ERR_UNSUPPORTED, "causal_mask: the masked value's last extent differs from the kernel's row length");
                        return false;
                    }
                    if (si > 0x7fffffffLL) {
                        status = fail(PF_ERR_UNSUPPORTED, "causal_mask: extent too large");
                        return false;
                    }
                    ok = emit(pf::U_MASK_CAUSAL, pf::K_NONE, 0, 0.0f, (int32_t)si, true);
                    break;
                }
                default: ok = false; break;
            }
            if (!ok) return false;
            set_acc(id);
            return maybe_store_output(id);
        }
        // binary
        const int a = root(o.src[0]), b = root(o.src[1]);
        static const uint8_t fwd[6] = {pf::U_ADD, pf::U_SUB, pf::U_MUL, pf::U_DIV, pf::U_MAX, pf::U_MIN};
        static const uint8_t rev[6] = {pf::U_ADD, pf::U_RSUB, pf::U_MUL, pf::U_RDIV, pf::U_MAX, pf::U_MIN};
        uint8_t code, kind, slot;
        if (a == b) {
            if (!load_acc(a)) return false;
            if (a < d->n_inputs) {
                if (!operand_of(a, &kind, &slot)) return false;  // the same input on both sides
            } else {
                // the same computed value on both sides: park a copy in a temporary
                if (loc[a].kind != LOC_TMP && !spill_acc_if_live(0)) return false;  // uses[a] >= 2: this saves it
                if (loc[a].kind != LOC_TMP) {
                    status = fail(PF_ERR_UNSUPPORTED, "internal: operand used twice could not be parked");
                    return false;
                }
                kind = pf::K_TMP;
                slot = (uint8_t)loc[a].slot;
            }
            code = fwd[o.op];
            if (!emit(code, kind, slot)) return false;
            consume(a);
            consume(a);
        } else {
            int in_acc, other;
            bool reversed;
            if (acc_val == a) { in_acc = a; other = b; reversed = false; }
            else if (acc_val == b) { in_acc = b; other = a; reversed = true; }
            else {
                // prefer loading a computed / full-shape value into the accumulator
                const bool a_small = (a < d->n_inputs && numel(c->shape[a]) != region_numel) || loc[a].kind == LOC_ROW;
                const bool b_small = (b < d->n_inputs && numel(c->shape[b]) != region_numel) || loc[b].kind == LOC_ROW;
                if (a_small && !b_small) { in_acc = b; other = a; reversed = true; }
                else { in_acc = a; other = b; reversed = false; }
                if (!load_acc(in_acc)) return false;
            }
            if (!spill_acc_if_live(1)) return false;
            if (!operand_of(other, &kind, &slot)) return false;
            code = reversed ? rev[o.op] : fwd[o.op];
            if (!emit(code, kind, slot)) return false;
            consume(in_acc);
            consume(other);
        }
        set_acc(id);
        return maybe_store_output(id);
    }

    int64_t region_inner = 0;
};

// value ids of chain inputs never reach zero uses through consume() bookkeeping problems: inputs keep
// LOC_FULL / LOC_VEC for the whole region, so only computed values matter for temporaries.

// Layout-only chains with concatenations or slices: nothing to lower, the planner evaluates the index map.
pf_status lower_layout(const pf_chain_desc* d, const Checked& c, Lowered* L) {
    (void)c;
    for (int k = 0; k < d->n_ops; ++k) {
        const OpClass cls = kOps[d->ops[k].op].cls;
        if (cls != OC_CONCAT && cls != OC_SLICE && cls != OC_PERMUTE && cls != OC_RESHAPE)
            return fail(PF_ERR_UNSUPPORTED, "op %d (%s): concat / slice are implemented in layout-only chains (with permute and reshape)", k,
                        kOps[d->ops[k].op].name);
    }
    L->core = pf::CORE_GATHER;
    L->main_dtype = d->out_dtype[0];
    for (int o = 0; o < d->n_outputs; ++o)
        if (d->out_dtype[o] != L->main_dtype) return fail(PF_ERR_DTYPE, "outputs of different dtypes are not implemented");
    for (int k = 0; k < d->n_inputs; ++k)
        if (d->inputs[k].dtype != L->main_dtype) return fail(PF_ERR_DTYPE, "input %d: a layout-only chain cannot convert between dtypes", k);
    L->n_out = d->n_outputs;
    return PF_OK;
}

// One-token attention (paper section 8, GPT-2 case study): the three contraction / concatenation operators are
// accepted in exactly one arrangement, matched structurally from the final operator backwards:
//   o = VECMAT(SOFTMAX([SCALE](MATVEC(K', q))), V'),  K' = CONCAT_ROWS(K, k) or an input, V' likewise.
pf_status lower_attention(const pf_chain_desc* d, const Checked& c, Lowered* L) {
    const int n_in = d->n_inputs;
    auto op_of = [&](int v) -> const pf_op_desc* { return v >= n_in ? &d->ops[v - n_in] : nullptr; };
    auto bad = [&](const char* what) { return fail(PF_ERR_UNSUPPORTED, "attention chain: %s", what); };
    const int final_v = n_in + d->n_ops - 1;
    const pf_op_desc* vm = op_of(final_v);
    if (!vm || vm->op != PF_VECMAT) return bad("the last operator must be vecmat(softmax(...), values)");
    const pf_op_desc* sm = op_of(vm->src[0]);
    if (!sm || sm->op != PF_SOFTMAX) return bad("vecmat's first operand must be a softmax");
    int used_ops = 2;
    const pf_op_desc* x = op_of(sm->src[0]);
    L->attn_scale = 1.0f;
    if (x && x->op == PF_SCALE) {
        L->attn_scale = x->f[0];
        x = op_of(x->src[0]);
        ++used_ops;
    }
    if (!x || x->op != PF_MATVEC) return bad("the softmax must be taken over (scaled) matvec(keys, q)");
    ++used_ops;
    const int q_in = x->src[1];
    if (q_in >= n_in) return bad("q must be a chain input");
    int k_val = x->src[0], v_val = vm->src[1];
    int kc_val = -1, vc_val = -1;  // value ids of the concatenation results
    int K_in = k_val, V_in = v_val, kn_in = -1, vn_in = -1;
    if (const pf_op_desc* kc = op_of(k_val)) {
        if (kc->op != PF_CONCAT_ROWS || kc->src[0] >= n_in || kc->src[1] >= n_in) return bad("keys must be an input or concat_rows(input, input)");
        kc_val = k_val;
        K_in = kc->src[0];
        kn_in = kc->src[1];
        ++used_ops;
    }
    if (const pf_op_desc* vc = op_of(v_val)) {
        if (vc->op != PF_CONCAT_ROWS || vc->src[0] >= n_in || vc->src[1] >= n_in) return bad("values must be an input or concat_rows(input, input)");
        vc_val = v_val;
        V_in = vc->src[0];
        vn_in = vc->src[1];
        ++used_ops;
    }
    if ((kn_in < 0) != (vn_in < 0)) return bad("keys and values must both be concatenated or both be inputs");
    if (used_ops != d->n_ops) return bad("operators outside the attention pattern");
    if (c.shape[K_in] != c.shape[V_in]) return bad("key and value caches differ in shape");
    L->core = pf::CORE_ATTN_DECODE;
    L->attn_in[0] = q_in;
    L->attn_in[1] = kn_in;
    L->attn_in[2] = vn_in;
    L->attn_in[3] = K_in;
    L->attn_in[4] = V_in;
    for (int o = 0; o < d->n_outputs; ++o) {
        const int v = d->out_value[o];
        if (v == final_v) L->attn_out[0] = o;
        else if (v == kc_val) L->attn_out[1] = o;
        else if (v == vc_val) L->attn_out[2] = o;
        else return bad("only the attention result and the grown caches can be outputs");
    }
    if (L->attn_out[0] < 0) return bad("the attention result must be an output");
    L->main_dtype = d->out_dtype[L->attn_out[0]];
    for (int o = 0; o < d->n_outputs; ++o)
        if (d->out_dtype[o] != L->main_dtype) return fail(PF_ERR_DTYPE, "outputs of different dtypes are not implemented");
    for (int i = 0; i < 5; ++i)
        if (L->attn_in[i] >= 0 && d->inputs[L->attn_in[i]].dtype != L->main_dtype)
            return fail(PF_ERR_DTYPE, "input %d: dtype differs from the chain's main dtype", L->attn_in[i]);
    if (!std::isfinite(L->attn_scale) || !(L->attn_scale > 0.0f)) return bad("the score scale must be positive and finite");
    L->pre_shape = c.shape[K_in];
    L->post_shape = c.shape[final_v];
    L->n_out = d->n_outputs;
    return PF_OK;
}

pf_status lower_chain(const pf_chain_desc* d, const Checked& c, Lowered* L) {
    const int n_in = d->n_inputs, n_val = d->n_inputs + d->n_ops;
    for (int k = 0; k < d->n_ops; ++k) {
        const OpClass cls = kOps[d->ops[k].op].cls;
        if (cls == OC_CONCAT_ROWS || cls == OC_MATVEC || cls == OC_VECMAT) return lower_attention(d, c, L);
    }
    for (int k = 0; k < d->n_ops; ++k) {
        const OpClass cls = kOps[d->ops[k].op].cls;
        if (cls == OC_CONCAT || cls == OC_SLICE) return lower_layout(d, c, L);
    }
    // Row program: a chain written in basic operators only (element-wise, reduce over the last dimension,
    // broadcast of the reduced value back over its row; paper section 6) whose result has the full shape.
    // The reduce -> broadcast pairs need a synchronisation no wider than a row (section 5.1), so they become
    // steps of one register-resident program instead of a kernel boundary.
    int n_reduce = 0, n_other_core = 0;
    for (int k = 0; k < d->n_ops; ++k) {
        const OpClass cls = kOps[d->ops[k].op].cls;
        if (cls == OC_REDUCE && !reduces_other_dims(d->ops[k], c.shape[d->ops[k].src[0]].size())) ++n_reduce;
        else if (!is_elementwise(cls) && cls != OC_RESHAPE) ++n_other_core;  // (a reduction over other dimensions is a core of its own)
    }
    const bool row_prog = n_reduce >= 1 && n_other_core == 0 && c.shape[n_in + d->n_ops - 1].back() != 1;
    // the core: first operator that is neither element-wise nor a reshape
    L->core_op = -1;
    for (int k = 0; k < d->n_ops && !row_prog; ++k) {
        const OpClass cls = kOps[d->ops[k].op].cls;
        if (!is_elementwise(cls) && cls != OC_RESHAPE) {
            if (L->core_op >= 0)
                return fail(PF_ERR_UNSUPPORTED, "op %d (%s): a chain may hold one reduce / normalise / permute step", k, kOps[d->ops[k].op].name);
            L->core_op = k;
        }
    }
    Lowerer lw;
    lw.d = d;
    lw.c = &c;
    lw.L = L;
    lw.row_prog = row_prog;
    lw.alias.resize(n_val);
    for (int v = 0; v < n_val; ++v) lw.alias[v] = v;
    for (int k = 0; k < d->n_ops; ++k)
        if (kOps[d->ops[k].op].cls == OC_RESHAPE) lw.alias[n_in + k] = lw.alias[d->ops[k].src[0]];
    lw.uses.assign(n_val, 0);
    for (int k = 0; k < d->n_ops; ++k) {
        if (kOps[d->ops[k].op].cls == OC_RESHAPE) continue;
        for (int s = 0; s < d->ops[k].n_src; ++s) lw.uses[lw.root(d->ops[k].src[s])]++;
    }
    for (int o = 0; o < d->n_outputs; ++o) lw.uses[lw.root(d->out_value[o])]++;
    lw.loc.assign(n_val, Lowerer::Loc());

    // the chain's final value: the last operator's result; it must be an output
    int last_op = d->n_ops - 1;
    lw.final_value = lw.root(n_in + last_op);
    bool final_is_output = false;
    for (int o = 0; o < d->n_outputs; ++o)
        if (lw.root(d->out_value[o]) == lw.final_value) {
            final_is_output = true;
            L->out_slot_to_user[0] = o;
        }
    if (!final_is_output) return fail(PF_ERR_UNSUPPORTED, "the last operator's result must be an output");
    if (lw.final_value < n_in) return fail(PF_ERR_UNSUPPORTED, "the chain computes nothing (only reshapes of an input)");
    L->n_out = 1;
    L->out_slot_to_user[1] = -1;

    // main dtype: that of the primary output; every tensor the kernels touch must share it
    L->main_dtype = d->out_dtype[L->out_slot_to_user[0]];
    for (int o = 0; o < d->n_outputs; ++o)
        if (d->out_dtype[o] != L->main_dtype) return fail(PF_ERR_DTYPE, "outputs of different dtypes are not implemented");

    memset(&L->pro, 0, sizeof(L->pro));
    memset(&L->epi, 0, sizeof(L->epi));

    const int core_k = L->core_op;
    const int pro_end = core_k >= 0 ? core_k : d->n_ops;
    // shape entering the core (or leaving the chain when there is none)
    int pre_value;
    if (core_k >= 0) pre_value = d->ops[core_k].src[0];
    else pre_value = n_in + d->n_ops - 1;
    L->pre_shape = c.shape[pre_value];
    L->post_shape = core_k >= 0 ? c.shape[n_in + core_k] : L->pre_shape;

    if (row_prog) {
        L->core = pf::CORE_ROWPROG;
        for (int k = 0; k < d->n_ops; ++k)
            if (kOps[d->ops[k].op].cls == OC_RESHAPE)
                return fail(PF_ERR_UNSUPPORTED, "reshapes inside a chain with in-line reductions are not implemented");
    }
    if (core_k >= 0) {
        const pf_op_desc& o = d->ops[core_k];
        switch (o.op) {
            case PF_SOFTMAX: L->core = pf::CORE_SOFTMAX; break;
            case PF_LAYERNORM: L->core = pf::CORE_LAYERNORM; break;
            case PF_RMSNORM: L->core = pf::CORE_RMSNORM; break;
            case PF_GROUPNORM: L->core = pf::CORE_GROUPNORM; L->groups = o.i[0]; break;
            case PF_REDUCE_SUM:
            case PF_REDUCE_MAX:
            case PF_REDUCE_MEAN: {
                L->core = o.op == PF_REDUCE_SUM ? pf::CORE_REDUCE_SUM : (o.op == PF_REDUCE_MAX ? pf::CORE_REDUCE_MAX : pf::CORE_REDUCE_MEAN);
                const Shape& xs = c.shape[o.src[0]];
                if (reduces_other_dims(o, xs.size())) {
                    // implemented: every dimension between the first and the last (pooling of a channels-last tensor)
                    bool pooled = xs.size() >= 3 && o.n_i == (int)xs.size() - 2;
                    for (int q = 0; q < o.n_i && pooled; ++q) pooled = o.i[q] == q + 1;
                    if (!pooled)
                        return fail(PF_ERR_UNSUPPORTED, "op %d (%s): reductions run over the last dimension, or over all dimensions between the first and the last", core_k, kOps[o.op].name);
                    L->core = pf::CORE_POOL;
                    L->pool_op = o.op == PF_REDUCE_SUM ? 0 : (o.op == PF_REDUCE_MAX ? 1 : 2);
                }
                break;
            }
            case PF_DWCONV2D: L->core = pf::CORE_DWCONV; break;
            case PF_PERMUTE:
                L->core = pf::CORE_PERMUTE;
                for (int q = 0; q < o.n_i; ++q) L->perm[q] = (int)o.i[q];
                break;
            default: return fail(PF_ERR_UNSUPPORTED, "unexpected core operator");
        }
        L->eps = o.f[0];
    }

    // ---- prologue
    lw.prog = &L->pro;
    lw.in_epi = false;
    lw.region_numel = numel(L->pre_shape);
    lw.region_inner = L->pre_shape.back();
    for (int k = 0; k < pro_end; ++k)
        if (!lw.lower_elementwise_op(k)) return lw.status;
    if (core_k >= 0) {
        const int src = lw.root(d->ops[core_k].src[0]);
        if (!lw.load_acc(src)) return lw.status;
        if (!lw.spill_acc_if_live(1)) return lw.status;
        lw.consume(src);
        // temporaries do not survive the core step
        for (int t = 0; t < PF_DEV_MAX_TMP; ++t)
            if (lw.tmp_busy[t]) return fail(PF_ERR_UNSUPPORTED, "a value computed before the core step is used after it");
        // affine parameters (and convolution kernels): indexed by the core step itself, not broadcast
        lw.cur_result_shape.clear();
        const pf_op_desc& o = d->ops[core_k];
        for (int s = 1; s < o.n_src; ++s) {
            const int p = lw.root(o.src[s]);
            if (p >= n_in) return fail(PF_ERR_UNSUPPORTED, "normalisation parameters must be chain inputs");
            Lowerer::Loc l;
            if (!lw.input_loc(p, &l, true)) return lw.status;
            if (l.kind != Lowerer::LOC_VEC) return fail(PF_ERR_UNSUPPORTED, "a normalisation parameter is also used as a full-shape operand");
            L->core_vec[s - 1] = l.slot;
            lw.consume(p);
        }
        // ---- epilogue
        const int core_val = n_in + core_k;
        lw.acc_val = -1;
        lw.set_acc(core_val);
        lw.prog = &L->epi;
        lw.in_epi = true;
        lw.region_numel = numel(L->post_shape);
        lw.region_inner = L->post_shape.back();
        if (!lw.maybe_store_output(core_val)) return lw.status;
        for (int k = core_k + 1; k < d->n_ops; ++k)
            if (!lw.lower_elementwise_op(k)) return lw.status;
    }
    if (lw.acc_val != lw.final_value) return fail(PF_ERR_UNSUPPORTED, "internal: final value is not in the accumulator");
    // every declared output must have been reached
    for (int o = 0; o < d->n_outputs; ++o) {
        if (o == L->out_slot_to_user[0]) continue;
        if (L->n_out < 2 || L->out_slot_to_user[1] != o) return fail(PF_ERR_UNSUPPORTED, "output %d cannot be produced by this chain shape", o);
    }

    // causal-mask load skipping: legal when the masked value depends on loaded data only through steps
    // that come before the mask and nothing computed before the mask is kept
    L->mask_si = 0;
    L->core_mask = 0;
    L->core_scale = 1.0f;
    if (L->core == pf::CORE_SOFTMAX || L->core == pf::CORE_ROWPROG) {
        int mask_at = -1;
        for (int i = 0; i < L->pro.n; ++i)
            if (L->pro.u[i].code == pf::U_MASK_CAUSAL) mask_at = i;
        if (mask_at >= 0) {
            bool ok = true;
            for (int i = 0; i < L->pro.n; ++i) {
                const pf::Uop& u = L->pro.u[i];
                if (u.code == pf::U_SAVE || u.code == pf::U_STORE) ok = false;
                if (i > mask_at && (u.kind == pf::K_FULL || u.kind == pf::K_TMP)) ok = false;
                if (i > mask_at && u.code == pf::U_MOV) ok = false;
            }
            // the kernels skip every full-shape operand beyond the diagonal alike: none may belong to the epilogue,
            // which runs on the masked columns too (softmax gives 0 there, later steps need not)
            for (int f = 0; f < L->n_full; ++f)
                if (L->full_is_epi[f]) ok = false;
            if (ok) L->mask_si = (uint32_t)L->pro.u[mask_at].ival;
        }
        // a mask that is the last prologue step moves into the softmax core ...
        if (L->core == pf::CORE_SOFTMAX && L->mask_si != 0 && mask_at == L->pro.n - 1) {
            L->core_mask = 1;
            L->pro.n -= 1;
        }
        // ... and so does a positive scale right before it: softmax(c * x) = exp(c * (x - max x)) / sum for c > 0
        if (L->core == pf::CORE_SOFTMAX && L->pro.n >= 2 && (L->core_mask || mask_at < 0)) {
            const pf::Uop& u = L->pro.u[L->pro.n - 1];
            if (u.code == pf::U_MUL && u.kind == pf::K_IMM && u.imm > 0.0f && std::isfinite(u.imm)) {
                L->core_scale = u.imm;
                L->pro.n -= 1;
            }
        }
        // with nothing but the load left in front of the core, vectors that are skipped can stand in as -inf
        if (L->core_mask && L->pro.n == 1 && L->pro.u[0].code == pf::U_MOV && L->pro.u[0].kind == pf::K_FULL) L->core_mask = 2;
    }
    return PF_OK;
}

// ---------------------------------------------------------------------------------------------
// recomposition: basic operators -> the composite operator they spell out
// ---------------------------------------------------------------------------------------------
// The paper splits every operator into the four basic kinds and lets the merged gOperator graph find the
// efficient schedule (section 6).  Here the efficient schedules are the hand-written cores, so the inverse step
// runs first: a sub-graph of basic operators that is exactly a softmax, a layer normalisation or an RMS
// normalisation over the last dimension is replaced by that operator when none of its interior values is
// used elsewhere.  The chain then gets the tuned core (scale and causal mask folded into the softmax, load
// skipping, the streaming variant for long rows, catalogue kernels) instead of a generic row program.  The
// rewritten chain computes the same function; anything that does not match stays a row program.
struct Recomposer {
    const pf_chain_desc* d;
    const Checked* c;
    int n_in;
    std::vector<pf_op_desc> ops;
    std::vector<int> uses;
    std::vector<char> dead;

    const pf_op_desc* def(int v, int op) const {  // the operator that defines value v, if it is an `op`
        if (v < n_in || dead[v - n_in]) return nullptr;
        const pf_op_desc* o = &ops[v - n_in];
        return o->op == op ? o : nullptr;
    }
    void count_uses() {
        uses.assign(n_in + (int)ops.size(), 0);
        for (size_t k = 0; k < ops.size(); ++k)
            if (!dead[k])
                for (int s = 0; s < ops[k].n_src; ++s) uses[ops[k].src[s]]++;
        for (int o = 0; o < d->n_outputs; ++o) uses[d->out_value[o]]++;
    }
    bool is_param(int v, int64_t n) const {  // a chain input of shape [n]
        return v < n_in && c->shape[v].size() == 1 && c->shape[v][0] == n;
    }
    void kill(int v) { dead[v - n_in] = 1; }

    // x * rsqrt(mean(x * x) + eps): returns x and eps; `n_val` = the product's value id
    bool match_rms_core(int n_val, int* x_out, float* eps_out, int kill_list[5]) const {
        const pf_op_desc* n = def(n_val, PF_MUL);
        if (!n) return false;
        for (int side = 0; side < 2; ++side) {
            const int x = n->src[side], r_val = n->src[1 - side];
            const pf_op_desc* r = def(r_val, PF_RSQRT);
            if (!r || uses[r_val] != 1) continue;
            const int ve_val = r->src[0];
            const pf_op_desc* ve = def(ve_val, PF_ADDC);
            if (!ve || uses[ve_val] != 1 || !(ve->f[0] >= 0.0f)) continue;
            const int ms_val = ve->src[0];
            const pf_op_desc* ms = def(ms_val, PF_REDUCE_MEAN);
            if (!ms || uses[ms_val] != 1) continue;
            const int sq_val = ms->src[0];
            const pf_op_desc* sq = def(sq_val, PF_MUL);
            if (!sq || uses[sq_val] != 1 || sq->src[0] != x || sq->src[1] != x) continue;
            *x_out = x;
            *eps_out = ve->f[0];
            kill_list[0] = r_val, kill_list[1] = ve_val, kill_list[2] = ms_val, kill_list[3] = sq_val, kill_list[4] = n_val;
            return true;
        }
        return false;
    }

    bool layernorm_at(int k) {  // ((h - mean h) * rsqrt(var + eps)) * gamma + beta
        if (ops[k].op != PF_ADD) return false;
        const int64_t n = c->shape[n_in + k].back();
        for (int side = 0; side < 2; ++side) {
            const int g_val = ops[k].src[side], beta = ops[k].src[1 - side];
            const pf_op_desc* g = def(g_val, PF_MUL);
            if (!g || uses[g_val] != 1 || !is_param(beta, n)) continue;
            for (int gs = 0; gs < 2; ++gs) {
                const int n_val = g->src[gs], gamma = g->src[1 - gs];
                if (!is_param(gamma, n) || n_val < n_in || uses[n_val] != 1) continue;
                int c_val, kl[5];
                float eps;
                if (!match_rms_core(n_val, &c_val, &eps, kl)) continue;
                const pf_op_desc* cen = def(c_val, PF_SUB);
                if (!cen || uses[c_val] != 3) continue;
                const int h = cen->src[0], mu_val = cen->src[1];
                const pf_op_desc* mu = def(mu_val, PF_REDUCE_MEAN);
                if (!mu || uses[mu_val] != 1 || mu->src[0] != h) continue;
                for (int q = 0; q < 5; ++q) kill(kl[q]);
                kill(c_val), kill(mu_val), kill(g_val);
                pf_op_desc o;
                memset(&o, 0, sizeof(o));
                o.op = PF_LAYERNORM, o.n_src = 3, o.src[0] = h, o.src[1] = gamma, o.src[2] = beta, o.f[0] = eps;
                ops[k] = o;
                return true;
            }
        }
        return false;
    }
    bool rmsnorm_at(int k) {  // (x * rsqrt(mean(x * x) + eps)) * gamma
        if (ops[k].op != PF_MUL) return false;
        const int64_t n = c->shape[n_in + k].back();
        for (int gs = 0; gs < 2; ++gs) {
            const int n_val = ops[k].src[gs], gamma = ops[k].src[1 - gs];
            if (!is_param(gamma, n) || n_val < n_in || uses[n_val] != 1) continue;
            int x, kl[5];
            float eps;
            if (!match_rms_core(n_val, &x, &eps, kl)) continue;
            for (int q = 0; q < 5; ++q) kill(kl[q]);
            pf_op_desc o;
            memset(&o, 0, sizeof(o));
            o.op = PF_RMSNORM, o.n_src = 2, o.src[0] = x, o.src[1] = gamma, o.f[0] = eps;
            ops[k] = o;
            return true;
        }
        return false;
    }
    bool softmax_at(int k) {  // exp(x - max x) / sum exp(x - max x)
        if (ops[k].op != PF_DIV) return false;
        const int e_val = ops[k].src[0], s_val = ops[k].src[1];
        const pf_op_desc* sum = def(s_val, PF_REDUCE_SUM);
        const pf_op_desc* e = def(e_val, PF_EXP);
        if (!sum || !e || sum->src[0] != e_val || uses[s_val] != 1 || uses[e_val] != 2) return false;
        const int d_val = e->src[0];
        const pf_op_desc* dif = def(d_val, PF_SUB);
        if (!dif || uses[d_val] != 1) return false;
        const int x = dif->src[0], m_val = dif->src[1];
        const pf_op_desc* m = def(m_val, PF_REDUCE_MAX);
        if (!m || uses[m_val] != 1 || m->src[0] != x) return false;
        kill(s_val), kill(e_val), kill(d_val), kill(m_val);
        pf_op_desc o;
        memset(&o, 0, sizeof(o));
        o.op = PF_SOFTMAX, o.n_src = 1, o.src[0] = x;
        ops[k] = o;
        return true;
    }

    // Returns true and fills *out when at least one sub-graph was replaced.
    bool run(pf_chain_desc* out) {
        n_in = d->n_inputs;
        ops.assign(d->ops, d->ops + d->n_ops);
        dead.assign(ops.size(), 0);
        bool changed = false;
        for (int pass = 0; pass < 3; ++pass)
            for (int k = 0; k < (int)ops.size(); ++k) {
                if (dead[k]) continue;
                count_uses();
                const bool hit = pass == 0 ? layernorm_at(k) : pass == 1 ? softmax_at(k) : rmsnorm_at(k);
                changed = changed || hit;
            }
        if (!changed) return false;
        // compact: drop the dead operators, renumber the values
        std::vector<int> renum(n_in + ops.size(), -1);
        for (int v = 0; v < n_in; ++v) renum[v] = v;
        *out = *d;
        int n = 0;
        for (size_t k = 0; k < ops.size(); ++k) {
            if (dead[k]) continue;
            pf_op_desc o = ops[k];
            for (int s = 0; s < o.n_src; ++s) {
                if (renum[o.src[s]] < 0) return false;  // (cannot happen: interior values have no other use)
                o.src[s] = renum[o.src[s]];
            }
            renum[n_in + (int)k] = n_in + n;
            out->ops[n++] = o;
        }
        out->n_ops = n;
        for (int o = 0; o < d->n_outputs; ++o) {
            if (renum[d->out_value[o]] < 0) return false;
            out->out_value[o] = renum[d->out_value[o]];
        }
        return true;
    }
};

// ---------------------------------------------------------------------------------------------
// spec catalogue (host view)
// ---------------------------------------------------------------------------------------------
struct SpecTable {
    std::vector<pf::SpecDesc> row, group, perm;
    SpecTable() {
#define PF_ADD_SPEC(vec, id_, nf_, nv_, nt_, core_, gamma_, beta_, pro_, epi_)              \
    {                                                                                       \
        pf::SpecDesc s;                                                                     \
        memset(&s, 0, sizeof(s));                                                           \
        s.id = id_; s.nf = nf_; s.nv = nv_; s.nt = nt_; s.core = pf::core_;                 \
        s.gamma = gamma_; s.beta = beta_;                                                   \
        const uint32_t p[] = {0u, pro_};                                                    \
        const uint32_t e[] = {0u, epi_};                                                    \
        s.n_pro = (int)(sizeof(p) / sizeof(p[0])) - 1;                                      \
        s.n_epi = (int)(sizeof(e) / sizeof(e[0])) - 1;                                      \
        for (int i = 0; i < s.n_pro; ++i) s.pro[i] = p[i + 1];                              \
        for (int i = 0; i < s.n_epi; ++i) s.epi[i] = e[i + 1];                              \
        vec.push_back(s);                                                                   \
    }
#define PF_ROW_X(id, nf, nv, nt, core, gamma, beta, pro, epi) PF_ADD_SPEC(row, id, nf, nv, nt, core, gamma, beta, PF_L(pro), PF_L(epi))
        PF_ROW_SPECS(PF_ROW_X)
#define PF_GROUP_X(id, nf, nv, nt, core, gamma, beta, pro, epi) PF_ADD_SPEC(group, id, nf, nv, nt, core, gamma, beta, PF_L(pro), PF_L(epi))
        PF_GROUP_SPECS(PF_GROUP_X)
#define PF_PERM_X(id, nf, nv, nt, core, gamma, beta, pro, epi) PF_ADD_SPEC(perm, id, nf, nv, nt, core, gamma, beta, PF_L(pro), PF_L(epi))
        PF_PERM_SPECS(PF_PERM_X)
    }
};

const SpecTable& spec_table() {
    static const SpecTable t;
    return t;
}

bool list_equal(const pf::Program& p, const uint32_t* list, int n) {
    if (p.n != n) return false;
    for (int i = 0; i < n; ++i) {
        const uint32_t packed = (uint32_t)p.u[i].code | ((uint32_t)p.u[i].kind << 8) | ((uint32_t)p.u[i].slot << 16);
        if (packed != list[i]) return false;
    }
    return true;
}

int match_spec(const std::vector<pf::SpecDesc>& table, const Lowered& L) {
    if (L.general_bcast) return 0;  // catalogue kernels are built without the general broadcast addressing
    if (L.n_out != 1) return 0;
    for (const pf::SpecDesc& s : table) {
        if (s.nf != L.n_full || s.nv != L.n_vec || s.nt != L.n_tmp || s.core != L.core) continue;
        if (s.gamma != L.core_vec[0] || s.beta != L.core_vec[1]) continue;
        if (!list_equal(L.pro, s.pro, s.n_pro) || !list_equal(L.epi, s.epi, s.n_epi)) continue;
        return s.id;
    }
    return 0;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// the plan
// ---------------------------------------------------------------------------------------------
struct pf_plan_s {
    pf_chain_desc desc;
    Lowered low;
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
    int stencil_ks = 3;       // kernel extent of the depthwise convolution
    int row_log2l = 6;        // row family: log2 of the lanes of a wave that share a row
    pf::BcastTerm bcast_host[PF_DEV_MAX_VEC][PF_DEV_MAX_BCAST_TERMS];  // general broadcasting terms, staged on the host
    void* bcast_dev = nullptr;  // ... and their copy in device memory
    bool group_general = false; // group family: groups of any width (general kernels)
    uint32_t dyn_lds = 0;     // group family: dynamic LDS bytes of each launch
    uint32_t ew_total_vecs = 0, ew_vecs_per_row = 0;
    dim3 grid, block;
    dim3 grid2, block2;       // second launch (two-pass group variant)
    uint32_t lds_bytes = 0;
    void* workspace = nullptr;
    uint32_t* ws_error = nullptr;  // device word a kernel sets when one of its bounded waits ran out
    uint64_t workspace_bytes = 0;
    uint64_t in_bytes[PF_MAX_INPUTS];
    uint64_t out_bytes[PF_MAX_OUTPUTS];
    Shape out_shape[PF_MAX_OUTPUTS];
    int n_launches = 1;
    mutable uint32_t epoch = 0;
};

namespace {

constexpr int kStencilRowsHost = 6;   // output rows per strip of the stencil kernels (kStencilRows on the device side)
constexpr int kStencilRows5Host = 4;  // ... for 5 x 5 kernels (kStencilRows5)

int env_int(const char* name, int dflt) {
    const char* s = getenv(name);
    if (!s || !*s) return dflt;
    return atoi(s);
}

// the chain's structure as template arguments for the plan-time specialisation
pf::JitSpec make_jit_spec(const Lowered& L) {
    pf::JitSpec j;
    j.nf = L.n_full;
    j.nv = L.n_vec;
    j.nt = L.n_tmp;
    j.core = L.core;
    j.gamma = L.core_vec[0];
    j.beta = L.core_vec[1];
    j.flags = L.general_bcast ? 1 : 0;
    for (int i = 0; i < L.pro.n; ++i)
        j.pro.push_back((uint32_t)L.pro.u[i].code | ((uint32_t)L.pro.u[i].kind << 8) | ((uint32_t)L.pro.u[i].slot << 16));
    for (int i = 0; i < L.epi.n; ++i)
        j.epi.push_back((uint32_t)L.epi.u[i].code | ((uint32_t)L.epi.u[i].kind << 8) | ((uint32_t)L.epi.u[i].slot << 16));
    return j;
}

// Plan-time specialisation needs the device (the compiled kernel is loaded onto it).
bool jit_possible(int device) {
    if (!pf::jit_enabled()) return false;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device < 0 || device >= n) return false;
    return hipSetDevice(device) == hipSuccess;
}

pf::FastDiv make_fastdiv(uint32_t d);

pf_status fill_vec_args(pf_plan_s* p, const Checked& c) {
    const Lowered& L = p->low;
    const int es = dtype_size(L.main_dtype);
    for (int v = 0; v < L.n_vec; ++v) {
        const int in = L.vec_input[v];
        const int64_t n = numel(c.shape[in]);
        const int64_t inner = (L.vec_is_epi[v] ? L.post_shape : L.pre_shape).back();
        pf::VecArg& va = p->args.vec[v];
        va.ptr = nullptr;
        va.dtype = L.main_dtype;
        va.pad = 0;
        va.terms = nullptr;
        if (n > 0xffffffffLL) return fail(PF_ERR_UNSUPPORTED, "broadcast input %d too large", in);
        va.numel = (uint32_t)n;
        va.period_rows = 1;
        va.n_terms = 0;
        va.col_bcast = 0;
        if (n == 1) continue;
        const Shape& os = c.shape[in];
        const Shape& ps = L.vec_partner[v];
        if (!ps.empty() && !is_trailing(os, ps)) {
            // ---- general broadcasting: extents of 1 anywhere.  One term per run of kept row dimensions.
            const Shape& region = L.vec_is_epi[v] ? L.post_shape : L.pre_shape;
            if (!broadcasts_onto(os, ps) || ps.back() != inner || numel(ps) != numel(region))
                return fail(PF_ERR_UNSUPPORTED, "broadcast input %d: its shape does not broadcast over the kernel's rows", in);
            const size_t rank = ps.size(), off = rank - os.size();
            auto op_extent = [&](size_t i) { return i < off ? (int64_t)1 : os[i - off]; };
            p->low.general_bcast = true;
            va.col_bcast = (op_extent(rank - 1) == 1 && inner != 1) ? 1u : 0u;
            if (!va.col_bcast && (inner * es) % 16 != 0) p->ragged = true;
            int64_t div = 1, stride = 1;  // rows of the value / operand rows inside the dimension being looked at
            bool in_run = false;
            for (size_t q = rank - 1; q-- > 0;) {
                const int64_t e = ps[q], oe = op_extent(q);
                if (e == 1) continue;
                if (oe == e) {
                    if (in_run) {
                        pf::BcastTerm& t = p->bcast_host[v][va.n_terms - 1];
                        t.mod = make_fastdiv((uint32_t)(t.mod.d * e));
                    } else {
                        if (va.n_terms == PF_DEV_MAX_BCAST_TERMS)
                            return fail(PF_ERR_UNSUPPORTED, "broadcast input %d: more than %d separate runs of kept dimensions", in, PF_DEV_MAX_BCAST_TERMS);
                        pf::BcastTerm& t = p->bcast_host[v][va.n_terms++];
                        memset(&t, 0, sizeof(t));
                        t.div = make_fastdiv((uint32_t)div);
                        t.mod = make_fastdiv((uint32_t)e);
                        t.stride = (uint32_t)stride;
                        in_run = true;
                    }
                    stride *= e;
                } else {
                    in_run = false;
                }
                div *= e;
                if (div > 0xffffffffLL) return fail(PF_ERR_UNSUPPORTED, "broadcast input %d: too many rows", in);
            }
            if (va.n_terms == 0) {
                // nothing kept among the row dimensions: one operand row for every row of the value
                pf::BcastTerm& t = p->bcast_host[v][va.n_terms++];
                memset(&t, 0, sizeof(t));
                t.div = make_fastdiv(1u);
                t.mod = make_fastdiv(1u);
                t.stride = 0;
            }
            continue;
        }
        if ((n * es) % 16 != 0) p->ragged = true;  // gathered element by element (row and element-wise families)
        if (n >= inner) {
            if (n % inner != 0) return fail(PF_ERR_UNSUPPORTED, "broadcast input %d does not tile the kernel's rows", in);
            va.period_rows = (uint32_t)(n / inner);
        } else if (inner % n != 0) {
            return fail(PF_ERR_UNSUPPORTED, "broadcast input %d does not tile the kernel's rows", in);
        }
    }
    if (L.general_bcast) {
        if (hipSetDevice(p->device) != hipSuccess || hipMalloc(&p->bcast_dev, sizeof(p->bcast_host)) != hipSuccess)
            return fail(PF_ERR_NOMEM, "device memory for broadcast terms");
        if (hipMemcpy(p->bcast_dev, p->bcast_host, sizeof(p->bcast_host), hipMemcpyHostToDevice) != hipSuccess)
            return fail(PF_ERR_HIP, "upload of broadcast terms failed");
        for (int v = 0; v < L.n_vec; ++v)
            if (p->args.vec[v].n_terms)
                p->args.vec[v].terms = static_cast<const pf::BcastTerm*>(p->bcast_dev) + (size_t)v * PF_DEV_MAX_BCAST_TERMS;
    }
    return PF_OK;
}

pf_status plan_row(pf_plan_s* p, int forced_variant) {
    const Lowered& L = p->low;
    const int es = dtype_size(L.main_dtype);
    const int vec = 16 / es;
    const int64_t n = L.pre_shape.back();
    const int64_t rows = numel(L.pre_shape) / n;
    if ((n * es) % 16 != 0) p->ragged = true;
    if (rows > 0xffffffffLL || n > 0x7fffffffLL) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the row family");
    const int64_t vpr = (n + vec - 1) / vec;
    // candidates (waves per row, vectors per lane); prefer little idle lanes, a statically specialised
    // kernel, small workgroups, a single wave per row
    const bool reduce_only = L.core == pf::CORE_REDUCE_SUM || L.core == pf::CORE_REDUCE_MAX || L.core == pf::CORE_REDUCE_MEAN;
    const int matched = (!reduce_only && !p->ragged && env_int("PF_NO_STATIC", 0) == 0) ? match_spec(spec_table().row, L) : 0;
    // no catalogue entry: the same kernel templates are specialised for this chain's structure at plan time
    // (also catalogue entries in launch shapes that were not instantiated at build time)
    const bool jit_ok = jit_possible(p->device);
    auto have_static = [&](int k, int rpw, bool wave_rows, unsigned threads) {
        if (matched && pf::row_static_available(matched, k, rpw, wave_rows, threads)) return true;
        if (!jit_ok) return false;
        return (k == 1 || k == 2 || k == 4) && (rpw == 1 || rpw == 2 || rpw == 4) && k * rpw <= 4 && (wave_rows || rpw == 1) &&
               threads <= 1024;
    };
    int best_wpr = 0, best_k = 0;
    long best_score = -1;
    const int ks[3] = {1, 2, 4};
    for (int ki = 0; ki < 3 && forced_variant != PF_VARIANT_ROW_STREAM; ++ki) {
        const int k = ks[ki];
        const int64_t wpr = (vpr + 64 * k - 1) / (64 * k);
        if (wpr > 16) continue;
        if (forced_variant == PF_VARIANT_ROW_WAVE && wpr != 1) continue;
        if (forced_variant == PF_VARIANT_ROW_BLOCK && wpr == 1) continue;
        const double waste = 1.0 - (double)vpr / (double)(wpr * 64 * k);
        const unsigned threads = 64u * (unsigned)wpr * (wpr >= 4 ? 1u : (unsigned)(4 / wpr));
        long score = (waste > 0.26 ? 4000 : (waste > 0.13 ? 2000 : 0)) + (wpr > 4 ? 1000 : 0) + (wpr > 1 ? 100 : 0) + k;
        if ((matched || jit_ok) && !have_static(k, 1, wpr == 1, threads)) score += 500;
        if (best_score < 0 || score < best_score) {
            best_score = score;
            best_wpr = (int)wpr;
            best_k = k;
        }
    }
    p->reduce_only = reduce_only;
    if (p->reduce_only) {
        // the epilogue runs on one value per row: no tensor operands there
        for (int i = 0; i < L.epi.n; ++i)
            if (L.epi.u[i].kind != pf::K_NONE && L.epi.u[i].kind != pf::K_IMM)
                return fail(PF_ERR_UNSUPPORTED, "after a keep-dim reduction only unary and constant steps are implemented");
        for (int i = 0; i < L.epi.n; ++i)
            if (L.epi.u[i].code == pf::U_MASK_CAUSAL || L.epi.u[i].code == pf::U_STORE)
                return fail(PF_ERR_UNSUPPORTED, "after a keep-dim reduction only unary and constant steps are implemented");
        if (L.n_out != 1) return fail(PF_ERR_UNSUPPORTED, "a keep-dim reduction has one output");
    }
    p->family = PF_FAMILY_ROW;
    p->args.n_inner = (uint32_t)n;
    p->args.rows = (uint64_t)rows;
    if (best_score < 0 && L.core == pf::CORE_ROWPROG)
        return fail(PF_ERR_UNSUPPORTED, "chains with in-line reductions need rows that fit one workgroup's registers (row length %lld)", (long long)n);
    if (best_score < 0) {
        // Rows longer than a workgroup keeps in registers (or on request): the streaming variant, a workgroup
        // per row, two walks over the row.
        if (forced_variant >= 0 && forced_variant != PF_VARIANT_ROW_STREAM)
            return fail(PF_ERR_UNSUPPORTED, "variant %d is not possible for row length %lld", forced_variant, (long long)n);
        if (rows > 0x7fffffffLL || n * es > 0x7fffffffLL) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the streaming row variant");
        p->variant = PF_VARIANT_ROW_STREAM;
        p->k = 2;
        p->spec_id = 0;
        p->row.waves_per_row = 8;
        p->row.rows_per_block = 1;
        p->row.rows_per_wave = 1;
        p->block = dim3(512);
        p->grid = dim3((uint32_t)rows);
        p->lds_bytes = (2 * 16 + 8 * 3) * 4;
        if (jit_ok) {
            std::string err;
            p->jit_fn = pf::jit_row_stream_kernel(p->device, L.main_dtype, p->ragged, make_jit_spec(L), &err);
            if (p->jit_fn) p->spec_id = pf::kSpecJit;
            else if (env_int("PF_LOG", 0)) fprintf(stderr, "[pf] plan-time specialisation unavailable, using the interpreter: %s\n", err.c_str());
        }
        return PF_OK;
    }
    p->variant = best_wpr == 1 ? PF_VARIANT_ROW_WAVE : PF_VARIANT_ROW_BLOCK;
    p->k = best_k;
    p->row.waves_per_row = (uint32_t)best_wpr;
    p->row.rows_per_block = best_wpr >= 4 ? 1u : (uint32_t)(4 / best_wpr);
    p->row.rows_per_wave = 1;
    // Rows per wave: a wave that owns short rows takes several at once, so that it has about 4 KB of loads
    // in flight (what it takes to cover the HBM latency at full occupancy), as long as enough waves remain
    // (16 per SIMD) to fill the device evenly and a specialised kernel exists for the combination.
    if (best_wpr == 1 && (matched || jit_ok) && L.n_out == 1) {
        const int64_t bytes_per_row_in_flight = (int64_t)L.n_full * best_k * 1024;
        int rpw = 1;
        while (rpw < 4 && bytes_per_row_in_flight * rpw < 4096 && best_k * rpw * 2 <= 4 && rows / (rpw * 2) >= 16384) rpw *= 2;
        const int forced = env_int("PF_ROWS_PER_WAVE", 0);
        if (forced > 0) rpw = forced;
        if (rpw > 1 && have_static(best_k, rpw, true, 256)) p->row.rows_per_wave = (uint32_t)rpw;
    }
    p->block = dim3(64u * best_wpr * p->row.rows_per_block);
    p->lds_bytes = best_wpr > 1 ? 2 * 16 * 4 : 0;
    // Short rows (at most 32 vectors): several rows side by side in a wave, 8 / 16 / 32 lanes each, instead of
    // one row on a wave whose other lanes idle.  Exists in plan-time specialised form only.
    int log2l = 6;
    if (best_wpr == 1 && best_k == 1 && vpr <= 32 && jit_ok && !reduce_only && L.n_out == 1 && rows >= 256) {
        log2l = 3;
        while ((1 << log2l) < vpr) ++log2l;
    }
    {
        const int forced_l = env_int("PF_ROW_LOG2_LANES", 0);
        if (forced_l >= 3 && forced_l <= 6 && best_wpr == 1 && best_k == 1 && vpr <= (1 << forced_l) && jit_ok && !reduce_only && L.n_out == 1) log2l = forced_l;
    }
    p->row_log2l = log2l;
    p->spec_id = (log2l == 6 && matched && pf::row_static_available(matched, p->k, (int)p->row.rows_per_wave, best_wpr == 1, p->block.x)) ? matched : 0;
    if (!p->spec_id && jit_ok && have_static(p->k, (int)p->row.rows_per_wave, best_wpr == 1, p->block.x)) {
        std::string err;
        if (reduce_only) p->jit_fn = pf::jit_row_reduce_kernel(p->device, L.main_dtype, p->k, p->ragged, make_jit_spec(L), &err);
        else p->jit_fn = pf::jit_row_kernel(p->device, L.main_dtype, p->k, (int)p->row.rows_per_wave, best_wpr == 1, p->ragged,
                                       p->block.x <= 256 ? 256 : 1024, log2l, make_jit_spec(L), &err);
        if (p->jit_fn) p->spec_id = pf::kSpecJit;
        else if (env_int("PF_LOG", 0)) fprintf(stderr, "[pf] plan-time specialisation unavailable, using the interpreter: %s\n", err.c_str());
    }
    if (!p->spec_id) {
        p->row.rows_per_wave = 1;
        p->row_log2l = 6;
    }
    {
        const int64_t rows_per_block = (int64_t)p->row.rows_per_block * p->row.rows_per_wave * (64 >> p->row_log2l);
        p->grid = dim3((uint32_t)((rows + rows_per_block - 1) / rows_per_block));
    }
    return PF_OK;
}

pf_status plan_ew(pf_plan_s* p) {
    const Lowered& L = p->low;
    const int es = dtype_size(L.main_dtype);
    const int vec = 16 / es;
    const int64_t n = L.pre_shape.back();
    const int64_t total = numel(L.pre_shape);
    if ((n * es) % 16 != 0) p->ragged = true;
    if (p->ragged) {
        for (int i = 0; i < L.pro.n; ++i)
            if (L.pro.u[i].code == pf::U_MASK_CAUSAL)
                return fail(PF_ERR_UNSUPPORTED, "a causal mask without a row reduction needs rows of whole 16-byte vectors");
    }
    const int64_t total_vecs = (total + vec - 1) / vec;
    if (total_vecs > 0xffffffffLL) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the element-wise family");
    p->family = PF_FAMILY_ELEMENTWISE;
    p->variant = PF_VARIANT_EW_FLAT;
    p->k = 1;
    p->ew_total_vecs = (uint32_t)total_vecs;
    p->ew_vecs_per_row = (uint32_t)std::max<int64_t>(1, n / vec);
    p->block = dim3(256);
    p->grid = dim3((uint32_t)((total_vecs + 256 * p->k - 1) / (256 * p->k)));
    p->args.n_inner = (uint32_t)n;
    p->args.rows = (uint64_t)(total / n);
    if (jit_possible(p->device)) {
        std::string err;
        p->jit_fn = pf::jit_ew_kernel(p->device, L.main_dtype, p->k, p->ragged, make_jit_spec(L), &err);
        if (p->jit_fn) p->spec_id = pf::kSpecJit;
        else if (env_int("PF_LOG", 0)) fprintf(stderr, "[pf] plan-time specialisation unavailable, using the interpreter: %s\n", err.c_str());
    }
    return PF_OK;
}

}  // namespace

namespace {

pf::FastDiv make_fastdiv(uint32_t d) {
    pf::FastDiv f;
    f.d = d;
    if (d <= 1) {
        f.m = 0; f.s1 = 0; f.s2 = 0;
        return f;
    }
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    f.m = (uint32_t)((((1ull << 32) * ((1ull << l) - d)) / d) + 1);
    f.s1 = 1;
    f.s2 = l - 1;
    return f;
}

// ---- transpose family
pf_status plan_perm(pf_plan_s* p, int forced_variant) {
    const Lowered& L = p->low;
    const int es = dtype_size(L.main_dtype);
    const int vec = 16 / es;
    const Shape& in = L.pre_shape;
    const int rank = (int)in.size();
    if (numel(in) > 0xffffffffLL) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the transpose family");
    // extents that are not whole vectors on either side (or a broadcast operand that is not): element-granular kernels
    const bool ragged = p->ragged || (L.pre_shape.back() * es) % 16 != 0 || (L.post_shape.back() * es) % 16 != 0;
    p->ragged = ragged;
    if (ragged && (L.pre_shape.back() == 1 || L.post_shape.back() == 1))
        return fail(PF_ERR_UNSUPPORTED, "permutations of tensors whose innermost extent is 1 are not implemented (reshape it away)");
    for (int i = 0; i < L.pro.n; ++i)
        if (L.pro.u[i].code == pf::U_STORE) return fail(PF_ERR_UNSUPPORTED, "secondary outputs are not implemented in the transpose family");
    for (int i = 0; i < L.epi.n; ++i)
        if (L.epi.u[i].code == pf::U_STORE) return fail(PF_ERR_UNSUPPORTED, "secondary outputs are not implemented in the transpose family");
    // input strides
    std::vector<int64_t> istr(rank);
    int64_t acc = 1;
    for (int k = rank - 1; k >= 0; --k) { istr[k] = acc; acc *= in[k]; }
    // output dims in order, dropping extent-1 dims and merging dims that stay adjacent
    struct Dim { int64_t extent, in_stride; };
    std::vector<Dim> od;
    for (int q = 0; q < rank; ++q) {
        const int src = L.perm[q];
        if (in[src] == 1) continue;
        // (ragged: dimensions are not merged, so that the innermost dimension of each side is one the vectors of
        // broadcast operands and the partial last vector can be told from)
        if (!ragged && !od.empty() && od.back().in_stride == in[src] * istr[src]) {
            od.back().extent *= in[src];
            od.back().in_stride = istr[src];
        } else {
            od.push_back(Dim{in[src], istr[src]});
        }
    }
    if (od.empty()) od.push_back(Dim{1, 1});
    const int m = (int)od.size();
    pf::PermGeom& g = p->permg;
    memset(&g, 0, sizeof(g));
    g.in_n_inner = (uint32_t)L.pre_shape.back();
    g.out_n_inner = (uint32_t)L.post_shape.back();
    g.div_in_inner = make_fastdiv(g.in_n_inner);
    g.div_out_inner = make_fastdiv(g.out_n_inner);
    g.total_vecs = (uint32_t)(numel(in) / vec);
    for (int f = 0; f < L.n_full; ++f) if (L.full_is_epi[f]) g.epi_full_mask |= 1u << f;
    for (int v = 0; v < L.n_vec; ++v) if (L.vec_is_epi[v]) g.epi_vec_mask |= 1u << v;
    // output strides of the merged dims
    std::vector<int64_t> ostr(m);
    acc = 1;
    for (int q = m - 1; q >= 0; --q) { ostr[q] = acc; acc *= od[q].extent; }
    p->family = PF_FAMILY_TRANSPOSE;
    p->spec_id = (env_int("PF_NO_STATIC", 0) || ragged) ? 0 : match_spec(spec_table().perm, L);
    p->args.n_inner = g.in_n_inner;
    p->args.rows = (uint64_t)(numel(in) / g.in_n_inner);

    if (od.back().in_stride != 1) {
        // ---- the innermost dimension changes: square tiles over (input-innermost I, output-innermost O)
        if (forced_variant >= 0 && forced_variant != PF_VARIANT_T_TILE)
            return fail(PF_ERR_UNSUPPORTED, "variant %d is not implemented for this permutation", forced_variant);
        int qi = -1;
        for (int q = 0; q < m; ++q)
            if (od[q].in_stride == 1) qi = q;
        if (qi < 0) return fail(PF_ERR_UNSUPPORTED, "internal: no contiguous input dimension");
        const int64_t n_i = od[qi].extent, n_o = od.back().extent;
        if (!ragged && ((n_i * es) % 16 != 0 || (n_o * es) % 16 != 0))
            return fail(PF_ERR_ALIGNMENT, "transposed extents (%lld, %lld) are not multiples of 16 bytes", (long long)n_i, (long long)n_o);
        const bool pro_trivial = L.pro.n == 1 && L.pro.u[0].code == pf::U_MOV && L.pro.u[0].kind == pf::K_FULL && L.pro.u[0].slot == 0;
        if (es == 2 && !pro_trivial && L.epi.n != 0)
            return fail(PF_ERR_UNSUPPORTED, "16-bit chains may compute on one side of an innermost-changing permutation only");
        if (L.n_full < 1 || L.pro.n < 1 || L.pro.u[0].code != pf::U_MOV || L.pro.u[0].kind != pf::K_FULL || L.pro.u[0].slot != 0)
            return fail(PF_ERR_UNSUPPORTED, "the permuted value must start from a full-shape input");
        const int64_t te = 8 * vec;
        int r = 0;
        uint64_t total_tiles = 1;
        for (int q = 0; q < m - 1; ++q) {
            if (q == qi) continue;
            g.extent[r] = (uint32_t)od[q].extent;
            g.in_stride[r] = (uint32_t)od[q].in_stride;
            g.out_stride[r] = (uint32_t)ostr[q];
            ++r;
        }
        g.extent[r] = (uint32_t)((n_i + te - 1) / te);
        g.in_stride[r] = (uint32_t)te;
        g.out_stride[r] = (uint32_t)(te * ostr[qi]);
        ++r;
        g.extent[r] = (uint32_t)((n_o + te - 1) / te);
        g.in_stride[r] = (uint32_t)(te * od.back().in_stride);
        g.out_stride[r] = (uint32_t)te;
        ++r;
        g.rank = r;
        for (int q = 0; q < r; ++q) {
            g.div[q] = make_fastdiv(g.extent[q]);
            total_tiles *= g.extent[q];
        }
        if (total_tiles > 0x7fffffffull) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the transpose family");
        g.total_vecs = (uint32_t)total_tiles;
        g.tile_a = (uint32_t)n_i;
        g.tile_b = (uint32_t)n_o;
        g.t_in_stride_o = (uint32_t)od.back().in_stride;
        g.t_out_stride_i = (uint32_t)ostr[qi];
        p->variant = PF_VARIANT_T_TILE;
        p->k = vec;
        p->block = dim3(256);
        p->grid = dim3((uint32_t)((total_tiles + 3) / 4));
        p->lds_bytes = 0;
        if (!p->spec_id && jit_possible(p->device)) {
            std::string err;
            p->jit_fn = pf::jit_perm_kernel(p->device, L.main_dtype, p->variant, p->k, ragged, make_jit_spec(L), &err);
            if (p->jit_fn) p->spec_id = pf::kSpecJit;
            else if (env_int("PF_LOG", 0)) fprintf(stderr, "[pf] plan-time specialisation unavailable, using the interpreter: %s\n", err.c_str());
        }
        return PF_OK;
    }
    const int64_t inner = od.back().extent;
    if (!ragged && (inner * es) % 16 != 0) return fail(PF_ERR_ALIGNMENT, "innermost run of %lld elements is not a multiple of 16 bytes", (long long)inner);
    const int64_t inner_vecs = (inner + vec - 1) / vec;  // the last one partial when ragged
    if (ragged) {
        const int64_t tv = numel(in) / inner * inner_vecs;
        if (tv > 0xffffffffLL) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the transpose family");
        g.total_vecs = (uint32_t)tv;
    }
    // LDS-staged variant: [batch, A, B, inner] -> [batch, B, A, inner]
    bool lds_ok = false;
    uint32_t ta = 0, tb = 0;
    int ia = -1, ib = -1;  // output positions of B (first) and A (second): out = [batch?, B, A, inner]
    if (!ragged && (m == 3 || m == 4)) {
        ib = m - 3;
        ia = m - 2;
        const Dim& B = od[ib];
        const Dim& A = od[ia];
        // in the input A is outside B: stride(A) == extent(B) * stride(B), stride(B) == inner
        const bool pattern = B.in_stride == inner && A.in_stride == B.extent * inner && (m == 3 || od[0].in_stride == A.extent * A.in_stride);
        if (pattern) {
            const int64_t inner_v = inner / vec;
            // tile: tb inner rows of B per input run, ta of A per output run; keep the tile near 32 KB
            for (int64_t cand_b = std::min<int64_t>(B.extent, 32); cand_b >= 1 && !lds_ok; --cand_b) {
                if (B.extent % cand_b != 0) continue;
                for (int64_t cand_a = 32; cand_a >= 2; --cand_a) {
                    if (A.extent % cand_a != 0) continue;
                    const int64_t bytes = cand_a * (cand_b * inner_v + 16) * 16;
                    if (bytes > 48 * 1024 || cand_a * cand_b * inner_v < 256) continue;
                    ta = (uint32_t)cand_a; tb = (uint32_t)cand_b; lds_ok = true;
                    break;
                }
            }
        }
    }
    int variant = forced_variant >= 0 ? forced_variant : PF_VARIANT_T_ROWS;
    if (variant == PF_VARIANT_T_LDS_ROWS && !lds_ok)
        return fail(PF_ERR_UNSUPPORTED, "the LDS-staged variant needs a [.., A, B, inner] -> [.., B, A, inner] permutation with tileable extents");
    if (variant != PF_VARIANT_T_ROWS && variant != PF_VARIANT_T_LDS_ROWS)
        return fail(PF_ERR_UNSUPPORTED, "variant %d is not implemented for this permutation", variant);
    p->variant = variant;
    if (variant == PF_VARIANT_T_LDS_ROWS) {
        const Dim& B = od[ib];
        const Dim& A = od[ia];
        const int64_t batch = m == 4 ? od[0].extent : 1;
        g.rank = 4;
        g.extent[0] = (uint32_t)batch;
        g.extent[1] = (uint32_t)(A.extent / ta);
        g.extent[2] = (uint32_t)(B.extent / tb);
        g.extent[3] = (uint32_t)(inner / vec);
        g.in_stride[0] = m == 4 ? (uint32_t)od[0].in_stride : 0u;
        g.in_stride[1] = (uint32_t)A.in_stride;
        g.in_stride[2] = (uint32_t)B.in_stride;
        g.in_stride[3] = 1;
        g.out_stride[0] = m == 4 ? (uint32_t)ostr[0] : 0u;
        g.out_stride[1] = (uint32_t)ostr[ia];
        g.out_stride[2] = (uint32_t)ostr[ib];
        g.out_stride[3] = 1;
        g.tile_a = ta;
        g.tile_b = tb;
        {
            // pad the staged line so that stepping one line advances the bank index (256 bytes of bank space =
            // 16 vectors) by one inner row: pitch = row (mod 16 vectors) must equal inner (mod 16 vectors)
            const int64_t inner_v = inner / vec, row_v = tb * inner_v;
            const int64_t pad = (((inner_v - row_v) % 16) + 16) % 16;
            g.lds_pitch = (uint32_t)(row_v + (env_int("PF_LDS_PAD", -1) >= 0 ? env_int("PF_LDS_PAD", 0) : pad));
        }
        p->k = 1;
        p->block = dim3(256);
        p->grid = dim3((uint32_t)(batch * (A.extent / ta) * (B.extent / tb)));
        p->lds_bytes = (uint32_t)(ta * g.lds_pitch * 16);
    } else {
        if (m > PF_DEV_MAX_RANK) return fail(PF_ERR_UNSUPPORTED, "too many dimensions");
        g.rank = m;
        for (int q = 0; q < m; ++q) {
            g.extent[q] = (uint32_t)(q == m - 1 ? inner_vecs : od[q].extent);
            g.in_stride[q] = (uint32_t)od[q].in_stride;
            g.out_stride[q] = (uint32_t)ostr[q];
            g.div[q] = make_fastdiv(g.extent[q]);
        }
        p->k = (g.total_vecs >= 65536u && !ragged) ? 2 : 1;
        g.tile_a = (uint32_t)inner;  // (ragged kernels: length of the innermost run)
        p->block = dim3(256);
        p->grid = dim3((g.total_vecs + 256u * p->k - 1) / (256u * p->k));
        p->lds_bytes = 0;
    }
    if (!p->spec_id && jit_possible(p->device)) {
        std::string err;
        p->jit_fn = pf::jit_perm_kernel(p->device, L.main_dtype, p->variant, p->k, ragged, make_jit_spec(L), &err);
        if (p->jit_fn) p->spec_id = pf::kSpecJit;
        else if (env_int("PF_LOG", 0)) fprintf(stderr, "[pf] plan-time specialisation unavailable, using the interpreter: %s\n", err.c_str());
    }
    return PF_OK;
}

// ---- group family
pf_status plan_group(pf_plan_s* p, int forced_variant) {
    const Lowered& L = p->low;
    const int es = dtype_size(L.main_dtype);
    const int vec = 16 / es;
    const Shape& sh = L.pre_shape;
    const int64_t samples = sh[0], C = sh.back();
    const int64_t hw = numel(sh) / (samples * C);
    const int64_t G = L.groups;
    if ((C * es) % 16 != 0) return fail(PF_ERR_ALIGNMENT, "channel count %lld is not a multiple of 16 bytes", (long long)C);
    if (p->ragged) return fail(PF_ERR_ALIGNMENT, "a broadcast input of the group family is not a multiple of 16 bytes");
    const int64_t cpg = C / G;
    const int64_t vpg = cpg / vec, cv = C / vec;
    // Groups that are a power-of-two number of whole vectors take the kernels' shuffle-tree path; any other width
    // takes the general one (per-element sums, parts merged through LDS).
    const bool general = cpg % vec != 0 || (vpg & (vpg - 1)) != 0 || vpg > 64 || env_int("PF_GROUP_GENERAL", 0) != 0;
    if (general && G > 512) return fail(PF_ERR_UNSUPPORTED, "more than 512 groups");
    if (samples * hw > 0xffffffffLL || samples > 65535) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the group family");
    for (int i = 0; i < L.pro.n; ++i)
        if (L.pro.u[i].code == pf::U_STORE) return fail(PF_ERR_UNSUPPORTED, "secondary outputs are not implemented in the group family");
    for (int i = 0; i < L.epi.n; ++i)
        if (L.epi.u[i].code == pf::U_STORE) return fail(PF_ERR_UNSUPPORTED, "secondary outputs are not implemented in the group family");
    pf::GroupGeom& g = p->group;
    memset(&g, 0, sizeof(g));
    g.samples = (uint32_t)samples;
    g.hw = (uint32_t)hw;
    g.channels = (uint32_t)C;
    g.groups = (uint32_t)G;
    g.cv = (uint32_t)cv;
    g.vpg = (uint32_t)vpg;
    g.log2_vpg = 0;
    while ((1u << g.log2_vpg) < g.vpg) ++g.log2_vpg;
    g.div_cv = make_fastdiv(g.cv);
    g.cpg = (uint32_t)cpg;
    g.div_cpg = make_fastdiv(g.cpg);
    g.parts = 1;
    for (int64_t v = 0; v < cv; ++v) g.parts = std::max<uint32_t>(g.parts, (uint32_t)((v * vec + vec - 1) / cpg - (v * vec) / cpg + 1));
    const uint32_t gen_lds = general ? 512u * g.parts * 3u * (uint32_t)sizeof(float) : 0u;
    p->group_general = general;
    // 2: statistics straight from the packed 16-bit pairs (needs pairs that never straddle groups and nothing but the
    // load in front of the normalisation; the kernel checks the rest at compile time)
    const int gen_parts = !general ? 0 : ((cpg % 2 == 0 && L.main_dtype != PF_F32 && L.pro.n == 1) ? 2 : 1);
    g.spin_limit = (uint32_t)env_int("PF_GROUP_SPIN_LIMIT", 1 << 22);  // polls before a wait gives up (tests force it small)
    p->family = PF_FAMILY_GROUP;
    p->spec_id = (env_int("PF_NO_STATIC", 0) || general) ? 0 : match_spec(spec_table().group, L);

    hipDeviceProp_t prop;
    if (hipSetDevice(p->device) != hipSuccess || hipGetDeviceProperties(&prop, p->device) != hipSuccess)
        return fail(PF_ERR_HIP, "cannot query device %d (the group family needs the device at plan time)", p->device);
    const int n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

    // Workgroups of 512 threads; a tile is NV position steps of 512 / cv positions each.
    const uint32_t threads = 512;
    if (g.cv > threads) return fail(PF_ERR_UNSUPPORTED, "more than %d channels", (int)threads * vec);
    g.pos_per_step = threads / g.cv;
    g.vec_per_channel = 1;
    for (int v = 0; v < L.n_vec; ++v)
        if (p->args.vec[v].numel > (uint32_t)C || p->args.vec[v].n_terms != 0) g.vec_per_channel = 0;
    // lanes that share a group when partials are merged: as many as fit, a power of two, at most 64
    g.lanes_per_group = 1;
    while (g.lanes_per_group < 64u && g.lanes_per_group * 2u * g.groups <= threads) g.lanes_per_group *= 2u;

    auto tiling = [&](int nv_c, uint32_t* bps_out) {
        const uint32_t ppb = (uint32_t)nv_c * g.pos_per_step;
        *bps_out = (uint32_t)((hw + ppb - 1) / ppb);
    };
    // The largest tile that still leaves enough workgroups.  The two-launch variant wants two per compute unit.  The
    // one-launch variant does better with fewer, larger tiles, down to about two for every three compute units: all
    // of them are resident at once, and fewer tiles mean fewer words in the exchange (measured: [16,32,32,640]
    // 24.6 us with 688 tiles of 4 steps, 16.9 us with 176 of 16; [16,64,64,128] 16.5 -> 13.2 us).
    const bool fused_candidate = L.n_full == 1 && g.vec_per_channel && forced_variant != PF_VARIANT_GROUP_TWO_PASS &&
                                 (p->spec_id != 0 || jit_possible(p->device));
    const uint64_t min_tiles = fused_candidate ? ((uint64_t)n_cu * 2 + 2) / 3 : 2 * (uint64_t)n_cu;
    const int cands[3] = {16, 8, 4};
    const int forced_nv = env_int("PF_GROUP_NV", 0);
    int nv = 0;
    uint32_t bps = 0;
    for (int ci = 0; ci < 3 && nv == 0; ++ci) {
        if (forced_nv && cands[ci] != forced_nv) continue;
        if (general && !(gen_parts == 2 && jit_possible(p->device)) && cands[ci] == 16 && !forced_nv) continue;  // (16 vectors fit the general kernels' registers only with packed statistics)
        uint32_t b;
        tiling(cands[ci], &b);
        if ((uint64_t)b * samples >= min_tiles || ci == 2 || forced_nv) {
            nv = cands[ci];
            bps = b;
        }
    }
    if (nv == 0) return fail(PF_ERR_INVALID_ARG, "PF_GROUP_NV must be 4, 8 or 16");
    const uint64_t tiles = (uint64_t)bps * samples;
    if (tiles > 0x7fffffffull) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the group family");

    // resident variant: catalogue entry, one full operand, per-channel broadcast operands only, and a grid the
    // device holds at once
    const bool jit_ok = p->spec_id == 0 && jit_possible(p->device);
    const pf::JitSpec jspec = make_jit_spec(L);
    std::string jit_err;
    hipFunction_t fused_fn = nullptr;
    bool resident_ok = L.n_full == 1 && g.vec_per_channel && forced_variant != PF_VARIANT_GROUP_TWO_PASS;
    if (resident_ok && p->spec_id == 0) {
        // not in the catalogue: the fused kernel exists only if it can be specialised now
        fused_fn = jit_ok ? pf::jit_group_kernel(p->device, L.main_dtype, nv, 0, gen_parts, jspec, &jit_err) : nullptr;
        if (!fused_fn) resident_ok = false;
    }
    uint32_t res_grid = 0;
    if (resident_ok) {
        const int per_cu = fused_fn ? pf::jit_blocks_per_cu(fused_fn, (int)threads, gen_lds)
                                    : pf::group_resident_blocks_per_cu(p->spec_id, L.main_dtype, nv, (int)threads);
        const uint64_t cap = (uint64_t)std::max(per_cu, 0) * n_cu;
        uint64_t grid = std::min<uint64_t>(tiles, cap);
        grid = grid / bps * bps;  // whole samples per round, so every wait is for co-resident workgroups
        if (grid < bps) resident_ok = false;
        else res_grid = (uint32_t)grid;
    }
    int variant = forced_variant >= 0 ? forced_variant : (resident_ok ? PF_VARIANT_GROUP_RESIDENT : PF_VARIANT_GROUP_TWO_PASS);
    if (variant == PF_VARIANT_GROUP_RESIDENT && !resident_ok)
        return fail(PF_ERR_UNSUPPORTED, "the register-resident variant is not available for this chain or shape");
    if (variant != PF_VARIANT_GROUP_RESIDENT && variant != PF_VARIANT_GROUP_TWO_PASS)
        return fail(PF_ERR_UNSUPPORTED, "unknown group variant %d", variant);
    p->variant = variant;
    p->block = dim3(threads);
    g.pos_per_block = (uint32_t)nv * g.pos_per_step;
    g.blocks_per_sample = bps;
    p->k = nv;
    if (variant == PF_VARIANT_GROUP_RESIDENT) {
        p->grid = dim3(res_grid);
        p->n_launches = 1;
        if (fused_fn) {
            p->jit_fn = fused_fn;
            p->spec_id = pf::kSpecJit;
        }
    } else {
        p->grid = dim3((uint32_t)tiles);
        p->grid2 = p->grid;
        p->block2 = p->block;
        p->n_launches = 2;
        if (jit_ok) {
            p->jit_fn = pf::jit_group_kernel(p->device, L.main_dtype, nv, 1, gen_parts, jspec, &jit_err);
            p->jit_fn2 = p->jit_fn ? pf::jit_group_kernel(p->device, L.main_dtype, nv, 2, gen_parts, jspec, &jit_err) : nullptr;
            if (p->jit_fn && p->jit_fn2) p->spec_id = pf::kSpecJit;
        }
    }
    if (jit_ok && p->spec_id == 0 && env_int("PF_LOG", 0))
        fprintf(stderr, "[pf] plan-time specialisation unavailable, using the interpreter: %s\n", jit_err.c_str());
    p->lds_bytes = general ? gen_lds + 512 * 2 * 4 + 4 : 512 * 3 * 4 + 512 * 2 * 4 + 4;
    p->dyn_lds = gen_lds;
    // workspace: partials of the two-launch variant, or two parities of exchange words (all-ones = empty) of the
    // resident one; then the error word
    const uint64_t part_bytes = variant == PF_VARIANT_GROUP_RESIDENT ? 0 : (uint64_t)samples * g.blocks_per_sample * g.groups * 4 * sizeof(float);
    const uint64_t gather_bytes =
        variant == PF_VARIANT_GROUP_RESIDENT ? (((uint64_t)2 * samples * g.groups * g.blocks_per_sample * sizeof(uint64_t)) + 255) / 256 * 256 : 0;
    p->workspace_bytes = part_bytes + gather_bytes + 256;
    if (hipMalloc(&p->workspace, p->workspace_bytes) != hipSuccess) return fail(PF_ERR_NOMEM, "workspace allocation of %llu bytes failed", (unsigned long long)p->workspace_bytes);
    char* ws = static_cast<char*>(p->workspace);
    if (hipMemset(ws, 0, p->workspace_bytes) != hipSuccess || (gather_bytes && hipMemset(ws + part_bytes, 0xff, gather_bytes) != hipSuccess))
        return fail(PF_ERR_HIP, "workspace clear failed");
    g.ws_partial = part_bytes ? reinterpret_cast<float*>(ws) : nullptr;
    g.ws_gather = gather_bytes ? reinterpret_cast<uint64_t*>(ws + part_bytes) : nullptr;
    g.ws_error = reinterpret_cast<uint32_t*>(ws + part_bytes + gather_bytes);
    p->args.n_inner = (uint32_t)C;
    p->args.rows = (uint64_t)(samples * hw);
    return PF_OK;
}

// ---- stencil family
pf_status plan_stencil(pf_plan_s* p, const Checked& c, int forced_variant) {
    const Lowered& L = p->low;
    const int es = dtype_size(L.main_dtype);
    const int vec = 16 / es;
    const Shape& xs = L.pre_shape;  // [n, h, w, c]
    const Shape& ks = c.shape[p->desc.ops[L.core_op].src[1]];
    if (ks[0] != ks[1] || (ks[0] != 3 && ks[0] != 5))
        return fail(PF_ERR_UNSUPPORTED, "dwconv2d: 3 x 3 and 5 x 5 kernels are implemented (got %lld x %lld)", (long long)ks[0], (long long)ks[1]);
    const int ksz = (int)ks[0];
    const int out_rows = ksz == 3 ? kStencilRowsHost : kStencilRows5Host;
    const int64_t n = xs[0], h = xs[1], w = xs[2], ch = xs[3];
    if ((ch * es) % 16 != 0) return fail(PF_ERR_ALIGNMENT, "channel count %lld is not a multiple of 16 bytes", (long long)ch);
    if (p->ragged) return fail(PF_ERR_ALIGNMENT, "a broadcast input of the stencil family is not a multiple of 16 bytes");
    if (n * h * w > 0xffffffffLL || n > 65535 || (h + out_rows - 1) / out_rows > 65535) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the stencil family");
    if (L.n_out != 1) return fail(PF_ERR_UNSUPPORTED, "secondary outputs are not implemented in the stencil family");
    for (int i = 0; i < L.pro.n; ++i)
        if (L.pro.u[i].code == pf::U_MASK_CAUSAL) return fail(PF_ERR_UNSUPPORTED, "causal_mask next to a convolution is not implemented");
    for (int i = 0; i < L.epi.n; ++i)
        if (L.epi.u[i].code == pf::U_MASK_CAUSAL) return fail(PF_ERR_UNSUPPORTED, "causal_mask next to a convolution is not implemented");
    pf::StencilGeom& g = p->stencil;
    memset(&g, 0, sizeof(g));
    g.n = (uint32_t)n;
    g.h = (uint32_t)h;
    g.w = (uint32_t)w;
    g.c = (uint32_t)ch;
    g.cv = (uint32_t)(ch / vec);
    g.row_vecs = (uint32_t)(w * g.cv);
    g.div_cv = make_fastdiv(g.cv);
    for (int f = 0; f < L.n_full; ++f)
        if (L.full_is_epi[f]) g.epi_full_mask |= 1u << f;
    for (int v = 0; v < L.n_vec; ++v)
        if (L.vec_is_epi[v]) g.epi_vec_mask |= 1u << v;
    p->family = PF_FAMILY_STENCIL;
    p->k = 1;
    p->spec_id = 0;
    p->block = dim3(256);
    p->grid = dim3((g.row_vecs + 255u) / 256u, (uint32_t)((h + out_rows - 1) / out_rows), (uint32_t)n);
    p->n_launches = 1;
    p->stencil_ks = ksz;
    p->args.n_inner = (uint32_t)ch;
    p->args.rows = (uint64_t)(n * h * w);
    const pf_op_desc& conv = p->desc.ops[L.core_op];
    const int64_t stride = conv.n_i == 1 ? conv.i[0] : 1;
    if (stride > 1) {
        // down-sampling convolution: one lane per output column and channel vector, taps loaded where they are used
        if (forced_variant >= 0 && forced_variant != PF_VARIANT_STENCIL_STRIDED)
            return fail(PF_ERR_UNSUPPORTED, "a strided convolution runs on the strided variant only");
        const int64_t oh = (h - 1) / stride + 1, ow = (w - 1) / stride + 1;
        g.stride = (uint32_t)stride;
        g.oh = (uint32_t)oh;
        g.ow = (uint32_t)ow;
        g.out_row_vecs = (uint32_t)(ow * g.cv);
        // output rows per workgroup: 4 (the kernel vectors are loaded once per workgroup), fewer while that leaves
        // a compute unit with less than about eight workgroups
        hipDeviceProp_t prop;
        const int n_cu = (hipGetDeviceProperties(&prop, p->device) == hipSuccess && prop.multiProcessorCount > 0) ? prop.multiProcessorCount : 256;
        const int64_t tiles_x = (g.out_row_vecs + 255) / 256;
        int64_t strip = 4;
        while (strip > 1 && tiles_x * ((oh + strip - 1) / strip) * n < 8 * (int64_t)n_cu) strip /= 2;
        g.strip_rows = (uint32_t)strip;
        if ((oh + strip - 1) / strip > 65535) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the stencil family");
        p->variant = PF_VARIANT_STENCIL_STRIDED;
        p->lds_bytes = 0;
        p->grid = dim3((uint32_t)tiles_x, (uint32_t)((oh + strip - 1) / strip), (uint32_t)n);
        if (jit_possible(p->device)) {
            std::string err;
            p->jit_fn = pf::jit_stencil_kernel(p->device, L.main_dtype, p->variant, ksz, make_jit_spec(L), &err);
            if (p->jit_fn) p->spec_id = pf::kSpecJit;
            else if (env_int("PF_LOG", 0)) fprintf(stderr, "[pf] plan-time specialisation unavailable, using the interpreter: %s\n", err.c_str());
        }
        return PF_OK;
    }
    if (forced_variant == PF_VARIANT_STENCIL_STRIDED) return fail(PF_ERR_UNSUPPORTED, "the strided variant is for strides above 1");
    // Staged variant (values activated once, shared through an LDS tile) when the tile fits; its entries are
    // packed in the storage type if the prologue keeps storage precision and the kernel is specialised.
    const bool jit_ok = jit_possible(p->device);
    bool exact_pro = L.main_dtype != PF_F32 && L.pro.n >= 1 && L.pro.u[0].code == pf::U_MOV && L.pro.u[0].kind == pf::K_FULL;
    for (int i = 1; i < L.pro.n; ++i)
        if (L.pro.u[i].code != pf::U_RELU && L.pro.u[i].code != pf::U_NEG) exact_pro = false;
    const uint32_t entry_bytes = (L.main_dtype == PF_F32 || (exact_pro && jit_ok)) ? 16u : 32u;
    const uint64_t tile_bytes = (uint64_t)(out_rows + ksz - 1) * (256u + 2u * (uint32_t)(ksz / 2) * g.cv) * entry_bytes;
    // per workgroup: 64 KB everywhere; up to 96 KB where the device offers 160 KB (gfx950), which still leaves
    // room for a second, smaller workgroup on the compute unit
    uint64_t lds_limit = 64 * 1024;
    {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, p->device) == hipSuccess && prop.sharedMemPerBlock >= 160 * 1024) lds_limit = 96 * 1024;
    }
    const bool staged_ok = tile_bytes <= lds_limit;
    int variant = forced_variant >= 0 ? forced_variant : (staged_ok ? PF_VARIANT_STENCIL_STAGED : PF_VARIANT_STENCIL_DIRECT);
    if (variant == PF_VARIANT_STENCIL_DIRECT && ksz != 3)
        return fail(PF_ERR_UNSUPPORTED, "5 x 5 kernels need the staged variant, whose LDS tile (%llu bytes) does not fit here", (unsigned long long)tile_bytes);
    if (variant != PF_VARIANT_STENCIL_STAGED && variant != PF_VARIANT_STENCIL_DIRECT) return fail(PF_ERR_UNSUPPORTED, "unknown stencil variant %d", variant);
    if (variant == PF_VARIANT_STENCIL_STAGED && !staged_ok)
        return fail(PF_ERR_UNSUPPORTED, "the staged variant needs an LDS tile of %llu bytes (limit %llu)", (unsigned long long)tile_bytes,
                    (unsigned long long)lds_limit);
    p->variant = variant;
    p->lds_bytes = variant == PF_VARIANT_STENCIL_STAGED ? (uint32_t)tile_bytes : 0u;
    if (variant == PF_VARIANT_STENCIL_STAGED) {
        // one-dimensional grid, tiles numbered so that neighbours share a compute die's L2
        g.tiles_x = p->grid.x;
        g.tiles_y = p->grid.y;
        const uint64_t tiles = (uint64_t)p->grid.x * p->grid.y * p->grid.z;
        if (tiles > 0x7ffffff0ull) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the stencil family");
        g.tiles = (uint32_t)tiles;
        g.tiles_per_die = (uint32_t)((tiles + 7) / 8);
        p->grid = dim3(g.tiles_per_die * 8u);
    }
    if (jit_ok) {
        std::string err;
        p->jit_fn = pf::jit_stencil_kernel(p->device, L.main_dtype, variant, ksz, make_jit_spec(L), &err);
        if (p->jit_fn) p->spec_id = pf::kSpecJit;
        else {
            if (env_int("PF_LOG", 0)) fprintf(stderr, "[pf] plan-time specialisation unavailable, using the interpreter: %s\n", err.c_str());
            // the interpreted kernel never packs its tile
            if (variant == PF_VARIANT_STENCIL_STAGED && entry_bytes == 16u && L.main_dtype != PF_F32) {
                const uint64_t big = tile_bytes * 2;
                if (big > lds_limit && ksz != 3) return fail(PF_ERR_UNSUPPORTED, "5 x 5 kernels need the staged variant, whose LDS tile does not fit here");
                if (big > lds_limit) {
                    p->variant = PF_VARIANT_STENCIL_DIRECT;
                    p->lds_bytes = 0;
                    p->grid = dim3(g.tiles_x, g.tiles_y, (uint32_t)n);
                } else {
                    p->lds_bytes = (uint32_t)big;
                }
            }
        }
    }
    return PF_OK;
}

// ---- gather family
int64_t gcd64(int64_t a, int64_t b) {
    while (b != 0) {
        const int64_t t = a % b;
        a = b;
        b = t;
    }
    return a;
}

// Where element `e` (flat index) of value `v` comes from: walks the operators backwards to a chain input.
void gather_source(const pf_chain_desc* d, const Checked& c, int v, int64_t e, int* in_id, int64_t* in_flat) {
    const int n_in = d->n_inputs;
    while (v >= n_in) {
        const pf_op_desc& o = d->ops[v - n_in];
        const Shape& os = c.shape[v];
        const int rank = (int)os.size();
        if (o.op == PF_RESHAPE) {
            v = o.src[0];
            continue;
        }
        int64_t idx[PF_MAX_RANK];
        int64_t rem = e;
        for (int q = rank - 1; q >= 0; --q) {
            idx[q] = rem % os[q];
            rem /= os[q];
        }
        int src = o.src[0];
        int64_t sidx[PF_MAX_RANK];
        if (o.op == PF_PERMUTE) {
            for (int q = 0; q < rank; ++q) sidx[o.i[q]] = idx[q];
        } else if (o.op == PF_SLICE) {
            for (int q = 0; q < rank; ++q) sidx[q] = idx[q];
            sidx[o.i[0]] += o.i[1];
        } else {  // PF_CONCAT
            for (int q = 0; q < rank; ++q) sidx[q] = idx[q];
            const int64_t first = c.shape[o.src[0]][o.i[0]];
            if (idx[o.i[0]] >= first) {
                src = o.src[1];
                sidx[o.i[0]] -= first;
            }
        }
        const Shape& ss = c.shape[src];
        int64_t flat = 0;
        for (int q = 0; q < rank; ++q) flat = flat * ss[q] + sidx[q];
        e = flat;
        v = src;
    }
    *in_id = v;
    *in_flat = e;
}

pf_status plan_gather(pf_plan_s* p, const Checked& c) {
    const pf_chain_desc* d = &p->desc;
    const Lowered& L = p->low;
    const int es = dtype_size(L.main_dtype);
    const int vec = 16 / es;
    const int n_in = d->n_inputs;
    // Run length: for every value, a length G such that each aligned block of G elements (flat, row-major)
    // is contiguous inside one chain input.  0 stands for "the whole tensor" (gcd(0, x) = x).
    std::vector<int64_t> G(n_in + d->n_ops, 0);
    for (int k = 0; k < d->n_ops; ++k) {
        const pf_op_desc& o = d->ops[k];
        const int v = n_in + k;
        const Shape& os = c.shape[v];
        const int rank = (int)os.size();
        int64_t g = G[o.src[0]] ? G[o.src[0]] : numel(c.shape[o.src[0]]);
        if (o.op == PF_PERMUTE) {
            int64_t inner = 1;
            for (int q = rank - 1; q >= 0 && o.i[q] == q; --q) inner *= os[q];
            g = gcd64(g, inner);
        } else if (o.op == PF_SLICE) {
            int64_t inner = 1;
            for (int q = (int)o.i[0] + 1; q < rank; ++q) inner *= os[q];
            g = gcd64(gcd64(g, o.i[2] * inner), gcd64(o.i[1] * inner, c.shape[o.src[0]][o.i[0]] * inner));
        } else if (o.op == PF_CONCAT) {
            int64_t inner = 1;
            for (int q = (int)o.i[0] + 1; q < rank; ++q) inner *= os[q];
            const int64_t g1 = G[o.src[1]] ? G[o.src[1]] : numel(c.shape[o.src[1]]);
            g = gcd64(gcd64(g, g1), gcd64(c.shape[o.src[0]][o.i[0]] * inner, c.shape[o.src[1]][o.i[0]] * inner));
        }
        G[v] = g;
    }
    int64_t run = 0, total = 0;
    for (int o = 0; o < d->n_outputs; ++o) {
        const int v = d->out_value[o];
        run = gcd64(run, G[v] ? G[v] : numel(c.shape[v]));
        total += numel(c.shape[v]);
    }
    for (int k = 0; k < n_in; ++k)
        if (numel(c.shape[k]) > 0xffffffffLL) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the gather family");
    if (total > 0xffffffffLL) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the gather family");
    // very long runs are cut so that the copy has enough workgroups; cuts keep whole vectors
    while (run > 65536 && run % 2 == 0 && (run / 2) % vec == 0) run /= 2;
    const int64_t n_runs = total / run;
    if (n_runs > (1 << 22))
        return fail(PF_ERR_UNSUPPORTED, "layout chain moves runs of only %lld elements: %lld runs exceed the run table", (long long)run, (long long)n_runs);
    std::vector<pf::GatherRun> table((size_t)n_runs);
    size_t at = 0;
    for (int o = 0; o < d->n_outputs; ++o) {
        const int v = d->out_value[o];
        const int64_t n = numel(c.shape[v]);
        for (int64_t e = 0; e < n; e += run) {
            int in_id;
            int64_t in_flat;
            gather_source(d, c, v, e, &in_id, &in_flat);
            pf::GatherRun& r = table[at++];
            r.src_off = (uint32_t)in_flat;
            r.dst_off = (uint32_t)e;
            r.src_id = (uint8_t)in_id;
            r.dst_id = (uint8_t)o;
            r.pad = 0;
        }
    }
    if (hipSetDevice(p->device) != hipSuccess) return fail(PF_ERR_HIP, "cannot select device %d", p->device);
    p->workspace_bytes = (uint64_t)n_runs * sizeof(pf::GatherRun);
    if (hipMalloc(&p->workspace, p->workspace_bytes) != hipSuccess) return fail(PF_ERR_NOMEM, "run table allocation of %llu bytes failed", (unsigned long long)p->workspace_bytes);
    if (hipMemcpy(p->workspace, table.data(), p->workspace_bytes, hipMemcpyHostToDevice) != hipSuccess) return fail(PF_ERR_HIP, "run table upload failed");
    pf::GatherArgs& a = p->gather;
    memset(&a, 0, sizeof(a));
    a.table = static_cast<const pf::GatherRun*>(p->workspace);
    a.n_runs = (uint32_t)n_runs;
    a.run_elems = (uint32_t)run;
    a.vec_per_run = (uint32_t)((run + vec - 1) / vec);
    a.div_vpr = make_fastdiv(a.vec_per_run);
    const uint64_t work = (uint64_t)n_runs * a.vec_per_run;
    if (work > 0x7fffffffull) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the gather family");
    p->family = PF_FAMILY_GATHER;
    p->variant = 0;
    p->k = 1;
    p->spec_id = 0;
    p->block = dim3(256);
    p->grid = dim3((uint32_t)((work + 255) / 256));
    p->lds_bytes = 0;
    p->n_launches = 1;
    return PF_OK;
}

// ---- attention family
// ---- pool family
pf_status plan_pool(pf_plan_s* p) {
    const Lowered& L = p->low;
    const int es = dtype_size(L.main_dtype);
    const int vec = 16 / es;
    const Shape& xs = L.pre_shape;  // [n, spatial.., c]
    const int64_t n = xs[0], ch = xs.back();
    const int64_t hw = numel(xs) / (n * ch);
    if ((ch * es) % 16 != 0) return fail(PF_ERR_ALIGNMENT, "channel count %lld is not a multiple of 16 bytes", (long long)ch);
    if (p->ragged) return fail(PF_ERR_ALIGNMENT, "a broadcast input of the pool family is not a multiple of 16 bytes");
    const int64_t cv = ch / vec;
    if (cv > 512) return fail(PF_ERR_UNSUPPORTED, "more than %d channels", 512 * vec);
    if (n * hw > 0xffffffffLL || n > 0x7fffffLL) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the pool family");
    if (L.n_out != 1) return fail(PF_ERR_UNSUPPORTED, "secondary outputs are not implemented in the pool family");
    if (L.n_full < 1 || L.full_is_epi[0]) return fail(PF_ERR_UNSUPPORTED, "the pooled value must start from a full-shape input");
    for (int i = 0; i < L.pro.n; ++i)
        if (L.pro.u[i].code == pf::U_MASK_CAUSAL) return fail(PF_ERR_UNSUPPORTED, "causal_mask in front of a pooling is not implemented");
    for (int i = 0; i < L.epi.n; ++i)
        if (L.epi.u[i].code == pf::U_MASK_CAUSAL) return fail(PF_ERR_UNSUPPORTED, "causal_mask behind a pooling is not implemented");
    hipDeviceProp_t prop;
    const int n_cu = (hipGetDeviceProperties(&prop, p->device) == hipSuccess && prop.multiProcessorCount > 0) ? prop.multiProcessorCount : 256;
    pf::PoolGeom& g = p->pool;
    memset(&g, 0, sizeof(g));
    g.samples = (uint32_t)n;
    g.hw = (uint32_t)hw;
    g.channels = (uint32_t)ch;
    g.cv = (uint32_t)cv;
    g.div_cv = make_fastdiv(g.cv);
    g.pos_per_step = 512u / g.cv;
    g.inv_hw = 1.0f / (float)hw;
    for (int f = 0; f < L.n_full; ++f)
        if (L.full_is_epi[f]) g.epi_full_mask |= 1u << f;
    for (int v = 0; v < L.n_vec; ++v)
        if (L.vec_is_epi[v]) g.epi_vec_mask |= 1u << v;
    // A workgroup walks `chunks` chunks of nv position steps.  Slices are cut so that the device gets about four
    // workgroups per compute unit, at most 32 per sample (measured on [16, 64, 64, 512] fp16: 64 slices per sample
    // 21 us, 32: 17.7 us, 16: 17.1 us, 8: 19.5 us, 4: 28 us; with SiLU in front 32 slices are best).
    int nv = 8;
    while (nv > 1 && (int64_t)(nv / 2) * g.pos_per_step >= hw) nv /= 2;
    const int forced_nv = env_int("PF_POOL_NV", 0);
    if (forced_nv == 1 || forced_nv == 2 || forced_nv == 4 || forced_nv == 8) nv = forced_nv;
    const int64_t chunk_pos = (int64_t)nv * g.pos_per_step;
    const int64_t all_chunks = (hw + chunk_pos - 1) / chunk_pos;
    const int64_t want_bps = std::max<int64_t>(1, std::min<int64_t>(all_chunks, std::min<int64_t>(32, (4 * (int64_t)n_cu + n - 1) / n)));
    int64_t chunks = (all_chunks + want_bps - 1) / want_bps;
    const int forced_chunks = env_int("PF_POOL_CHUNKS", 0);
    if (forced_chunks > 0) chunks = forced_chunks;
    g.chunks = (uint32_t)chunks;
    g.pos_per_block = (uint32_t)(chunks * chunk_pos);
    g.blocks_per_sample = (uint32_t)((hw + chunks * chunk_pos - 1) / (chunks * chunk_pos));
    const uint64_t blocks = (uint64_t)g.blocks_per_sample * n;
    if (blocks > 0x7fffffffull) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the pool family");
    p->family = PF_FAMILY_POOL;
    p->variant = 0;
    p->k = nv;
    p->spec_id = 0;
    p->block = dim3(512);
    p->grid = dim3((uint32_t)blocks);
    p->lds_bytes = 512 * vec * 4 + 4;
    p->n_launches = 1;
    p->args.n_inner = (uint32_t)ch;
    p->args.rows = (uint64_t)(n * hw);
    if (g.blocks_per_sample > 1) {
        const uint64_t part_bytes = ((uint64_t)blocks * ch * sizeof(float) + 255) / 256 * 256;
        const uint64_t flag_bytes = ((uint64_t)blocks * sizeof(uint32_t) + 255) / 256 * 256;
        p->workspace_bytes = part_bytes + flag_bytes + 256;
        if (hipSetDevice(p->device) != hipSuccess || hipMalloc(&p->workspace, p->workspace_bytes) != hipSuccess)
            return fail(PF_ERR_NOMEM, "workspace allocation of %llu bytes failed", (unsigned long long)p->workspace_bytes);
        if (hipMemset(p->workspace, 0, p->workspace_bytes) != hipSuccess) return fail(PF_ERR_HIP, "workspace clear failed");
        g.ws_partial = reinterpret_cast<float*>(p->workspace);
        g.ws_flags = reinterpret_cast<uint32_t*>(static_cast<char*>(p->workspace) + part_bytes);
        g.ws_error = reinterpret_cast<uint32_t*>(static_cast<char*>(p->workspace) + part_bytes + flag_bytes);
        g.spin_limit = (uint32_t)env_int("PF_POOL_SPIN_LIMIT", 1 << 18);  // polling rounds before a wait gives up (tests force it small)
        p->ws_error = g.ws_error;
    }
    if (jit_possible(p->device)) {
        std::string err;
        p->jit_fn = pf::jit_pool_kernel(p->device, L.main_dtype, nv, L.pool_op, make_jit_spec(L), &err);
        if (p->jit_fn) p->spec_id = pf::kSpecJit;
        else if (env_int("PF_LOG", 0)) fprintf(stderr, "[pf] plan-time specialisation unavailable, using the interpreter: %s\n", err.c_str());
    }
    return PF_OK;
}

pf_status plan_attn(pf_plan_s* p, int forced_variant) {
    const Lowered& L = p->low;
    const int es = dtype_size(L.main_dtype);
    const int vec = 16 / es;
    const Shape& ks = L.pre_shape;  // [..., t, d]
    const int64_t d = ks.back(), t = ks[ks.size() - 2];
    const int64_t heads = numel(ks) / (t * d);
    const bool grows = L.attn_in[1] >= 0;
    const int64_t t_total = t + (grows ? 1 : 0);
    if ((d * es) % 16 != 0) return fail(PF_ERR_ALIGNMENT, "head dimension %lld is not a multiple of 16 bytes", (long long)d);
    const int64_t lpr = d / vec;
    if (lpr > 64 || (lpr & (lpr - 1)) != 0 || d > 256)
        return fail(PF_ERR_UNSUPPORTED, "head dimension %lld: needs a power-of-two number (<= 64) of 16-byte vectors and at most 256 elements", (long long)d);
    if (heads > 65535 || t_total > 0x7fffffffLL || t_total < 1) return fail(PF_ERR_UNSUPPORTED, "attention shape out of range");
    hipDeviceProp_t prop;
    if (hipSetDevice(p->device) != hipSuccess || hipGetDeviceProperties(&prop, p->device) != hipSuccess)
        return fail(PF_ERR_HIP, "cannot query device %d (the attention family needs the device at plan time)", p->device);
    const int n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    pf::AttnArgs& a = p->attn;
    memset(&a, 0, sizeof(a));
    a.t = (uint32_t)t;
    a.t_total = (uint32_t)t_total;
    a.d = (uint32_t)d;
    a.lanes_per_row = (uint32_t)lpr;
    a.log2_lpr = 0;
    while ((1u << a.log2_lpr) < a.lanes_per_row) ++a.log2_lpr;
    a.scale = L.attn_scale;
    // Rows per workgroup: 8 steps of 256 / lpr rows when that still gives every compute unit two workgroups,
    // else 4 (measured on MI355X: fewer, longer slices win until the device runs short of workgroups; one or
    // two steps per workgroup lose to the per-slice overhead, sixteen to register pressure).
    const int64_t rps = 256 / lpr;
    int nv = 4;
    if (heads * ((t_total + rps * 8 - 1) / (rps * 8)) >= 2 * (int64_t)n_cu) nv = 8;
    const int forced_nv = env_int("PF_ATTN_NV", 0);
    if (forced_nv == 1 || forced_nv == 2 || forced_nv == 4 || forced_nv == 8) nv = forced_nv;
    // Streaming variant: a workgroup walks `chunks` chunks of 2 steps each with the next chunk's loads in flight.
    // Measured on MI355X: it wins (10-13 %) when slices get long -- many heads (one slice per head: no device-scope
    // merge at all) or long caches -- and ties or loses below eight chunks per slice, where the one-pass kernel's
    // deeper load burst counts for more.  Slices are cut so that every compute unit still gets about three workgroups.
    int64_t chunks = 1;
    {
        const int64_t all_chunks = (t_total + rps * 2 - 1) / (rps * 2);
        const int64_t target_splits = std::max<int64_t>(1, (3 * (int64_t)n_cu + heads - 1) / heads);
        const int64_t c = (all_chunks + target_splits - 1) / target_splits;
        const int forced_chunks = env_int("PF_ATTN_CHUNKS", 0);
        chunks = forced_chunks > 0 ? forced_chunks : c;
    }
    int variant = forced_variant >= 0 ? forced_variant : (chunks >= 8 && !forced_nv ? PF_VARIANT_ATTN_STREAM : PF_VARIANT_ATTN_ONE_PASS);
    if (variant != PF_VARIANT_ATTN_ONE_PASS && variant != PF_VARIANT_ATTN_STREAM)
        return fail(PF_ERR_UNSUPPORTED, "unknown attention variant %d", variant);
    if (variant == PF_VARIANT_ATTN_STREAM) {
        nv = forced_nv == 4 ? 4 : 2;
        if (chunks < 1) chunks = 1;
    } else {
        chunks = 1;
    }
    a.chunks = (uint32_t)chunks;
    const int64_t splits = (t_total + rps * nv * chunks - 1) / (rps * nv * chunks);
    if (splits > 65535) return fail(PF_ERR_UNSUPPORTED, "too many cached rows for the attention family");
    p->family = PF_FAMILY_ATTENTION;
    p->variant = variant;
    p->k = nv;
    p->spec_id = 0;
    p->block = dim3(256);
    p->grid = dim3((uint32_t)splits, (uint32_t)heads);
    p->lds_bytes = (8 + 4 * 256 + 1) * 4;
    p->n_launches = 1;
    a.part_stride = (uint32_t)((d + 2 + 31) / 32 * 32);
    const uint64_t part_bytes = ((uint64_t)heads * splits * a.part_stride * sizeof(float) + 255) / 256 * 256;
    const uint64_t cnt_bytes = ((uint64_t)heads * sizeof(uint32_t) + 255) / 256 * 256;
    p->workspace_bytes = part_bytes + cnt_bytes;
    if (hipMalloc(&p->workspace, p->workspace_bytes) != hipSuccess) return fail(PF_ERR_NOMEM, "workspace allocation of %llu bytes failed", (unsigned long long)p->workspace_bytes);
    if (hipMemset(p->workspace, 0, p->workspace_bytes) != hipSuccess) return fail(PF_ERR_HIP, "workspace clear failed");
    a.ws_partial = reinterpret_cast<float*>(p->workspace);
    a.ws_counter = reinterpret_cast<uint32_t*>(static_cast<char*>(p->workspace) + part_bytes);
    return PF_OK;
}

pf_status plan_checked_desc(const pf_chain_desc* desc, int32_t device, int32_t variant, pf_plan** out);

}  // namespace

extern "C" {

pf_status pf_chain_validate(const pf_chain_desc* desc) {
    Checked c;
    return check_desc(desc, &c);
}

pf_status pf_chain_recompose(const pf_chain_desc* desc, pf_chain_desc* out, int32_t* changed) {
    Checked c;
    pf_status s = check_desc(desc, &c);
    if (s != PF_OK) return s;
    if (!out) return fail(PF_ERR_INVALID_ARG, "out is null");
    Recomposer rc;
    rc.d = desc, rc.c = &c;
    pf_chain_desc composite;
    const bool hit = rc.run(&composite);
    *out = hit ? composite : *desc;
    if (changed) *changed = hit ? 1 : 0;
    return PF_OK;
}

pf_status pf_chain_infer_shape(const pf_chain_desc* desc, int32_t value, pf_tensor_desc* out) {
    Checked c;
    pf_status s = check_desc(desc, &c);
    if (s != PF_OK) return s;
    if (!out) return fail(PF_ERR_INVALID_ARG, "out is null");
    if (value < 0 || value >= (int32_t)c.shape.size()) return fail(PF_ERR_INVALID_ARG, "value id %d out of range", value);
    const Shape& sh = c.shape[value];
    if (sh.size() > PF_MAX_RANK) return fail(PF_ERR_SHAPE, "rank exceeds PF_MAX_RANK");
    pf_tensor_desc t;
    memset(&t, 0, sizeof(t));
    t.dtype = value < desc->n_inputs ? desc->inputs[value].dtype : PF_F32;
    t.rank = (int32_t)sh.size();
    for (size_t i = 0; i < sh.size(); ++i) t.shape[i] = sh[i];
    *out = t;
    return PF_OK;
}

pf_status pf_chain_plan_variant(const pf_chain_desc* desc, int32_t device, int32_t variant, pf_plan** out) {
    if (!out) return fail(PF_ERR_INVALID_ARG, "out is null");
    Checked c;
    pf_status s = check_desc(desc, &c);
    if (s != PF_OK) return s;
    // a chain that spells a composite operator in basic operators is planned as that operator when that works
    if (env_int("PF_RECOMPOSE", 1) != 0) {
        Recomposer rc;
        rc.d = desc, rc.c = &c;
        pf_chain_desc composite;
        if (rc.run(&composite) && plan_checked_desc(&composite, device, variant, out) == PF_OK) return PF_OK;
    }
    return plan_checked_desc(desc, device, variant, out);
}

}  // extern "C"

namespace {

pf_status plan_checked_desc(const pf_chain_desc* desc, int32_t device, int32_t variant, pf_plan** out) {
    Checked c;
    pf_status s = check_desc(desc, &c);
    if (s != PF_OK) return s;
    pf_plan_s* p = new (std::nothrow) pf_plan_s();
    if (!p) return fail(PF_ERR_NOMEM, "out of host memory");
    p->desc = *desc;
    p->device = device;
    memset(&p->args, 0, sizeof(p->args));
    memset(&p->row, 0, sizeof(p->row));
    memset(&p->group, 0, sizeof(p->group));
    memset(&p->permg, 0, sizeof(p->permg));
    memset(&p->attn, 0, sizeof(p->attn));
    s = lower_chain(desc, c, &p->low);
    if (s == PF_OK && p->low.core != pf::CORE_ATTN_DECODE && p->low.core != pf::CORE_GATHER) {
        const Lowered& L = p->low;
        p->args.n_full = L.n_full;
        p->args.n_vec = L.n_vec;
        p->args.core = L.core;
        p->args.core_vec[0] = L.core_vec[0];
        p->args.core_vec[1] = L.core_vec[1];
        p->args.eps = L.eps;
        p->args.mask_si = L.mask_si;
        p->args.core_mask = L.core_mask;
        p->args.mask_div = make_fastdiv(L.mask_si ? L.mask_si : 1u);
        p->args.core_scale = L.core_scale;
        p->args.pro = L.pro;
        p->args.epi = L.epi;
        // pure layout work (nothing but the initial load): kernels move the raw bits, no conversion
        p->args.raw_copy = (L.pro.n == 1 && L.epi.n == 0 && L.pro.u[0].code == pf::U_MOV && L.pro.u[0].kind == pf::K_FULL) ? 1u : 0u;
        s = fill_vec_args(p, c);
    }
    if (s == PF_OK) {
        switch (p->low.core) {
            case pf::CORE_NONE: s = plan_ew(p); break;
            case pf::CORE_GROUPNORM: s = plan_group(p, variant); break;
            case pf::CORE_PERMUTE: s = plan_perm(p, variant); break;
            case pf::CORE_ATTN_DECODE: s = plan_attn(p, variant); break;
            case pf::CORE_GATHER: s = plan_gather(p, c); break;
            case pf::CORE_DWCONV: s = plan_stencil(p, c, variant); break;
            case pf::CORE_POOL: s = plan_pool(p); break;
            default: s = plan_row(p, variant); break;
        }
    }
    if (s == PF_OK) {
        for (int k = 0; k < desc->n_inputs; ++k) p->in_bytes[k] = (uint64_t)numel(c.shape[k]) * dtype_size(desc->inputs[k].dtype);
        for (int o = 0; o < desc->n_outputs; ++o) {
            p->out_shape[o] = c.shape[desc->out_value[o]];
            p->out_bytes[o] = (uint64_t)numel(p->out_shape[o]) * dtype_size(desc->out_dtype[o]);
        }
        if (env_int("PF_LOG", 0))
            fprintf(stderr, "[pf_chain] family=%d variant=%d spec=%d k=%d rpw=%u grid=%u block=%u uops=%d+%d full=%d vec=%d tmp=%d mask_si=%u\n",
                    p->family, p->variant, p->spec_id, p->k, p->row.rows_per_wave, p->grid.x, p->block.x, p->low.pro.n, p->low.epi.n, p->low.n_full,
                    p->low.n_vec, p->low.n_tmp, p->low.mask_si);
        *out = p;
        return PF_OK;
    }
    pf_chain_plan_destroy(p);
    return s;
}

}  // namespace

extern "C" {

pf_status pf_chain_plan(const pf_chain_desc* desc, int32_t device, pf_plan** out) {
    return pf_chain_plan_variant(desc, device, env_int("PF_FORCE_VARIANT", -1), out);
}

pf_status pf_chain_plan_get_info(const pf_plan* plan, pf_plan_info* info) {
    if (!plan || !info) return fail(PF_ERR_INVALID_ARG, "null argument");
    memset(info, 0, sizeof(*info));
    info->family = plan->family;
    info->variant = plan->variant;
    info->grid[0] = plan->grid.x; info->grid[1] = plan->grid.y; info->grid[2] = plan->grid.z;
    info->block[0] = plan->block.x; info->block[1] = plan->block.y; info->block[2] = plan->block.z;
    info->lds_bytes = plan->lds_bytes;
    info->workspace_bytes = plan->workspace_bytes + (plan->bcast_dev ? sizeof(plan->bcast_host) : 0);
    for (int k = 0; k < plan->desc.n_inputs; ++k) info->compulsory_read_bytes += plan->in_bytes[k];
    for (int o = 0; o < plan->desc.n_outputs; ++o) info->compulsory_write_bytes += plan->out_bytes[o];
    info->n_launches = plan->n_launches;
    info->n_micro_ops = plan->low.pro.n + plan->low.epi.n;
    info->spec_id = plan->spec_id;
    info->vectors_per_lane = plan->k;
    return PF_OK;
}

pf_status pf_chain_run(const pf_plan* plan, const void* const* inputs, void* const* outputs, void* stream) {
    if (!plan || !inputs || !outputs) return fail(PF_ERR_INVALID_ARG, "null argument");
    const pf_chain_desc& d = plan->desc;
    for (int k = 0; k < d.n_inputs; ++k) {
        if (!inputs[k]) return fail(PF_ERR_INVALID_ARG, "input %d is null", k);
        if ((uintptr_t)inputs[k] % 16 != 0) return fail(PF_ERR_ALIGNMENT, "input %d is not 16-byte aligned", k);
    }
    for (int o = 0; o < d.n_outputs; ++o) {
        if (!outputs[o]) return fail(PF_ERR_INVALID_ARG, "output %d is null", o);
        if ((uintptr_t)outputs[o] % 16 != 0) return fail(PF_ERR_ALIGNMENT, "output %d is not 16-byte aligned", o);
        const uintptr_t ob = (uintptr_t)outputs[o], oe = ob + plan->out_bytes[o];
        for (int k = 0; k < d.n_inputs; ++k) {
            const uintptr_t ib = (uintptr_t)inputs[k], ie = ib + plan->in_bytes[k];
            if (ob < ie && ib < oe) {
                const bool same = ob == ib && plan->out_bytes[o] == plan->in_bytes[k];
                // in place only where every element is read before it is written by the same lane
                const bool in_place_ok = plan->family == PF_FAMILY_ELEMENTWISE || plan->family == PF_FAMILY_ROW || plan->family == PF_FAMILY_GROUP;
                if (!same || !in_place_ok)
                    return fail(PF_ERR_ALIAS, "output %d overlaps input %d", o, k);
            }
        }
        for (int j = 0; j < o; ++j) {
            const uintptr_t jb = (uintptr_t)outputs[j], je = jb + plan->out_bytes[j];
            if (ob < je && jb < oe) return fail(PF_ERR_ALIAS, "outputs %d and %d overlap", j, o);
        }
    }
    const Lowered& L = plan->low;
    if (plan->family == PF_FAMILY_ATTENTION) {
        pf::AttnArgs at = plan->attn;
        at.q = inputs[L.attn_in[0]];
        at.k_new = L.attn_in[1] >= 0 ? inputs[L.attn_in[1]] : nullptr;
        at.v_new = L.attn_in[2] >= 0 ? inputs[L.attn_in[2]] : nullptr;
        at.k_cache = inputs[L.attn_in[3]];
        at.v_cache = inputs[L.attn_in[4]];
        at.o = outputs[L.attn_out[0]];
        at.k_out = L.attn_out[1] >= 0 ? outputs[L.attn_out[1]] : nullptr;
        at.v_out = L.attn_out[2] >= 0 ? outputs[L.attn_out[2]] : nullptr;
        const hipError_t ea = pf::launch_attn_decode(L.main_dtype, at, plan->variant, plan->k, plan->grid, (hipStream_t)stream);
        if (ea != hipSuccess) return fail(PF_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(ea));
        return PF_OK;
    }
    if (plan->family == PF_FAMILY_GATHER) {
        pf::GatherArgs ga = plan->gather;
        for (int k = 0; k < plan->desc.n_inputs; ++k) ga.in[k] = inputs[k];
        for (int o = 0; o < plan->desc.n_outputs; ++o) ga.out[o] = outputs[o];
        const hipError_t eg = pf::launch_gather(L.main_dtype, ga, plan->grid, (hipStream_t)stream);
        if (eg != hipSuccess) return fail(PF_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(eg));
        return PF_OK;
    }
    pf::ChainArgs a = plan->args;
    for (int f = 0; f < L.n_full; ++f) a.full[f] = inputs[L.full_input[f]];
    for (int v = 0; v < L.n_vec; ++v) a.vec[v].ptr = inputs[L.vec_input[v]];
    for (int s = 0; s < L.n_out; ++s) a.out[s] = outputs[L.out_slot_to_user[s]];
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    switch (plan->family) {
        case PF_FAMILY_ROW:
            if (plan->variant == PF_VARIANT_ROW_STREAM) {
                if (plan->spec_id == pf::kSpecJit) {
                    void* params[] = {&a};
                    e = pf::jit_launch(plan->jit_fn, plan->grid, plan->block, 0, params, st);
                } else {
                    e = pf::launch_row_stream(L.main_dtype, a, plan->ragged, plan->grid, st);
                }
            } else if (plan->spec_id == pf::kSpecJit) {
                pf::RowGeom g = plan->row;
                void* params[] = {&a, &g};
                e = pf::jit_launch(plan->jit_fn, plan->grid, plan->block, 0, params, st);
            } else if (plan->spec_id) e = pf::launch_row_static(plan->spec_id, L.main_dtype, a, plan->row, plan->k, plan->grid, plan->block, st);
            else e = pf::launch_row_generic(L.main_dtype, a, plan->row, plan->k, plan->reduce_only, plan->ragged, plan->grid, plan->block, st);
            break;
        case PF_FAMILY_ELEMENTWISE:
            if (plan->spec_id == pf::kSpecJit) {
                uint32_t total_vecs = plan->ew_total_vecs, vecs_per_row = plan->ew_vecs_per_row;
                void* params[] = {&a, &total_vecs, &vecs_per_row};
                e = pf::jit_launch(plan->jit_fn, plan->grid, plan->block, 0, params, st);
            } else {
                e = pf::launch_ew(L.main_dtype, a, plan->ew_total_vecs, plan->ew_vecs_per_row, plan->k, plan->ragged, plan->grid, st);
            }
            break;
        case PF_FAMILY_GROUP: {
            if (plan->variant == PF_VARIANT_GROUP_RESIDENT) {
                // the fused kernel alternates between two sets of exchange slots by launch number, which is a
                // kernel argument: a recorded launch would replay the same number
                hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
                if (hipStreamIsCapturing(st, &cs) == hipSuccess && cs != hipStreamCaptureStatusNone)
                    return fail(PF_ERR_UNSUPPORTED, "the one-launch GroupNorm variant cannot be recorded into a graph; plan the two-launch variant for that");
            }
            pf::GroupGeom g = plan->group;
            g.epoch = ++plan->epoch;
            const uint32_t tiles = g.samples * g.blocks_per_sample;
            if (plan->spec_id == pf::kSpecJit) {
                uint32_t t = tiles;
                void* params[] = {&a, &g, &t};
                e = pf::jit_launch(plan->jit_fn, plan->grid, plan->block, plan->dyn_lds, params, st);
                if (e == hipSuccess && plan->variant == PF_VARIANT_GROUP_TWO_PASS)
                    e = pf::jit_launch(plan->jit_fn2, plan->grid2, plan->block2, plan->dyn_lds, params, st);
            } else if (plan->variant == PF_VARIANT_GROUP_TWO_PASS) {
                const bool gen = plan->group_general;
                e = pf::launch_group(1, gen, plan->spec_id, L.main_dtype, a, g, plan->k, tiles, plan->grid, plan->block, plan->dyn_lds, st);
                if (e == hipSuccess)
                    e = pf::launch_group(2, gen, plan->spec_id, L.main_dtype, a, g, plan->k, tiles, plan->grid2, plan->block2, plan->dyn_lds, st);
            } else {
                e = pf::launch_group(0, false, plan->spec_id, L.main_dtype, a, g, plan->k, tiles, plan->grid, plan->block, 0, st);
            }
            break;
        }
        case PF_FAMILY_POOL:
            if (plan->spec_id == pf::kSpecJit) {
                pf::PoolGeom g = plan->pool;
                void* params[] = {&a, &g};
                e = pf::jit_launch(plan->jit_fn, plan->grid, plan->block, 0, params, st);
            } else {
                e = pf::launch_pool(L.main_dtype, a, plan->pool, L.pool_op, plan->k, plan->grid, st);
            }
            break;
        case PF_FAMILY_STENCIL:
            if (plan->spec_id == pf::kSpecJit) {
                pf::StencilGeom g = plan->stencil;
                void* params[] = {&a, &g};
                e = pf::jit_launch(plan->jit_fn, plan->grid, plan->block, plan->lds_bytes, params, st);
            } else {
                e = pf::launch_stencil(L.main_dtype, a, plan->stencil, plan->variant, plan->stencil_ks, plan->lds_bytes, plan->grid, st);
            }
            break;
        case PF_FAMILY_TRANSPOSE:
            if (plan->spec_id == pf::kSpecJit) {
                pf::PermGeom g = plan->permg;
                void* params[] = {&a, &g};
                e = pf::jit_launch(plan->jit_fn, plan->grid, plan->block, plan->variant == PF_VARIANT_T_LDS_ROWS ? plan->lds_bytes : 0u, params, st);
            } else {
                e = pf::launch_perm(plan->spec_id, L.main_dtype, a, plan->permg, plan->variant, plan->k, plan->ragged, plan->grid, plan->block,
                                    plan->lds_bytes, st);
            }
            break;
        default: return fail(PF_ERR_INVALID_ARG, "corrupt plan");
    }
    if (e != hipSuccess) return fail(PF_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(e));
    return PF_OK;
}

pf_status pf_chain_plan_poll_error(const pf_plan* plan, int32_t* flag) {
    if (!plan || !flag) return fail(PF_ERR_INVALID_ARG, "null argument");
    *flag = 0;
    uint32_t* err = plan->family == PF_FAMILY_GROUP ? plan->group.ws_error : plan->ws_error;
    if (!err) return PF_OK;
    uint32_t word = 0;
    if (hipMemcpy(&word, err, sizeof(word), hipMemcpyDeviceToHost) != hipSuccess)
        return fail(PF_ERR_HIP, "cannot read the error word");
    if (word != 0u && hipMemset(err, 0, sizeof(word)) != hipSuccess) return fail(PF_ERR_HIP, "cannot clear the error word");
    *flag = (int32_t)word;
    return PF_OK;
}

void pf_chain_plan_destroy(pf_plan* plan) {
    if (!plan) return;
    if (plan->workspace) (void)hipFree(plan->workspace);
    if (plan->bcast_dev) (void)hipFree(plan->bcast_dev);
    delete plan;
}

const char* pf_status_str(pf_status s) {
    switch (s) {
        case PF_OK: return "PF_OK";
        case PF_ERR_INVALID_ARG: return "PF_ERR_INVALID_ARG";
        case PF_ERR_SHAPE: return "PF_ERR_SHAPE";
        case PF_ERR_DTYPE: return "PF_ERR_DTYPE";
        case PF_ERR_UNSUPPORTED: return "PF_ERR_UNSUPPORTED";
        case PF_ERR_ALIGNMENT: return "PF_ERR_ALIGNMENT";
        case PF_ERR_ALIAS: return "PF_ERR_ALIAS";
        case PF_ERR_NOMEM: return "PF_ERR_NOMEM";
        case PF_ERR_HIP: return "PF_ERR_HIP";
        default: return "PF_ERR_UNKNOWN";
    }
}

const char* pf_last_error(void) { return g_last_error.c_str(); }

uint64_t pf_jit_compile_count(void) { return pf::jit_compile_count(); }

pf_status pf_copy_probe(const void* src, void* dst, uint64_t bytes, int32_t variant, void* stream) {
    if (!src || !dst) return fail(PF_ERR_INVALID_ARG, "null argument");
    if (bytes % 16 != 0 || (uintptr_t)src % 16 != 0 || (uintptr_t)dst % 16 != 0)
        return fail(PF_ERR_ALIGNMENT, "copy probe needs 16-byte aligned pointers and size");
    hipError_t e = pf::launch_copy_probe(src, dst, bytes, variant, (hipStream_t)stream);
    if (e != hipSuccess) return fail(PF_ERR_HIP, "copy probe launch failed: %s", hipGetErrorString(e));
    return PF_OK;
}

}  // extern "C"
