// Checking of a chain description: operator table, shape rules (numpy broadcasting), per-value shapes.
#include "pf_host_internal.h"

namespace pfh {

static thread_local std::string g_last_error;

pf_status fail(pf_status s, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return s;
}

const char* last_error() { return g_last_error.c_str(); }

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



constexpr int64_t kMaxElements = (int64_t)1 << 40;  // of any one tensor of a chain

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
        // extents are positive and their product stays far from the range of a 64-bit integer (every later size
        // computation -- bytes, rows, vectors -- multiplies it by small factors only)
        int64_t n = 1;
        for (int64_t e : s) {
            if (e <= 0) return fail(PF_ERR_SHAPE, "input %d: non-positive extent", k);
            if (e > kMaxElements / n) return fail(PF_ERR_SHAPE, "input %d: more than 2^40 elements", k);
            n *= e;
        }
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
        if (o.n_i < 0 || o.n_i > PF_MAX_RANK) return fail(PF_ERR_INVALID_ARG, "op %d (%s): n_i %d out of range", k, tr.name, o.n_i);
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
                int64_t n_new = 1;
                for (int64_t e : r) {
                    if (e <= 0) return fail(PF_ERR_SHAPE, "op %d (reshape): non-positive extent", k);
                    if (e > kMaxElements / n_new) return fail(PF_ERR_SHAPE, "op %d (reshape): element count changes", k);
                    n_new *= e;
                }
                if (n_new != numel(a)) return fail(PF_ERR_SHAPE, "op %d (reshape): element count changes", k);
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

}  // namespace pfh
