// Merge plans for chains that need more than one kernel.
//
// One kernel holds one exchange wider than a lane (a row reduction family, group statistics, a layout change,
// a pooling, a stencil): operators around it merge into its prologue and epilogue, and everything between two
// exchanges could go to either side.  The paper generates the candidate merge plans and picks one with a
// performance model that predicts a merged graph's time from its regular data movement (section 6, graph
// merging).  Here a merge plan is a set of cut points in the chain's operator order; the values that cross a cut
// are stored in device memory in fp32, whatever the chain's storage type: a chain computes in fp32 from its first
// load to its last store and rounds once, whether it is one kernel or several (a 16-bit chain of several kernels has
// its inputs widened and its outputs rounded by two conversion copies around the kernels, which the model prices).
// Every segment must lower to one kernel on its own; the model prices a segment at a launch cost plus
// the bytes it reads and writes over the bandwidth its kernel family reaches, and a dynamic programme over the
// cut points returns the cheapest plan under that model (the full search the paper prunes is tractable here
// because a chain has one operator order).
#include "pf_host_internal.h"

namespace pfh {

namespace {

// Performance model.  Launch cost and streaming rate are those of a plain copy kernel on this device
// (2.8 us + bytes / 6.7 TB/s); the family factors are the fractions of that rate the families' kernels reach on
// tensors of 75 to 170 MB (measured: element-wise 1.0, row normalisations 0.76 - 0.80, permutations that keep the
// innermost dimension 0.87, those that change it 0.7 - 0.8, group normalisation 0.65, pooling 0.6).
constexpr double kLaunchUs = 2.8;
constexpr double kCopyBytesPerUs = 6.7e6;

double family_factor(const Lowered& low) {
    switch (low.core) {
        case pf::CORE_NONE: return 0.97;
        case pf::CORE_PERMUTE: {
            const int rank = (int)low.pre_shape.size();
            return rank > 0 && low.perm[rank - 1] != rank - 1 ? 0.72 : 0.85;
        }
        case pf::CORE_GATHER: return 0.80;
        case pf::CORE_GROUPNORM: return 0.65;
        case pf::CORE_POOL: return 0.60;
        case pf::CORE_COLNORM: return 0.75;
        case pf::CORE_DWCONV: return 0.35;
        case pf::CORE_ATTN_DECODE: return 0.70;
        default: return 0.78;  // the row family's cores and row programs
    }
}

struct Segment {
    pf_chain_desc sub;
    int n_in = 0, n_out = 0;
    int in_value[PF_MAX_INPUTS];    // value id (of the whole chain) behind each input of the segment
    int out_value[PF_MAX_OUTPUTS];  // ... and behind each output
    uint64_t bytes = 0;
    double us = 0.0;
};

// The fp32 twin of a chain on 16-bit storage (same operators, every input and output fp32); false when the chain is
// fp32 already.
bool widened_twin(const pf_chain_desc* d, pf_chain_desc* twin) {
    if (d->n_outputs < 1 || d->out_dtype[0] == PF_F32) return false;
    *twin = *d;
    for (int k = 0; k < twin->n_inputs; ++k) twin->inputs[k].dtype = PF_F32;
    for (int o = 0; o < twin->n_outputs; ++o) twin->out_dtype[o] = PF_F32;
    return true;
}

// what the two conversion copies around the kernels of such a chain move
void cast_costs(const pf_chain_desc* d, const Checked& c, uint64_t* in_bytes, uint64_t* out_bytes) {
    *in_bytes = *out_bytes = 0;
    for (int k = 0; k < d->n_inputs; ++k) *in_bytes += (uint64_t)numel(c.shape[k]) * (dtype_size(d->inputs[k].dtype) + 4);
    for (int o = 0; o < d->n_outputs; ++o) *out_bytes += (uint64_t)numel(c.shape[d->out_value[o]]) * (dtype_size(d->out_dtype[o]) + 4);
}

// The conversion copies of a split chain on 16-bit storage are priced with its first and its last kernel.
void add_cast_costs(const pf_chain_desc* user, const Checked& c, int first, int last, uint64_t* bytes, double* us) {
    uint64_t in_bytes, out_bytes;
    cast_costs(user, c, &in_bytes, &out_bytes);
    if (first == 0) *bytes += in_bytes, *us += user->n_inputs * kLaunchUs + (double)in_bytes / (kCopyBytesPerUs * 0.97);
    if (last == user->n_ops) *bytes += out_bytes, *us += user->n_outputs * kLaunchUs + (double)out_bytes / (kCopyBytesPerUs * 0.97);
}

}  // namespace

// Builds the chain of operators [first, last) with everything it takes from outside as inputs and everything
// needed outside as outputs, and prices it.  PF_ERR_UNSUPPORTED when it is not one kernel.
static pf_status build_segment(const pf_chain_desc* d, const Checked& c, int first, int last, Segment* seg) {
    const int n_in = d->n_inputs;
    const int storage = d->out_dtype[0];
    pf_chain_desc& s = seg->sub;
    memset(&s, 0, sizeof(s));
    s.struct_size = sizeof(pf_chain_desc);
    s.version = d->version;
    std::vector<int> local(n_in + d->n_ops, -1);  // whole-chain value id -> id inside the segment
    // inputs, in order of first use
    for (int k = first; k < last; ++k) {
        const pf_op_desc& o = d->ops[k];
        for (int j = 0; j < o.n_src; ++j) {
            const int v = o.src[j];
            if (v >= n_in + first || local[v] >= 0) continue;
            if (seg->n_in == PF_MAX_INPUTS) return fail(PF_ERR_UNSUPPORTED, "operators %d..%d take more than %d tensors from outside", first, last - 1, PF_MAX_INPUTS);
            pf_tensor_desc& t = s.inputs[seg->n_in];
            if (v < n_in) {
                t = d->inputs[v];
            } else {
                const Shape& sh = c.shape[v];
                if (sh.size() > PF_MAX_RANK) return fail(PF_ERR_UNSUPPORTED, "value %d has more than %d dimensions", v, PF_MAX_RANK);
                t.dtype = storage;
                t.rank = (int32_t)sh.size();
                for (size_t i = 0; i < sh.size(); ++i) t.shape[i] = sh[i];
            }
            seg->in_value[seg->n_in] = v;
            local[v] = seg->n_in++;
        }
    }
    s.n_inputs = seg->n_in;
    for (int k = first; k < last; ++k) {
        pf_op_desc o = d->ops[k];
        for (int j = 0; j < o.n_src; ++j) o.src[j] = local[o.src[j]];
        local[n_in + k] = seg->n_in + (k - first);
        s.ops[k - first] = o;
    }
    s.n_ops = last - first;
    // outputs: results used by later operators, and the chain's own outputs
    for (int k = first; k < last; ++k) {
        const int v = n_in + k;
        bool later = false;
        for (int m = last; m < d->n_ops && !later; ++m)
            for (int j = 0; j < d->ops[m].n_src; ++j) later |= d->ops[m].src[j] == v;
        int user = -1;
        for (int o = 0; o < d->n_outputs; ++o)
            if (d->out_value[o] == v) user = o;
        if (!later && user < 0) continue;
        if (seg->n_out == PF_MAX_OUTPUTS) return fail(PF_ERR_UNSUPPORTED, "operators %d..%d produce more than %d tensors needed outside", first, last - 1, PF_MAX_OUTPUTS);
        // a chain output that later kernels read is read from the caller's buffer: it must be in the storage dtype
        if (later && user >= 0 && d->out_dtype[user] != storage) return fail(PF_ERR_UNSUPPORTED, "output %d is read again in another dtype", user);
        s.out_value[seg->n_out] = local[v];
        s.out_dtype[seg->n_out] = user >= 0 ? d->out_dtype[user] : storage;
        seg->out_value[seg->n_out++] = v;
    }
    if (seg->n_out == 0) return fail(PF_ERR_UNSUPPORTED, "operators %d..%d produce nothing that is used", first, last - 1);
    s.n_outputs = seg->n_out;

    // one kernel?  (as written, or with its basic operators recomposed)
    Checked sc;
    pf_status st = check_desc(&s, &sc);
    if (st != PF_OK) return st;
    Lowered low;
    st = lower_chain(&s, sc, &low);
    if (st != PF_OK) {
        pf_chain_desc composite;
        Checked cc;
        if (!recompose_chain(&s, sc, &composite) || check_desc(&composite, &cc) != PF_OK || lower_chain(&composite, cc, &low) != PF_OK) return st;
    }
    seg->bytes = 0;
    for (int k = 0; k < s.n_inputs; ++k) seg->bytes += (uint64_t)numel(sc.shape[k]) * dtype_size(s.inputs[k].dtype);
    for (int o = 0; o < s.n_outputs; ++o) seg->bytes += (uint64_t)numel(sc.shape[s.out_value[o]]) * dtype_size(s.out_dtype[o]);
    seg->us = kLaunchUs + (double)seg->bytes / (kCopyBytesPerUs * family_factor(low));
    return PF_OK;
}

pf_status segment_cost(const pf_chain_desc* d, int first, int last, double* us, uint64_t* bytes) {
    Checked c;
    pf_status st = check_desc(d, &c);
    if (st != PF_OK) return st;
    if (first < 0 || last > d->n_ops || first >= last) return fail(PF_ERR_INVALID_ARG, "operator range [%d, %d) is empty or outside the chain", first, last);
    // (a chain on 16-bit storage that is split runs as its fp32 twin: that is what a segment of it costs)
    pf_chain_desc twin;
    const bool whole = first == 0 && last == d->n_ops;
    const pf_chain_desc* dd = (!whole && widened_twin(d, &twin)) ? &twin : d;
    Segment seg;
    st = build_segment(dd, c, first, last, &seg);
    if (st != PF_OK) return st;
    if (dd != d) add_cast_costs(d, c, first, last, &seg.bytes, &seg.us);
    if (us) *us = seg.us;
    if (bytes) *bytes = seg.bytes;
    return PF_OK;
}

// The cheapest set of cuts under the model, never using a segment listed in `blocked` (pairs first, last).
pf_status partition_chain(const pf_chain_desc* user, const Checked& c, const std::vector<std::pair<int, int>>& blocked, pf_partition* out) {
    // a chain on 16-bit storage is split as its fp32 twin
    pf_chain_desc twin;
    const bool widen = widened_twin(user, &twin);
    const pf_chain_desc* d = widen ? &twin : user;
    const int n = d->n_ops;
    const double inf = 1e300;
    std::vector<double> best(n + 1, inf), seg_us((size_t)(n + 1) * (n + 1), 0.0);
    std::vector<uint64_t> seg_bytes((size_t)(n + 1) * (n + 1), 0);
    std::vector<int> from(n + 1, -1), parts(n + 1, 0);
    best[0] = 0.0;
    std::string first_error;
    for (int last = 1; last <= n; ++last) {
        for (int first = 0; first < last; ++first) {
            if (best[first] >= inf) continue;
            if (std::find(blocked.begin(), blocked.end(), std::make_pair(first, last)) != blocked.end()) continue;
            Segment seg;
            const bool whole = first == 0 && last == n;  // (the chain as one kernel runs on its own storage type)
            if (build_segment(whole ? user : d, c, first, last, &seg) != PF_OK) {
                if (first_error.empty()) first_error = last_error();
                continue;
            }
            if (widen && !whole) add_cast_costs(user, c, first, last, &seg.bytes, &seg.us);
            seg_us[(size_t)first * (n + 1) + last] = seg.us;
            seg_bytes[(size_t)first * (n + 1) + last] = seg.bytes;
            const double t = best[first] + seg.us;
            if (t < best[last]) best[last] = t, from[last] = first, parts[last] = parts[first] + 1;
        }
    }
    if (best[n] >= inf) return fail(PF_ERR_UNSUPPORTED, "no split of the chain into kernels is implemented (%s)", first_error.c_str());
    memset(out, 0, sizeof(*out));
    out->n_parts = parts[n];
    int last = n;
    for (int k = parts[n]; k > 0; --k) {
        const int first = from[last];
        out->first_op[k] = last;
        out->first_op[k - 1] = first;
        out->predicted_us[k - 1] = seg_us[(size_t)first * (n + 1) + last];
        out->bytes[k - 1] = seg_bytes[(size_t)first * (n + 1) + last];
        last = first;
    }
    return PF_OK;
}

// Plans every segment of the cheapest partition; a segment the device-side planning refuses is struck out and the
// search runs again.
pf_status plan_partitioned(const pf_chain_desc* user, int32_t device, pf_plan** out) {
    Checked c;
    pf_status st = check_desc(user, &c);
    if (st != PF_OK) return st;
    // kernels are planned for the fp32 twin of a chain on 16-bit storage; the plan widens and rounds around them
    pf_chain_desc twin;
    const bool widen = widened_twin(user, &twin);
    const pf_chain_desc* d = widen ? &twin : user;
    std::vector<std::pair<int, int>> blocked;
    blocked.push_back(std::make_pair(0, (int)d->n_ops));  // the caller has tried the whole chain as one kernel
    for (int attempt = 0; attempt < 64; ++attempt) {
        pf_partition part;
        st = partition_chain(user, c, blocked, &part);
        if (st != PF_OK) return st;
        pf_plan_s* p = new (std::nothrow) pf_plan_s();
        if (!p) return fail(PF_ERR_NOMEM, "out of host memory");
        p->desc = *user;
        p->device = device;
        p->composite = true;
        p->storage_dtype = user->out_dtype[0];
        // Tensors the plan owns live in one arena: values that cross a cut and are not chain outputs and, for a chain
        // on 16-bit storage, the fp32 copies of its inputs and outputs.
        std::vector<int> where(d->n_inputs + d->n_ops, -1);  // value id -> index into arena_offset
        std::vector<uint64_t> arena_offset;
        uint64_t arena_bytes = 0;
        auto arena_add = [&](int v) {
            where[v] = (int)arena_offset.size();
            arena_offset.push_back(arena_bytes);
            arena_bytes += ((uint64_t)numel(c.shape[v]) * sizeof(float) + 255) / 256 * 256;
            return where[v];
        };
        if (widen) {
            for (int k = 0; k < d->n_inputs; ++k) p->widen_in.push_back(pf_plan_s::Cast{k, arena_add(k), (uint64_t)numel(c.shape[k])});
            for (int o = 0; o < d->n_outputs; ++o) {
                const int v = d->out_value[o];
                if (where[v] < 0) arena_add(v);  // (two outputs may name one value)
                p->round_out.push_back(pf_plan_s::Cast{o, where[v], (uint64_t)numel(c.shape[v])});
            }
        }
        bool ok = true;
        for (int k = 0; k < part.n_parts && ok; ++k) {
            Segment seg;
            st = build_segment(d, c, part.first_op[k], part.first_op[k + 1], &seg);
            pf_plan* sub = nullptr;
            if (st == PF_OK) st = plan_one_kernel(&seg.sub, device, -1, &sub);
            if (st != PF_OK) {
                if (env_int("PF_LOG", 0)) fprintf(stderr, "[pf_chain] operators %d..%d cannot be planned as one kernel: %s\n", part.first_op[k], part.first_op[k + 1] - 1, last_error());
                blocked.push_back(std::make_pair(part.first_op[k], part.first_op[k + 1]));
                ok = false;
                break;
            }
            pf_plan_s::Part pp;
            pp.plan = sub;
            pp.n_in = seg.n_in, pp.n_out = seg.n_out;
            for (int i = 0; i < seg.n_in; ++i) {
                const int v = seg.in_value[i];
                if (v < d->n_inputs) {
                    if (widen) pp.in_kind[i] = 2, pp.in_index[i] = where[v];
                    else pp.in_kind[i] = 0, pp.in_index[i] = v;
                    continue;
                }
                int user_out = -1;
                for (int o = 0; o < d->n_outputs; ++o)
                    if (d->out_value[o] == v) user_out = o;
                if (user_out >= 0 && !widen) pp.in_kind[i] = 1, pp.in_index[i] = user_out;
                else pp.in_kind[i] = 2, pp.in_index[i] = where[v];
            }
            for (int o = 0; o < seg.n_out; ++o) {
                const int v = seg.out_value[o];
                int user_out = -1;
                for (int u = 0; u < d->n_outputs; ++u)
                    if (d->out_value[u] == v) user_out = u;
                if (user_out >= 0 && !widen) {
                    pp.out_kind[o] = 1, pp.out_index[o] = user_out;
                } else {
                    if (where[v] < 0) arena_add(v);
                    pp.out_kind[o] = 2, pp.out_index[o] = where[v];
                }
            }
            p->parts.push_back(pp);
        }
        if (ok) {
            if (arena_bytes) {
                if (hipSetDevice(device) != hipSuccess || hipMalloc(&p->arena, arena_bytes) != hipSuccess) {
                    (void)hipGetLastError();
                    pf_chain_plan_destroy(p);
                    return fail(PF_ERR_NOMEM, "no device memory for %llu bytes of tensors between kernels", (unsigned long long)arena_bytes);
                }
            }
            p->arena_bytes = arena_bytes;
            p->arena_offset = arena_offset;
            p->partition = part;
            p->family = p->parts[0].plan->family;
            p->variant = p->parts[0].plan->variant;
            p->grid = p->parts[0].plan->grid;
            p->block = p->parts[0].plan->block;
            p->n_launches = (int)(p->widen_in.size() + p->round_out.size());
            for (const pf_plan_s::Part& pp : p->parts) p->n_launches += pp.plan->n_launches;
            for (int k = 0; k < d->n_inputs; ++k) p->in_bytes[k] = (uint64_t)numel(c.shape[k]) * dtype_size(user->inputs[k].dtype);
            for (int o = 0; o < d->n_outputs; ++o) {
                p->out_shape[o] = c.shape[d->out_value[o]];
                p->out_bytes[o] = (uint64_t)numel(p->out_shape[o]) * dtype_size(user->out_dtype[o]);
            }
            if (env_int("PF_LOG", 0)) fprintf(stderr, "[pf_chain] %d kernels, %llu bytes between them\n", (int)p->parts.size(), (unsigned long long)arena_bytes);
            *out = p;
            return PF_OK;
        }
        pf_chain_plan_destroy(p);
    }
    return fail(PF_ERR_UNSUPPORTED, "no split of the chain into kernels could be planned");
}

}  // namespace pfh
