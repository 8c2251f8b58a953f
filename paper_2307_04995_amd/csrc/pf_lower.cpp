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
#include "pf_host_internal.h"

namespace pfh {


// ---------------------------------------------------------------------------------------------
// lowering
// ---------------------------------------------------------------------------------------------

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

    // A result computed from broadcast inputs alone (sigmoid of a per-row scale, say) is still smaller than the value
    // the kernel walks over; its inputs are addressed against the first full-size value it flows into.
    int partner_value(int id) const {
        int v = id;
        for (int hop = 0; hop < d->n_ops && numel(c->shape[v]) != region_numel; ++hop) {
            int next = -1;
            for (int k = v - d->n_inputs + 1; k < d->n_ops && next < 0; ++k)
                for (int j = 0; j < d->ops[k].n_src; ++j)
                    if (d->ops[k].src[j] == v) next = d->n_inputs + k;
            if (next < 0) break;
            v = next;
        }
        return v;
    }

    bool lower_elementwise_op(int k) {
        const pf_op_desc& o = d->ops[k];
        const int id = d->n_inputs + k;
        cur_result_shape = c->shape[partner_value(id)];
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

// Column family: move a dimension to the end, layer / RMS normalisation, move it back -- exactly these three
// operators on chain inputs, one output.  Swapping the normalisation across the two layout changes (section 5,
// operator swapping) leaves a normalisation over a strided dimension and no layout change at all.
static bool lower_column_norm(const pf_chain_desc* d, const Checked& c, Lowered* L) {
    if (d->n_ops != 3 || d->n_outputs != 1) return false;
    const int n_in = d->n_inputs;
    const pf_op_desc &p1 = d->ops[0], &nm = d->ops[1], &p2 = d->ops[2];
    if (kOps[p1.op].cls != OC_PERMUTE || kOps[p2.op].cls != OC_PERMUTE) return false;
    if (nm.op != PF_LAYERNORM && nm.op != PF_RMSNORM) return false;
    if (p1.src[0] >= n_in || nm.src[0] != n_in || p2.src[0] != n_in + 1 || d->out_value[0] != n_in + 2) return false;
    const Shape& in = c.shape[p1.src[0]];
    const int rank = (int)in.size();
    if (rank < 2 || p1.n_i != rank || p2.n_i != rank) return false;
    const int axis = (int)p1.i[rank - 1];
    if (axis >= rank - 1) return false;
    for (int q = 0; q < rank - 1; ++q)
        if (p1.i[q] != (q < axis ? q : q + 1)) return false;  // every other dimension keeps its place in the order
    for (int q = 0; q < rank; ++q)
        if (p1.i[p2.i[q]] != q) return false;  // the second permutation undoes the first
    const int gamma = nm.src[1], beta = nm.op == PF_LAYERNORM ? nm.src[2] : -1;
    if (gamma >= n_in || beta >= n_in) return false;
    const int dt = d->out_dtype[0];
    if (d->inputs[p1.src[0]].dtype != dt || d->inputs[gamma].dtype != dt || (beta >= 0 && d->inputs[beta].dtype != dt)) return false;
    if (c.shape[gamma].size() != 1 || c.shape[gamma][0] != in[axis]) return false;
    if (beta >= 0 && (c.shape[beta].size() != 1 || c.shape[beta][0] != in[axis])) return false;
    if (!std::isfinite(nm.f[0]) || nm.f[0] < 0.0f) return false;
    *L = Lowered();
    L->main_dtype = dt;
    L->core = pf::CORE_COLNORM;
    L->core_op = 1;
    L->eps = nm.f[0];
    L->col_in[0] = p1.src[0], L->col_in[1] = gamma, L->col_in[2] = beta;
    L->col_outer = 1, L->col_s = 1;
    for (int q = 0; q < axis; ++q) L->col_outer *= in[q];
    for (int q = axis + 1; q < rank; ++q) L->col_s *= in[q];
    L->col_c = in[axis];
    L->pre_shape = in;
    L->post_shape = in;
    L->n_out = 1;
    L->out_slot_to_user[0] = 0;
    return true;
}

pf_status lower_chain(const pf_chain_desc* d_in, const Checked& c, Lowered* L) {
    // A permutation that only moves extents of 1 leaves the order of the elements alone: it is a reshape (free),
    // not a layout change that needs a kernel of the transpose family.
    pf_chain_desc local = *d_in;
    for (int k = 0; k < local.n_ops; ++k) {
        pf_op_desc& o = local.ops[k];
        if (kOps[o.op].cls != OC_PERMUTE) continue;
        const Shape& in = c.shape[o.src[0]];
        const Shape& out = c.shape[local.n_inputs + k];
        int64_t last = -1;
        bool keeps_order = true;
        for (int q = 0; q < o.n_i; ++q) {
            if (in[o.i[q]] == 1) continue;
            keeps_order &= o.i[q] > last;
            last = o.i[q];
        }
        if (!keeps_order) continue;
        o.op = PF_RESHAPE;
        o.n_i = (int32_t)out.size();
        for (size_t q = 0; q < out.size(); ++q) o.i[q] = out[q];
    }
    // (a chain of nothing else stays a copy: a caller who asks for a permuted tensor gets one)
    bool computes = false;
    for (int k = 0; k < local.n_ops; ++k) computes |= kOps[local.ops[k].op].cls != OC_RESHAPE;
    const pf_chain_desc* d = computes ? &local : d_in;
    const int n_in = d->n_inputs, n_val = d->n_inputs + d->n_ops;
    if (lower_column_norm(d, c, L)) return PF_OK;
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

}  // namespace pfh
