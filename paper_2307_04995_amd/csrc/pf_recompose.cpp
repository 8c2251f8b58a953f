// Recomposition: basic operators -> the composite operator they spell out.
//
// The paper splits every operator into the four basic kinds and lets the merged gOperator graph find the
// efficient schedule (section 6).  Here the efficient schedules are the hand-written cores, so the inverse step
// runs first: a sub-graph of basic operators that is exactly a softmax, a layer normalisation or an RMS
// normalisation over the last dimension is replaced by that operator when none of its interior values is
// used elsewhere.  The chain then gets the tuned core (scale and causal mask folded into the softmax, load
// skipping, the streaming variant for long rows, catalogue kernels) instead of a generic row program.  The
// rewritten chain computes the same function; anything that does not match stays a row program.
#include "pf_host_internal.h"

namespace pfh {

namespace {

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

}  // namespace

bool recompose_chain(const pf_chain_desc* d, const Checked& c, pf_chain_desc* out) {
    Recomposer rc;
    rc.d = d, rc.c = &c;
    return rc.run(out);
}

}  // namespace pfh
