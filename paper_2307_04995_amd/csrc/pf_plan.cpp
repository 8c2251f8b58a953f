// Kernel-family planning: catalogue match or plan-time specialisation, launch geometry, workspace.
#include "pf_host_internal.h"
#include "pf_specs.h"

namespace pfh {

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
    if (L.general_bcast || L.scalar_vec) return 0;  // catalogue kernels are built without the general broadcast addressing
                                                    // and without the one-element operand case
    if (L.n_out != 1) return 0;
    for (const pf::SpecDesc& s : table) {
        if (s.nf != L.n_full || s.nv != L.n_vec || s.nt != L.n_tmp || s.core != L.core) continue;
        if (s.gamma != L.core_vec[0] || s.beta != L.core_vec[1]) continue;
        if (!list_equal(L.pro, s.pro, s.n_pro) || !list_equal(L.epi, s.epi, s.n_epi)) continue;
        return s.id;
    }
    return 0;
}


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
    j.flags = (L.general_bcast ? 1 : 0) | (L.scalar_vec ? 2 : 0);
    for (int i = 0; i < L.pro.n; ++i)
        j.pro.push_back((uint32_t)L.pro.u[i].code | ((uint32_t)L.pro.u[i].kind << 8) | ((uint32_t)L.pro.u[i].slot << 16));
    for (int i = 0; i < L.epi.n; ++i)
        j.epi.push_back((uint32_t)L.epi.u[i].code | ((uint32_t)L.epi.u[i].kind << 8) | ((uint32_t)L.epi.u[i].slot << 16));
    return j;
}

thread_local ScratchArena* tls_scratch = nullptr;

pf_status plan_workspace_alloc(pf_plan_s* p, uint64_t bytes, const char* what) {
    p->workspace_bytes = bytes;
    if (ScratchArena* a = tls_scratch) {
        const uint64_t at = (a->used + 255) / 256 * 256;
        if (at + bytes > a->cap)
            return fail(PF_ERR_NOMEM, "%s of %llu bytes does not fit the static scratch array (%llu bytes, %llu in use): use pf_chain_plan + pf_chain_run",
                        what, (unsigned long long)bytes, (unsigned long long)a->cap, (unsigned long long)at);
        p->workspace = a->base + at;
        p->workspace_borrowed = true;
        a->used = at + bytes;
        return PF_OK;
    }
    if (hipMalloc(&p->workspace, bytes) != hipSuccess) return fail(PF_ERR_NOMEM, "%s of %llu bytes failed", what, (unsigned long long)bytes);
    return PF_OK;
}

pf_status plan_workspace_fill(pf_plan_s* p, void* ptr, int byte, uint64_t bytes, bool must_hold) {
    if (bytes == 0) return PF_OK;
    if (planning_static()) {
        if (must_hold) p->fills.push_back(pf_plan_s::Fill{ptr, bytes, byte});
        return PF_OK;
    }
    if (hipMemset(ptr, byte, bytes) != hipSuccess) return fail(PF_ERR_HIP, "workspace clear failed");
    return PF_OK;
}

// A plan that should have got a kernel specialised for its chain runs on the run-time-interpreted kernels instead (the
// run-time compiler or the kernel headers are missing, or the compilation failed): several times slower, so the plan
// says so (pf_plan_info.interpreter_fallback) and keeps the reason for pf_last_error.
void note_interpreter_fallback(pf_plan_s* p, const std::string& why) {
    p->interpreter_fallback = true;
    p->fallback_reason = why;
    if (env_int("PF_LOG", 0)) fprintf(stderr, "[pf] plan-time specialisation unavailable, using the interpreter: %s\n", why.c_str());
}

// Plan-time specialisation needs the device (the compiled kernel is loaded onto it).
bool jit_possible(int device) {
    if (!pf::jit_enabled() || planning_static()) return false;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device < 0 || device >= n) return false;
    return hipSetDevice(device) == hipSuccess;
}


pf_status fill_vec_args(pf_plan_s* p, const Checked& c) {
    const Lowered& L = p->low;
    const int es = dtype_size(L.main_dtype);
    p->args.vec_plain_all = 1;
    for (int v = 0; v < L.n_vec; ++v) {
        const int in = L.vec_input[v];
        const int64_t n = numel(c.shape[in]);
        const int64_t inner = (L.vec_is_epi[v] ? L.post_shape : L.pre_shape).back();
        if (n != inner || c.shape[in].empty() || c.shape[in].back() != inner || (n * es) % 16 != 0) p->args.vec_plain_all = 0;
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
        if (n == 1) {
            p->low.scalar_vec = true;
            continue;
        }
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
        if (planning_static())
            return fail(PF_ERR_UNSUPPORTED, "broadcast inputs with extents of 1 inside their shape need a table in device memory: use pf_chain_plan + pf_chain_run");
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
        // With rows to spare, a wave that owns its row and idles through up to a quarter of its vector slots (they are
        // never loaded) still beats waves that share a row through LDS and barriers (768 fp32 columns, 65 536 rows:
        // 98.4 us against 106.6 us); with few rows the shared row wins, its lanes each doing a third of the arithmetic
        // (256 rows, replayed from a graph: 3.0 us against 3.6 us).
        if (wpr == 1 && rows >= 8192 && waste <= 0.26) score = k;
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
            else note_interpreter_fallback(p, err);
        }
        return PF_OK;
    }
    p->variant = best_wpr == 1 ? PF_VARIANT_ROW_WAVE : PF_VARIANT_ROW_BLOCK;
    p->k = best_k;
    p->row.waves_per_row = (uint32_t)best_wpr;
    p->row.rows_per_block = best_wpr >= 4 ? 1u : (uint32_t)(4 / best_wpr);
    if (best_wpr == 1 && env_int("PF_ROW_WAVES", 0) > 0) p->row.rows_per_block = (uint32_t)env_int("PF_ROW_WAVES", 4);
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
    // Waves that own their rows and have at most 2 KB of loads in flight each (one short row, or two whose tails a causal
    // mask cuts off) do better two to a workgroup than four: C2 15.3 -> 14.7 us, a plain softmax of 512 columns 18.3 ->
    // 17.9 us; with 4 KB per wave (C3) four are better (17.7 against 17.9 us), eight and sixteen worse for all.
    if (best_wpr == 1 && env_int("PF_ROW_WAVES", 0) == 0 && (int64_t)L.n_full * best_k * p->row.rows_per_wave * 1024 <= 2048) p->row.rows_per_block = 2;
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
        else note_interpreter_fallback(p, err);
    }
    if (!p->spec_id) {
        p->row.rows_per_wave = 1;
        p->row_log2l = 6;
    }
    {
        const int64_t rows_per_block = (int64_t)p->row.rows_per_block * p->row.rows_per_wave * (64 >> p->row_log2l);
        p->grid = dim3((uint32_t)((rows + rows_per_block - 1) / rows_per_block));
    }
    // Tensors of half a megabyte and more: the kernel is compiled for this shape (row length and count, mask period and
    // mode, waves per row as constants), which removes the tests and divisions in front of a wave's first load.  Not
    // below that: a compilation per shape is only worth it where the launch is long enough to notice.
    const int const_mode = env_int("PF_ROW_CONST", 1);
    if (p->spec_id && !reduce_only && jit_ok && const_mode != 0 && (const_mode == 2 || rows * n * es >= (512 << 10))) {
        pf::RowShapeConst sh;
        sh.n_inner = (uint32_t)n;
        sh.rows = (uint64_t)rows;
        sh.mask_si = L.mask_si;
        sh.core_mask = L.core_mask;
        sh.vec_plain_all = p->args.vec_plain_all;
        sh.waves_per_row = p->row.waves_per_row;
        sh.rows_per_block = p->row.rows_per_block;
        std::string err;
        hipFunction_t fn = pf::jit_row_kernel_const(p->device, L.main_dtype, p->k, (int)p->row.rows_per_wave, best_wpr == 1, p->ragged,
                                                   p->block.x <= 256 ? 256 : 1024, p->row_log2l, make_jit_spec(L), sh, &err);
        if (fn) {
            p->jit_fn = fn;
            p->spec_id = pf::kSpecJit;
        }
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
        else note_interpreter_fallback(p, err);
    }
    return PF_OK;
}


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
    bool uses_positions = L.n_vec != 0 || L.mask_si != 0 || L.core_mask != 0;
    for (int i = 0; i < L.pro.n; ++i) uses_positions |= L.pro.u[i].code == pf::U_MASK_CAUSAL;
    for (int i = 0; i < L.epi.n; ++i) uses_positions |= L.epi.u[i].code == pf::U_MASK_CAUSAL;
    const bool merge_ragged = ragged && !uses_positions && L.perm[rank - 1] != rank - 1 && env_int("PF_PERM_MERGE_RAGGED", 1) != 0;
    struct Dim { int64_t extent, in_stride; };
    std::vector<Dim> od;
    for (int q = 0; q < rank; ++q) {
        const int src = L.perm[q];
        if (in[src] == 1) continue;
        // (ragged: dimensions are not merged, so that the innermost dimension of each side is one the vectors of
        // broadcast operands and the partial last vector can be told from -- unless nothing in the chain looks at
        // positions: an innermost-changing permutation without broadcast operands or mask, where merging h and w of
        // a 7 x 7 feature map makes the transposed extent 49 instead of 7)
        if ((!ragged || merge_ragged) && !od.empty() && od.back().in_stride == in[src] * istr[src]) {
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
            else note_interpreter_fallback(p, err);
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
        // Two dimensions X, Y that swap around a kept innermost run ([.., Y, X, inner] -> [.., X, Y, inner]) and whose
        // run is short: walked in output order, a workgroup writes one long contiguous stretch but reads runs of `inner`
        // elements a whole X row apart.  Walking tx x ty blocks of (X, Y) instead gives both sides stretches of about
        // 512 bytes (C4, 128-byte runs: 14.3 us in output order, 13.3 us in blocks of 4 x 4; 2 x 2 to 4 x 16 within 0.2 us
        // of each other, 16 x 2 at 13.9 us).
        int tile_t = 0, tile_y = 0;
        if (!ragged && m >= 3 && m + 2 <= PF_DEV_MAX_RANK && od[m - 3].in_stride == inner && od[m - 2].in_stride == od[m - 3].extent * inner) {
            const int64_t run_bytes = inner * es;
            int64_t want = 1;
            while (want * 2 * run_bytes <= 512) want *= 2;
            int64_t tx = want, ty = want;
            while (tx > 1 && od[m - 3].extent % tx != 0) tx /= 2;
            while (ty > 1 && od[m - 2].extent % ty != 0) ty /= 2;
            const int forced = env_int("PF_PERM_BLOCK", -1), forced_y = env_int("PF_PERM_BLOCK_Y", forced);
            if (forced >= 1 && forced_y >= 1 && od[m - 3].extent % forced == 0 && od[m - 2].extent % forced_y == 0) tx = forced, ty = forced_y;
            if (forced != 0 && (tx > 1 || ty > 1)) tile_t = (int)tx, tile_y = (int)ty;
        }
        if (tile_t) {
            const Dim X = od[m - 3], Y = od[m - 2];
            const int64_t ox = ostr[m - 3], oy = ostr[m - 2];
            int r = 0;
            auto put = [&](int64_t extent, int64_t is, int64_t os) {
                g.extent[r] = (uint32_t)extent;
                g.in_stride[r] = (uint32_t)is;
                g.out_stride[r] = (uint32_t)os;
                g.div[r] = make_fastdiv(g.extent[r]);
                ++r;
            };
            for (int q = 0; q < m - 3; ++q) put(od[q].extent, od[q].in_stride, ostr[q]);
            put(X.extent / tile_t, X.in_stride * tile_t, ox * tile_t);
            put(Y.extent / tile_y, Y.in_stride * tile_y, oy * tile_y);
            put(tile_y, Y.in_stride, oy);
            put(tile_t, X.in_stride, ox);
            put(inner_vecs, 1, 1);
            g.rank = r;
        } else {
        g.rank = m;
        for (int q = 0; q < m; ++q) {
            g.extent[q] = (uint32_t)(q == m - 1 ? inner_vecs : od[q].extent);
            g.in_stride[q] = (uint32_t)od[q].in_stride;
            g.out_stride[q] = (uint32_t)ostr[q];
            g.div[q] = make_fastdiv(g.extent[q]);
        }
        }
        p->k = (g.total_vecs >= 65536u && !ragged) ? 2 : 1;
        if (!ragged && env_int("PF_PERM_K", 0) >= 1 && env_int("PF_PERM_K", 0) <= 16) p->k = env_int("PF_PERM_K", 2);
        g.tile_a = (uint32_t)inner;  // (ragged kernels: length of the innermost run)
        p->block = dim3(256);
        p->grid = dim3((g.total_vecs + 256u * p->k - 1) / (256u * p->k));
        p->lds_bytes = 0;
    }
    // Large tensors on the rows variant: the kernel is compiled for this geometry (index arithmetic on constants).  Worth
    // a compilation per shape only where the launch is long enough to notice; smaller ones keep the run-time geometry.
    if (p->variant == PF_VARIANT_T_ROWS && !ragged && !L.general_bcast && jit_possible(p->device) && env_int("PF_PERM_CONST", 1) != 0 &&
        (g.total_vecs >= (1u << 20) || env_int("PF_PERM_CONST", 1) == 2)) {
        uint32_t numel[PF_DEV_MAX_VEC] = {1, 1, 1, 1}, period[PF_DEV_MAX_VEC] = {1, 1, 1, 1};
        for (int v = 0; v < L.n_vec; ++v) {
            numel[v] = p->args.vec[v].numel;
            period[v] = p->args.vec[v].period_rows;
        }
        // eight vectors per lane (the built-in kernels exist for one and two): C4 12.9 us with two, 12.4 with four, 11.9
        // with eight, 12.0 with sixteen; six or twelve, which cut across the blocks, 13.0 - 13.6
        const int k_const = env_int("PF_PERM_K", 0) ? p->k : 8;
        std::string err;
        hipFunction_t fn = pf::jit_perm_rows_const(p->device, L.main_dtype, k_const, make_jit_spec(L), g, numel, period, &err);
        if (fn) {
            p->jit_fn = fn;
            p->spec_id = pf::kSpecJit;
            p->k = k_const;
            p->grid = dim3((g.total_vecs + 256u * p->k - 1) / (256u * p->k));
            return PF_OK;
        }
        if (p->k > 2) {
            p->k = 2;
            p->grid = dim3((g.total_vecs + 256u * p->k - 1) / (256u * p->k));
        }
    }
    if (!p->spec_id && jit_possible(p->device)) {
        std::string err;
        p->jit_fn = pf::jit_perm_kernel(p->device, L.main_dtype, p->variant, p->k, ragged, make_jit_spec(L), &err);
        if (p->jit_fn) p->spec_id = pf::kSpecJit;
        else note_interpreter_fallback(p, err);
    }
    return PF_OK;
}

// ---- group family
pf_status plan_group(pf_plan_s* p, int forced_variant) {
    // on the static scratch array: the two-launch variant, which waits for nobody and so has no failed wait to report
    if (planning_static()) forced_variant = PF_VARIANT_GROUP_TWO_PASS;
    const Lowered& L = p->low;
    const int es = dtype_size(L.main_dtype);
    const int vec = 16 / es;
    const Shape& sh = L.pre_shape;
    const int64_t samples = sh[0], C = sh.back();
    const int64_t hw = numel(sh) / (samples * C);
    const int64_t G = L.groups;
    // A channel count that is not a whole number of vectors: positions start at element alignment and end in a partial
    // vector.  The general kernels (interpreted or specialised now) read and write such vectors element by element.
    const bool ragged_c = (C * es) % 16 != 0;
    if (p->ragged && !ragged_c) return fail(PF_ERR_ALIGNMENT, "a broadcast input of the group family is not a multiple of 16 bytes");
    const int64_t cpg = C / G;
    const int64_t vpg = cpg / vec, cv = (C + vec - 1) / vec;
    // Groups that are a power-of-two number of whole vectors take the kernels' shuffle-tree path; any other width
    // takes the general one (per-element sums, parts merged through LDS).
    const bool general = ragged_c || cpg % vec != 0 || (vpg & (vpg - 1)) != 0 || vpg > 64 || env_int("PF_GROUP_GENERAL", 0) != 0;
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
    for (int64_t v = 0; v < cv; ++v) g.parts = std::max<uint32_t>(g.parts, (uint32_t)(std::min<int64_t>(v * vec + vec - 1, C - 1) / cpg - (v * vec) / cpg + 1));
    g.ragged = ragged_c ? 1u : 0u;
    const uint32_t gen_lds = general ? 512u * g.parts * 3u * (uint32_t)sizeof(float) : 0u;
    p->group_general = general;
    // 2: statistics straight from the packed 16-bit pairs (needs pairs that never straddle groups and nothing but the
    // load in front of the normalisation; the kernel checks the rest at compile time)
    // 3: channel counts that are not whole vectors; 4: both
    const bool packed_stats = cpg % 2 == 0 && L.main_dtype != PF_F32 && L.pro.n == 1;
    const int gen_parts = !general ? 0 : ragged_c ? (packed_stats ? 4 : 3) : (packed_stats ? 2 : 1);
    g.spin_limit = (uint32_t)env_int("PF_GROUP_SPIN_LIMIT", 1 << 22);  // polls before a wait gives up (tests force it small)
    p->family = PF_FAMILY_GROUP;
    p->spec_id = (env_int("PF_NO_STATIC", 0) || general) ? 0 : match_spec(spec_table().group, L);

    hipDeviceProp_t prop;
    if (hipSetDevice(p->device) != hipSuccess || hipGetDeviceProperties(&prop, p->device) != hipSuccess)
        return fail(PF_ERR_HIP, "cannot query device %d (the group family needs the device at plan time)", p->device);
    const int n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

    // Workgroups of 512 threads; a tile is NV position steps of 512 / cv positions each.
    // (workgroups of 256 or 128 threads, i.e. twice or four times the tiles, were measured on C5: 33.5 and 46.9 us
    // against 29.0; 1 024 threads, one workgroup per compute unit, 31.2 against 30.8)
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
        if (general && !((gen_parts == 2 || gen_parts == 4) && jit_possible(p->device)) && cands[ci] == 16 && !forced_nv) continue;  // (16 vectors fit the general kernels' registers only with packed statistics)
        uint32_t b;
        tiling(cands[ci], &b);
        if ((uint64_t)b * samples >= min_tiles || ci == 2 || forced_nv) {
            nv = cands[ci];
            bps = b;
        }
    }
    if (nv == 0) return fail(PF_ERR_INVALID_ARG, "PF_GROUP_NV must be 4, 8 or 16");
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
        if (fused_fn && nv == 16 && !forced_nv && pf::jit_scratch_bytes(fused_fn) > 0) {
            // The kernel of 16 vectors per lane does not fit the registers for this chain: what it spills goes through
            // memory once per workgroup (measured on [16,64,64,320] with groups of 10: 16 KiB per workgroup, traffic 1.16 x
            // the tensor).  Tiles of 12 steps do fit.
            uint32_t b12;
            tiling(12, &b12);
            hipFunction_t fn12 = pf::jit_group_kernel(p->device, L.main_dtype, 12, 0, gen_parts, jspec, &jit_err);
            if (fn12 && pf::jit_scratch_bytes(fn12) == 0) {
                fused_fn = fn12;
                nv = 12;
                bps = b12;
            }
        }
        if (!fused_fn) resident_ok = false;
    }
    const uint64_t tiles = (uint64_t)bps * samples;
    if (tiles > 0x7fffffffull) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the group family");
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
        // tensors of 4 MB and more: the kernel compiled for this geometry (see the kernel's header)
        const int const_mode = env_int("PF_GROUP_CONST", 1);
        if (!general && jit_possible(p->device) && const_mode != 0 && (const_mode == 2 || samples * hw * C * es >= (4 << 20))) {
            std::string err;
            hipFunction_t fn = pf::jit_group_kernel_const(p->device, L.main_dtype, nv, gen_parts, jspec, g, (uint32_t)tiles, res_grid, threads, &err);
            if (fn && pf::jit_blocks_per_cu(fn, (int)threads, gen_lds) * n_cu >= (int)res_grid) {
                p->jit_fn = fn;
                p->spec_id = pf::kSpecJit;
            }
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
        // (tiles of 12 steps exist in plan-time specialised form only)
        if (nv == 12 && p->spec_id != pf::kSpecJit) return fail(PF_ERR_UNSUPPORTED, "plan-time specialisation failed for the two-launch kernels: %s", jit_err.c_str());
    }
    if (jit_ok && p->spec_id == 0) note_interpreter_fallback(p, jit_err);
    p->lds_bytes = general ? gen_lds + 512 * 2 * 4 + 4 : 512 * 3 * 4 + 512 * 2 * 4 + 4;
    p->dyn_lds = gen_lds;
    // workspace: partials of the two-launch variant, or two parities of exchange words (all-ones = empty) of the
    // resident one; then the error word
    const uint64_t part_bytes = variant == PF_VARIANT_GROUP_RESIDENT ? 0 : (uint64_t)samples * g.blocks_per_sample * g.groups * 4 * sizeof(float);
    const uint64_t gather_bytes =
        variant == PF_VARIANT_GROUP_RESIDENT ? (((uint64_t)2 * samples * g.groups * g.blocks_per_sample * sizeof(uint64_t)) + 255) / 256 * 256 : 0;
    pf_status ws_st = plan_workspace_alloc(p, part_bytes + gather_bytes + 256, "workspace allocation");
    if (ws_st != PF_OK) return ws_st;
    char* ws = static_cast<char*>(p->workspace);
    if ((ws_st = plan_workspace_fill(p, ws, 0, part_bytes, false)) != PF_OK) return ws_st;
    if ((ws_st = plan_workspace_fill(p, ws + part_bytes, 0xff, gather_bytes, true)) != PF_OK) return ws_st;
    if ((ws_st = plan_workspace_fill(p, ws + part_bytes + gather_bytes, 0, 256, true)) != PF_OK) return ws_st;
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
    // a channel count that is not a whole number of vectors: element-aligned positions, a partial last vector
    const bool ragged_c = (ch * es) % 16 != 0;
    if (p->ragged && !ragged_c) return fail(PF_ERR_ALIGNMENT, "a broadcast input of the stencil family is not a multiple of 16 bytes");
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
    g.cv = (uint32_t)((ch + vec - 1) / vec);
    g.ragged = ragged_c ? 1u : 0u;
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
            p->jit_fn = pf::jit_stencil_kernel(p->device, L.main_dtype, p->variant, ksz, ragged_c, make_jit_spec(L), &err);
            if (p->jit_fn) p->spec_id = pf::kSpecJit;
            else note_interpreter_fallback(p, err);
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
        p->jit_fn = pf::jit_stencil_kernel(p->device, L.main_dtype, variant, ksz, ragged_c, make_jit_spec(L), &err);
        if (p->jit_fn) p->spec_id = pf::kSpecJit;
        else {
            note_interpreter_fallback(p, err);
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
    if (planning_static())
        return fail(PF_ERR_UNSUPPORTED, "layout-only chains with concat / slice need a run table in device memory: use pf_chain_plan + pf_chain_run");
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
    // vectors per lane: two once every compute unit still gets a dozen workgroups (concat -> channel shuffle -> split
    // of [128, 232, 28, 28] fp16: one 19.8 us, two 17.6 us, four 18.1 us)
    int k = work >= (uint64_t)2 * 256 * 4096 ? 2 : 1;
    const int forced_k = env_int("PF_GATHER_K", 0);
    if (forced_k == 1 || forced_k == 2 || forced_k == 4) k = forced_k;
    p->k = k;
    p->spec_id = 0;
    p->block = dim3(256);
    p->grid = dim3((uint32_t)((work + 256 * (uint64_t)k - 1) / (256 * (uint64_t)k)));
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
    // a channel count that is not a whole number of vectors: element-aligned positions, a partial last vector
    const bool ragged_c = (ch * es) % 16 != 0;
    if (p->ragged && !ragged_c) return fail(PF_ERR_ALIGNMENT, "a broadcast input of the pool family is not a multiple of 16 bytes");
    const int64_t cv = (ch + vec - 1) / vec;
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
    g.ragged = ragged_c ? 1u : 0u;
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
        if (planning_static())
            return fail(PF_ERR_UNSUPPORTED, "a pooling split over several workgroups per sample waits on the device, and a wait that gives up is reported "
                                            "through the plan: use pf_chain_plan + pf_chain_run");
        if (hipSetDevice(p->device) != hipSuccess) return fail(PF_ERR_HIP, "cannot select device %d", p->device);
        pf_status ws_st = plan_workspace_alloc(p, part_bytes + 256, "workspace allocation");
        if (ws_st != PF_OK) return ws_st;
        if ((ws_st = plan_workspace_fill(p, p->workspace, 0xff, part_bytes, true)) != PF_OK) return ws_st;
        if ((ws_st = plan_workspace_fill(p, static_cast<char*>(p->workspace) + part_bytes, 0, 256, true)) != PF_OK) return ws_st;
        g.ws_partial = reinterpret_cast<uint32_t*>(p->workspace);
        g.ws_error = reinterpret_cast<uint32_t*>(static_cast<char*>(p->workspace) + part_bytes);
        g.spin_limit = (uint32_t)env_int("PF_POOL_SPIN_LIMIT", 1 << 18);  // re-reads before a wait gives up (tests force it small)
        g.merge_rows = (uint32_t)std::max<int64_t>(1, 512 / ch);
        p->ws_error = g.ws_error;
    }
    if (jit_possible(p->device)) {
        std::string err;
        p->jit_fn = pf::jit_pool_kernel(p->device, L.main_dtype, nv, L.pool_op, ragged_c, make_jit_spec(L), &err);
        if (p->jit_fn) p->spec_id = pf::kSpecJit;
        else note_interpreter_fallback(p, err);
    }
    return PF_OK;
}

// ---- column family
pf_status plan_column(pf_plan_s* p) {
    const Lowered& L = p->low;
    const int es = dtype_size(L.main_dtype), vec = 16 / es;
    if (L.col_c > 1024) return fail(PF_ERR_UNSUPPORTED, "normalisation over a strided dimension holds at most 1024 values per position in registers (got %lld)", (long long)L.col_c);
    const int64_t s_vecs = (L.col_s + vec - 1) / vec, tiles = (s_vecs + 7) / 8;
    p->ragged = L.col_s % vec != 0;  // rows at element alignment, partial last vector
    if (L.col_outer * tiles > 0x7fffffffLL || L.col_outer * L.col_c * L.col_s > 0xffffffffLL * 4) return fail(PF_ERR_UNSUPPORTED, "tensor too large for the column family");
    pf::ColArgs& a = p->col;
    memset(&a, 0, sizeof(a));
    a.c = (uint32_t)L.col_c;
    a.s = (uint32_t)L.col_s;
    a.s_vecs = (uint32_t)s_vecs;
    a.tiles_per_outer = (uint32_t)tiles;
    a.inv_c = 1.0f / (float)L.col_c;
    a.eps = L.eps;
    // vectors per lane: the smallest instantiated count that holds the column (32 row groups per workgroup)
    p->k = 32;
    for (int kc : {24, 16, 12, 8, 6, 4, 3, 2, 1})
        if ((int64_t)kc * 32 >= L.col_c) p->k = kc;
    p->family = PF_FAMILY_COLUMN;
    p->variant = 0;
    p->spec_id = 0;
    p->grid = dim3((uint32_t)(L.col_outer * tiles));
    p->block = dim3(256);
    p->lds_bytes = 4 * 8 * (uint32_t)vec * 4;
    p->n_launches = 1;
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
    // A plan that owns its workspace merges by polling self-describing words (a bounded wait, reported through the plan);
    // a call that plans and runs in one go has no plan to report through and keeps the counted, wait-free merge.
    const bool polled = !planning_static() && env_int("PF_ATTN_POLLED", 1) != 0;
    pf_status ws_st = plan_workspace_alloc(p, part_bytes + cnt_bytes + 256, "workspace allocation");
    if (ws_st != PF_OK) return ws_st;
    if ((ws_st = plan_workspace_fill(p, p->workspace, polled ? 0xff : 0, part_bytes, polled)) != PF_OK) return ws_st;
    if ((ws_st = plan_workspace_fill(p, static_cast<char*>(p->workspace) + part_bytes, 0, cnt_bytes + 256, true)) != PF_OK) return ws_st;
    a.ws_partial = reinterpret_cast<float*>(p->workspace);
    a.ws_counter = reinterpret_cast<uint32_t*>(static_cast<char*>(p->workspace) + part_bytes);
    if (polled) {
        a.polled = 1;
        a.spin_limit = (uint32_t)env_int("PF_ATTN_SPIN_LIMIT", 1 << 20);  // re-reads before a wait gives up (tests force it small)
        a.ws_error = reinterpret_cast<uint32_t*>(static_cast<char*>(p->workspace) + part_bytes + cnt_bytes);
        p->ws_error = a.ws_error;
    }
    return PF_OK;
}

pf_status plan_checked_desc(const pf_chain_desc* desc, int32_t device, int32_t variant, pf_plan** out) {
    Checked c;
    pf_status s = check_desc(desc, &c);
    if (s != PF_OK) return s;
    pf_plan_s* p = new (std::nothrow) pf_plan_s();
    if (!p) return fail(PF_ERR_NOMEM, "out of host memory");
    const uint64_t scratch_used_before = tls_scratch ? tls_scratch->used : 0;
    p->desc = *desc;
    p->device = device;
    memset(&p->args, 0, sizeof(p->args));
    memset(&p->row, 0, sizeof(p->row));
    memset(&p->group, 0, sizeof(p->group));
    memset(&p->permg, 0, sizeof(p->permg));
    memset(&p->attn, 0, sizeof(p->attn));
    s = lower_chain(desc, c, &p->low);
    if (s == PF_OK && p->low.core != pf::CORE_ATTN_DECODE && p->low.core != pf::CORE_GATHER && p->low.core != pf::CORE_COLNORM) {
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
            case pf::CORE_COLNORM: s = plan_column(p); break;
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
    if (tls_scratch) tls_scratch->used = scratch_used_before;  // a plan that failed gives its share of the scratch array back
    return s;
}

pf_status plan_one_kernel(const pf_chain_desc* desc, int32_t device, int32_t variant, pf_plan** out) {
    Checked c;
    pf_status s = check_desc(desc, &c);
    if (s != PF_OK) return s;
    // a chain that spells a composite operator in basic operators is planned as that operator when that works
    if (env_int("PF_RECOMPOSE", 1) != 0) {
        pf_chain_desc composite;
        if (recompose_chain(desc, c, &composite) && plan_checked_desc(&composite, device, variant, out) == PF_OK) return PF_OK;
    }
    return plan_checked_desc(desc, device, variant, out);
}

}  // namespace pfh
