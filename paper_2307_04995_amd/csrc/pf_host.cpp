// Host side of the fused-chain library: description checking, shape inference, lowering of a chain to
// micro-programs, kernel-family choice, launch geometry, and the C ABI of include/pf_chain.h.
#include "pf_host_internal.h"

using namespace pfh;

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
    pf_chain_desc composite;
    const bool hit = recompose_chain(desc, c, &composite);
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
    // planning makes `device` current (allocations, the run-time compiler); the caller's current device is put back
    struct DeviceRestore {
        int prev = -1;
        ~DeviceRestore() {
            if (prev >= 0) (void)hipSetDevice(prev);
        }
    } restore;
    if (hipGetDevice(&restore.prev) != hipSuccess) restore.prev = -1;
    pf_status s = plan_one_kernel(desc, device, variant, out);
    if (s == PF_OK && (*out)->interpreter_fallback)  // PF_OK, but the caller can see why the plan is slow
        (void)fail(PF_OK, "plan-time specialisation unavailable, the run-time-interpreted kernels run: %s", (*out)->fallback_reason.c_str());
    // more than one exchange wider than a lane (or one a single kernel cannot hold): several kernels, split where the
    // performance model says the bytes are fewest
    if (s == PF_ERR_UNSUPPORTED && variant < 0 && desc->n_ops > 1 && env_int("PF_PARTITION", 1) != 0) {
        const std::string single = last_error();
        if (plan_partitioned(desc, device, out) == PF_OK) return PF_OK;
        const std::string split = last_error();
        return fail(s, "%s; as several kernels: %s", single.c_str(), split.c_str());
    }
    return s;
}

pf_status pf_chain_partition(const pf_chain_desc* desc, pf_partition* out) {
    Checked c;
    pf_status s = check_desc(desc, &c);
    if (s != PF_OK) return s;
    if (!out) return fail(PF_ERR_INVALID_ARG, "out is null");
    return partition_chain(desc, c, std::vector<std::pair<int, int>>(), out);
}

pf_status pf_chain_segment_cost(const pf_chain_desc* desc, int32_t first_op, int32_t last_op, double* us, uint64_t* bytes) {
    return segment_cost(desc, first_op, last_op, us, bytes);
}

}  // extern "C"

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
    info->n_kernels = 1;
    info->interpreter_fallback = plan->interpreter_fallback ? 1 : 0;
    if (plan->composite) {  // family, variant, grid and block are the first kernel's; the sums are the chain's
        info->n_kernels = (int32_t)plan->parts.size();
        info->workspace_bytes = plan->arena_bytes;
        info->n_micro_ops = 0;
        pf_plan_info sub;
        for (const pf_plan_s::Part& pp : plan->parts) {
            pf_chain_plan_get_info(pp.plan, &sub);
            info->workspace_bytes += sub.workspace_bytes;
            info->n_micro_ops += sub.n_micro_ops;
            info->lds_bytes = std::max(info->lds_bytes, sub.lds_bytes);
            info->interpreter_fallback |= sub.interpreter_fallback;
        }
        pf_chain_plan_get_info(plan->parts[0].plan, &sub);
        info->spec_id = sub.spec_id;
        info->vectors_per_lane = sub.vectors_per_lane;
    }
    return PF_OK;
}

pf_status pf_chain_plan_get_partition(const pf_plan* plan, pf_partition* out) {
    if (!plan || !out) return fail(PF_ERR_INVALID_ARG, "null argument");
    if (plan->composite) {
        *out = plan->partition;
        return PF_OK;
    }
    memset(out, 0, sizeof(*out));
    out->n_parts = 1;
    out->first_op[0] = 0;
    out->first_op[1] = plan->desc.n_ops;
    double us = 0.0;
    uint64_t bytes = 0;
    if (segment_cost(&plan->desc, 0, plan->desc.n_ops, &us, &bytes) == PF_OK) out->predicted_us[0] = us, out->bytes[0] = bytes;
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
                // (column family: a workgroup has its whole slab in registers before it stores any of it, and slabs are disjoint)
                const bool in_place_ok = plan->family == PF_FAMILY_ELEMENTWISE || plan->family == PF_FAMILY_ROW || plan->family == PF_FAMILY_GROUP ||
                                         plan->family == PF_FAMILY_COLUMN;
                if (!same || !in_place_ok)
                    return fail(PF_ERR_ALIAS, "output %d overlaps input %d", o, k);
            }
        }
        for (int j = 0; j < o; ++j) {
            const uintptr_t jb = (uintptr_t)outputs[j], je = jb + plan->out_bytes[j];
            if (ob < je && jb < oe) return fail(PF_ERR_ALIAS, "outputs %d and %d overlap", j, o);
        }
    }
    if (plan->composite) {
        // a value written by one kernel and read by the next may not share memory with anything the caller passed
        for (int o = 0; o < d.n_outputs; ++o)
            for (int k = 0; k < d.n_inputs; ++k) {
                const uintptr_t ob = (uintptr_t)outputs[o], oe = ob + plan->out_bytes[o], ib = (uintptr_t)inputs[k], ie = ib + plan->in_bytes[k];
                if (ob < ie && ib < oe) return fail(PF_ERR_ALIAS, "output %d overlaps input %d (the chain runs as several kernels)", o, k);
            }
        for (const pf_plan_s::Cast& w : plan->widen_in) {
            const hipError_t ew = pf::launch_cast(d.inputs[w.user].dtype, PF_F32, inputs[w.user], (char*)plan->arena + plan->arena_offset[w.slot], w.numel, (hipStream_t)stream);
            if (ew != hipSuccess) return fail(PF_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(ew));
        }
        for (const pf_plan_s::Part& pp : plan->parts) {
            const void* in[PF_MAX_INPUTS];
            void* outp[PF_MAX_OUTPUTS];
            for (int i = 0; i < pp.n_in; ++i)
                in[i] = pp.in_kind[i] == 0 ? inputs[pp.in_index[i]] : pp.in_kind[i] == 1 ? (const void*)outputs[pp.in_index[i]] : (const void*)((const char*)plan->arena + plan->arena_offset[pp.in_index[i]]);
            for (int o = 0; o < pp.n_out; ++o)
                outp[o] = pp.out_kind[o] == 1 ? outputs[pp.out_index[o]] : (void*)((char*)plan->arena + plan->arena_offset[pp.out_index[o]]);
            const pf_status ps = pf_chain_run(pp.plan, in, outp, stream);
            if (ps != PF_OK) return ps;
        }
        for (const pf_plan_s::Cast& r : plan->round_out) {
            const hipError_t er = pf::launch_cast(PF_F32, d.out_dtype[r.user], (const char*)plan->arena + plan->arena_offset[r.slot], outputs[r.user], r.numel, (hipStream_t)stream);
            if (er != hipSuccess) return fail(PF_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(er));
        }
        return PF_OK;
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
    if (plan->family == PF_FAMILY_COLUMN) {
        pf::ColArgs ca = plan->col;
        ca.x = inputs[L.col_in[0]];
        ca.gamma = inputs[L.col_in[1]];
        ca.beta = L.col_in[2] >= 0 ? inputs[L.col_in[2]] : nullptr;
        ca.out = outputs[0];
        const hipError_t ec = pf::launch_colnorm(L.main_dtype, ca, plan->k, L.col_in[2] < 0, plan->ragged, plan->grid, (hipStream_t)stream);
        if (ec != hipSuccess) return fail(PF_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(ec));
        return PF_OK;
    }
    if (plan->family == PF_FAMILY_GATHER) {
        pf::GatherArgs ga = plan->gather;
        for (int k = 0; k < plan->desc.n_inputs; ++k) ga.in[k] = inputs[k];
        for (int o = 0; o < plan->desc.n_outputs; ++o) ga.out[o] = outputs[o];
        const hipError_t eg = pf::launch_gather(L.main_dtype, ga, plan->k, plan->grid, (hipStream_t)stream);
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
            g.epoch = plan->epoch + 1;  // (counted below, once the launch has been accepted: a failed launch must not flip the slots' parity)
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
            if (e == hipSuccess) plan->epoch = g.epoch;
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
    if (plan->composite) {
        for (const pf_plan_s::Part& pp : plan->parts) {
            int32_t f = 0;
            const pf_status ps = pf_chain_plan_poll_error(pp.plan, &f);
            if (ps != PF_OK) return ps;
            *flag |= f;
        }
        return PF_OK;
    }
    uint32_t* err = plan->family == PF_FAMILY_GROUP ? plan->group.ws_error : plan->ws_error;
    if (!err) return PF_OK;
    uint32_t word = 0;
    if (hipMemcpy(&word, err, sizeof(word), hipMemcpyDeviceToHost) != hipSuccess)
        return fail(PF_ERR_HIP, "cannot read the error word");
    if (word != 0u) {
        // A wait gave up: the launch's outputs are invalid, and the exchange words may be in a state the next launch
        // does not expect (slots of the wrong parity still filled, partial results of late slices still published).  Put the
        // workspace back the way the planner left it.  (The caller has synchronised: nothing of this plan is running.)
        bool ok = hipMemset(err, 0, sizeof(word)) == hipSuccess;
        if (plan->family == PF_FAMILY_GROUP && plan->group.ws_gather) {
            const pf::GroupGeom& g = plan->group;
            ok = ok && hipMemset(g.ws_gather, 0xff, (size_t)2 * g.samples * g.groups * g.blocks_per_sample * sizeof(uint64_t)) == hipSuccess;
        }
        if (plan->family == PF_FAMILY_POOL && plan->pool.ws_partial)
            ok = ok && hipMemset(plan->pool.ws_partial, 0xff,
                                 (size_t)plan->pool.samples * plan->pool.blocks_per_sample * plan->pool.channels * sizeof(uint32_t)) == hipSuccess;
        if (plan->family == PF_FAMILY_ATTENTION && plan->attn.polled)
            ok = ok && hipMemset(plan->attn.ws_partial, 0xff, (size_t)plan->grid.x * plan->grid.y * plan->attn.part_stride * sizeof(float)) == hipSuccess;
        if (!ok) return fail(PF_ERR_HIP, "cannot re-arm the workspace");
    }
    *flag = (int32_t)word;
    return PF_OK;
}

void pf_chain_plan_destroy(pf_plan* plan) {
    if (!plan) return;
    if (plan->workspace && !plan->workspace_borrowed) (void)hipFree(plan->workspace);
    if (plan->bcast_dev) (void)hipFree(plan->bcast_dev);
    for (pf_plan_s::Part& pp : plan->parts) pf_chain_plan_destroy(pp.plan);
    if (plan->arena) (void)hipFree(plan->arena);
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

const char* pf_last_error(void) { return pfh::last_error(); }

uint64_t pf_jit_compile_count(void) { return pf::jit_compile_count(); }
uint64_t pf_jit_cache_hits(void) { return pf::jit_disk_hits(); }

pf_status pf_copy_probe(const void* src, void* dst, uint64_t bytes, int32_t variant, void* stream) {
    if (!src || !dst) return fail(PF_ERR_INVALID_ARG, "null argument");
    if (bytes % 16 != 0 || (uintptr_t)src % 16 != 0 || (uintptr_t)dst % 16 != 0)
        return fail(PF_ERR_ALIGNMENT, "copy probe needs 16-byte aligned pointers and size");
    hipError_t e = pf::launch_copy_probe(src, dst, bytes, variant, (hipStream_t)stream);
    if (e != hipSuccess) return fail(PF_ERR_HIP, "copy probe launch failed: %s", hipGetErrorString(e));
    return PF_OK;
}

}  // extern "C"
