"""Shared helpers of the GPU parity tests: run a chain through the C ABI, evaluate the oracle, compare."""
import os
from contextlib import contextmanager

import numpy as np
import torch

import workloads as wl

TORCH_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}

# Parity bars (the benchmark spec): fp32 max-abs 1e-5; 16-bit max-abs 2e-2 and max-rel 1e-2, the relative
# error evaluated where |oracle| >= 1e-3 (below that one rounding step of the storage type exceeds 1 %).
F32_ABS = 1e-5
H_ABS = 2e-2
H_REL = 1e-2
REL_FLOOR = 1e-3


@contextmanager
def env(**kw):
    old = {k: os.environ.get(k) for k in kw}
    try:
        for k, v in kw.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = str(v)
        yield
    finally:
        for k, v in old.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v


def gpu_run(spec, inputs, variant=None, generic=False, guard=True):
    """Run the chain on cuda:0 through the C ABI.  Returns (outputs on CPU, plan info).  With guard=True
    every output sits between two sentinel regions that must come back untouched."""
    from paper_2307_04995_amd import binding as pf
    dev_in = [t.cuda() for t in inputs]
    with env(PF_NO_STATIC="1" if generic else None):
        plan = pf.Plan(spec, 0, variant)
    info = plan.info()
    info.parts = plan.partition()  # the cut points the plan runs with (one part for a single kernel)
    shapes = plan.output_shapes()
    outs, guards = [], []
    pad = 512  # elements
    for shape, (_, dt) in zip(shapes, spec.outputs):
        n = int(np.prod(shape))
        buf = torch.full((n + 2 * pad,), 768.0, dtype=TORCH_DT[dt], device="cuda")
        guards.append(buf)
        outs.append(buf[pad:pad + n].view(shape))
    plan.run_ptrs([t.data_ptr() for t in dev_in], [o.data_ptr() for o in outs],
                  torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    res = []
    for buf, o in zip(guards, outs):
        if guard:
            head = buf[:pad].float().cpu()
            tail = buf[-pad:].float().cpu()
            assert torch.all(head == 768.0) and torch.all(tail == 768.0), "kernel wrote outside its output"
        res.append(o.detach().cpu().clone())
    plan.close()
    return res, info


def oracle_run(spec, inputs):
    from oracle import pf_oracle as orc
    return orc.evaluate_outputs(spec, [wl.widen(t) for t in inputs])


def compare(got: torch.Tensor, want: np.ndarray, dtype: str, what: str = ""):
    g = wl.widen(got)
    assert g.shape == want.shape, f"{what}: shape {g.shape} != {want.shape}"
    nan_g, nan_w = np.isnan(g), np.isnan(want)
    assert np.array_equal(nan_g, nan_w), f"{what}: NaN pattern differs"
    inf_w = np.isinf(want)
    assert np.array_equal(g[inf_w], want[inf_w]), f"{what}: infinities differ"
    ok = ~(nan_w | inf_w)
    diff = np.abs(g[ok] - want[ok])
    max_abs = float(diff.max()) if diff.size else 0.0
    if dtype == "f32":
        assert max_abs <= F32_ABS, f"{what}: max-abs {max_abs:.3e} > {F32_ABS}"
        return max_abs, 0.0
    big = np.abs(want[ok]) >= REL_FLOOR
    max_rel = float((diff[big] / np.abs(want[ok][big])).max()) if big.any() else 0.0
    assert max_abs <= H_ABS, f"{what}: max-abs {max_abs:.3e} > {H_ABS}"
    assert max_rel <= H_REL, f"{what}: max-rel {max_rel:.3e} > {H_REL}"
    return max_abs, max_rel


def ulp_histogram(got: torch.Tensor, want: np.ndarray, dtype: str):
    """Distance, in units in the last place of the storage type, between the result and the oracle rounded to
    that type; counts for 0, 1, 2, 3-4, 5-8 and more ulps.  A report, not a gate: the bars above decide."""
    tdt = TORCH_DT[dtype]
    ref = torch.from_numpy(want).to(torch.float32).to(tdt) if dtype != "f32" else torch.from_numpy(want).to(tdt)
    def ordered(t):  # bit patterns -> integers ordered like the values (negative zero and zero coincide)
        b = wl.raw_bits(t).astype(np.int64)
        sign = np.int64(1) << (8 * t.element_size() - 1)
        return np.where(b & sign, -(b & (sign - 1)), b)
    finite = np.isfinite(want)
    d = np.abs(ordered(got) - ordered(ref))[finite]
    edges = [0, 1, 2, 3, 5, 9, np.iinfo(np.int64).max]
    counts, _ = np.histogram(d, bins=edges)
    return {"0": int(counts[0]), "1": int(counts[1]), "2": int(counts[2]), "3-4": int(counts[3]), "5-8": int(counts[4]),
            ">8": int(counts[5]), "max": int(d.max()) if d.size else 0, "elements": int(d.size)}


# ---- chains that run as several kernels: the tensors between kernels are stored in the chain's storage type ----

def crossing_values(spec, parts):
    """Value ids produced in one part of a split chain and used in a later one."""
    n_in = len(spec.inputs)
    part_of = {}
    for k, (a, b, _, _) in enumerate(parts):
        for op in range(a, b):
            part_of[n_in + op] = k
    crossing = set()
    for k, op in enumerate(spec.ops):
        for v in op.src:
            if v >= n_in and part_of[v] != part_of[n_in + k]:
                crossing.add(v)
    return sorted(crossing)


def round_to(dtype, nudge_seed=None):
    """Rounding of a float64 array to the storage type; with a seed, every value is then moved one unit in the last
    place up or down at random (what a stored tensor may differ by when it was computed in fp32 instead of fp64)."""
    if dtype == "f32":
        return lambda a: a.astype(np.float32)

    def rnd(a):
        t = torch.from_numpy(np.ascontiguousarray(a)).to(TORCH_DT[dtype])
        if nudge_seed is not None:
            g = np.random.default_rng(nudge_seed + a.size)
            step = torch.from_numpy(g.choice(np.array([-1, 1], dtype=np.int16), size=a.shape))
            bits = t.view(torch.int16)
            ok = torch.isfinite(t) & ((bits & 0x7fff) > 1)
            t = torch.where(ok, bits + step, bits).view(TORCH_DT[dtype])
        return t.to(torch.float64).numpy()
    return rnd


def oracle_with_storage(spec, inputs, dtype, nudge=None, parts=None):
    """The oracle with the values that cross between the kernels of a split rounded to the storage type.  `parts` is
    the split (structure only: which operators each kernel runs; a plan reports its own), by default the one
    pf_chain_partition returns.  nudge = (value id, seed): that stored tensor is also moved by one unit in the last
    place per element."""
    from oracle import pf_oracle as orc
    if parts is None:
        from paper_2307_04995_amd import binding as pf
        st, parts = pf.pf_chain_partition(pf.make_desc(spec))
        assert st == pf.PF_OK
    stored = {v: round_to(dtype) for v in crossing_values(spec, parts)}
    if nudge is not None:
        stored[nudge[0]] = round_to(dtype, nudge[1])
    return orc.evaluate_outputs(spec, [wl.widen(t) for t in inputs], stored)


def compare_split_16bit(spec, inputs, outs, dtype, what, parts):
    """The 16-bit bars for a chain that ran as several kernels.  A tensor stored between two kernels may differ by
    one unit in the last place from the oracle's (fp32 against fp64 arithmetic before the rounding); where later
    operators amplify that (differences of nearly equal values), no implementation can meet the relative bar.
    Such elements are recognised by the oracle itself: for every stored tensor in turn, its result with that
    tensor's values moved one unit up or down at random (two draws), and the largest effects summed over the
    tensors.  An element passes with a relative error within the bar, or an error within twice that sum; the
    absolute bar holds everywhere, and the plain relative bar on at least 95 % of the elements."""
    wants = oracle_with_storage(spec, inputs, dtype, parts=parts)
    effect = [np.zeros_like(w) for w in wants]
    for v in crossing_values(spec, parts):
        worst = [np.zeros_like(w) for w in wants]
        for seed in (977, 1979):
            nudged = oracle_with_storage(spec, inputs, dtype, nudge=(v, seed), parts=parts)
            worst = [np.maximum(a, np.abs(n - w)) for a, n, w in zip(worst, nudged, wants)]
        effect = [e + a for e, a in zip(effect, worst)]
    for got, want, eff in zip(outs, wants, effect):
        g = wl.widen(got)
        assert g.shape == want.shape and np.all(np.isfinite(want)) and np.all(np.isfinite(g)), what
        diff = np.abs(g - want)
        assert diff.max() <= H_ABS, f"{what}: max-abs {diff.max():.3e} > {H_ABS}"
        big = np.abs(want) >= REL_FLOOR
        within = diff <= H_REL * np.abs(want)
        explained = diff <= 2.0 * eff
        bad = big & ~within & ~explained
        assert not bad.any(), (f"{what}: {bad.sum()} elements beyond the relative bar that stored rounding does not explain "
                               f"(worst {(diff[bad] / np.abs(want[bad])).max():.3e})")
        assert (big & within).sum() >= 0.95 * big.sum(), f"{what}: only {(big & within).sum()} of {big.sum()} elements within the relative bar"



SPEC_JIT = 255   # plan info spec_id of a kernel specialised for the chain when the plan was made


def check_chain(spec, inputs, variant=None, generic=False, what=""):
    outs, info = gpu_run(spec, inputs, variant=variant, generic=generic)
    stats = []
    if info.n_kernels > 1:
        # several kernels: the tensors between them are rounded to the storage type, and so are the oracle's
        dt0 = spec.outputs[0][1]
        if dt0 == "f32":
            for o, w, u in zip(outs, oracle_with_storage(spec, inputs, dt0, parts=info.parts), oracle_run(spec, inputs)):
                stats.append(compare(o, w, "f32", what))
                compare(o, u, "f32", what + " (unrounded)")
        else:
            compare_split_16bit(spec, inputs, outs, dt0, what, info.parts)
        return outs, info, stats
    wants = oracle_run(spec, inputs)
    for o, w, (_, dt) in zip(outs, wants, spec.outputs):
        stats.append(compare(o, w, dt, what))
    if not generic and info.spec_id == SPEC_JIT:
        # the chain is not in the built-in catalogue and got a kernel of its own: the run-time-interpreted
        # kernel it would have used otherwise is held to the same bar
        from paper_2307_04995_amd import binding as pf
        try:
            outs_i, info_i = gpu_run(spec, inputs, variant=variant, generic=True)
        except pf.PfError as e:
            # a forced variant may exist only in specialised form (e.g. an LDS tile that fits only when packed)
            if variant is None or e.status != pf.PF_ERR_UNSUPPORTED:
                raise
            outs_i, info_i = gpu_run(spec, inputs, variant=None, generic=True)
        assert info_i.spec_id == 0
        for o, w, (_, dt) in zip(outs_i, wants, spec.outputs):
            compare(o, w, dt, what + " (interpreted)")
    return outs, info, stats
