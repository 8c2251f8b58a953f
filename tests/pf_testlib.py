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


SPEC_JIT = 255   # plan info spec_id of a kernel specialised for the chain when the plan was made


def check_chain(spec, inputs, variant=None, generic=False, what=""):
    """Run the chain as planned and compare every output with the oracle at the bars above: one comparison for every
    chain, whether it runs as one kernel or as several."""
    outs, info = gpu_run(spec, inputs, variant=variant, generic=generic)
    # a plan that should have been specialised and fell back to the interpreter (a kernel header that no longer
    # compiles, say) would still compute the right values, several times slower: it must not pass unnoticed
    if not generic and os.environ.get("PF_JIT", "1") != "0" and os.environ.get("PF_NO_STATIC", "0") == "0" and "PF_JIT_INCLUDE" not in os.environ:
        assert info.interpreter_fallback == 0, f"{what}: the plan fell back to the interpreter"
    stats = []
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
