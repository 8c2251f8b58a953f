"""pf_chain_run_static: the entry point that allocates nothing on the device.

Its kernels take their scratch memory (partial GroupNorm statistics, partial attention results and arrival
counters) from the library's static device array.  Every case runs two calls in a row on the same device, the
second with a smaller input, so that the second call meets whatever the first left in the array; each result must
equal, bit for bit, what pf_chain_plan + pf_chain_run produce with the same built-in kernels, and meet the parity
bars against the CPU oracle.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from pf_testlib import TORCH_DT, compare, env, oracle_run

pytestmark = pytest.mark.gpu


def run_static(spec, inputs):
    from paper_2307_04995_amd import binding as pf
    desc = pf.make_desc(spec)
    dev_in = [t.cuda() for t in inputs]
    outs = []
    for k, (_, dt) in enumerate(spec.outputs):
        st, t = pf.pf_chain_infer_shape(desc, desc.out_value[k])
        assert st == pf.PF_OK
        outs.append(torch.full(tuple(t.shape[j] for j in range(t.rank)), 768.0, dtype=TORCH_DT[dt], device="cuda"))
    st = pf.pf_chain_run_static(desc, 0, [t.data_ptr() for t in dev_in], [o.data_ptr() for o in outs],
                                torch.cuda.current_stream().cuda_stream)
    assert st == pf.PF_OK, pf.pf_last_error()
    torch.cuda.synchronize()
    return [o.cpu() for o in outs]


def run_planned(spec, inputs, variant=None):
    """The existing entry points, restricted to the built-in kernels (what the static entry point runs)."""
    from paper_2307_04995_amd import binding as pf
    with env(PF_JIT="0"):
        outs = pf.run_chain(spec, [t.cuda() for t in inputs], variant=variant)
    return [o.cpu() for o in outs]


def check_pair(build_big, build_small, variant=None):
    from paper_2307_04995_amd import binding as pf
    for which, (spec, ins) in (("first call", build_big), ("second call, smaller input", build_small)):
        got = run_static(spec, ins)
        ref = run_planned(spec, ins, variant)
        want = oracle_run(spec, ins)
        for g, r, w, (_, dt) in zip(got, ref, want, spec.outputs):
            assert np.array_equal(wl.raw_bits(g), wl.raw_bits(r)), f"{which}: differs from pf_chain_plan + pf_chain_run"
            compare(g, w, dt, which)
    assert pf.pf_jit_compile_count() >= 0


def test_groupnorm_silu_two_calls():
    from paper_2307_04995_amd import binding as pf
    check_pair(wl.c5_groupnorm_silu(n=3, h=24, w=40, ch=512, groups=32),
               wl.c5_groupnorm_silu(n=1, h=8, w=12, ch=256, groups=32),
               variant=pf.PF_VARIANT_GROUP_TWO_PASS)


def test_groupnorm_any_group_width_two_calls():
    from paper_2307_04995_amd import binding as pf
    check_pair(wl.x5_groupnorm_silu_wide_groups(n=2, h=20, w=20, ch=320, groups=32),
               wl.x5_groupnorm_silu_wide_groups(n=1, h=6, w=10, ch=160, groups=16),
               variant=pf.PF_VARIANT_GROUP_TWO_PASS)


def test_attention_two_calls():
    check_pair(wl.x2_decode_attention(b=2, h=5, t=700, d=64), wl.x2_decode_attention(b=1, h=3, t=130, d=64))


def test_chains_without_scratch():
    check_pair(wl.c3_bias_res_layernorm(rows=96, n=1024), wl.c2_causal_softmax(b=1, h=2, s=128))
    check_pair(wl.c4_bias_scale_permute(b=2, s=32, h=16, d=64), wl.c1_bias_res_layernorm_gelu(rows=16, n=768))


def test_interleaved_with_planned_runs():
    """Static calls between runs of an ordinary plan of another shape: neither disturbs the other."""
    from paper_2307_04995_amd import binding as pf
    spec_a, ins_a = wl.c5_groupnorm_silu(n=2, h=16, w=16, ch=512, groups=32)
    spec_b, ins_b = wl.c5_groupnorm_silu(n=1, h=12, w=12, ch=128, groups=8)
    ref_a = run_planned(spec_a, ins_a, pf.PF_VARIANT_GROUP_TWO_PASS)[0]
    ref_b = run_planned(spec_b, ins_b, pf.PF_VARIANT_GROUP_TWO_PASS)[0]
    for _ in range(3):
        assert np.array_equal(wl.raw_bits(run_static(spec_a, ins_a)[0]), wl.raw_bits(ref_a))
        assert np.array_equal(wl.raw_bits(run_planned(spec_a, ins_a, pf.PF_VARIANT_GROUP_TWO_PASS)[0]), wl.raw_bits(ref_a))
        assert np.array_equal(wl.raw_bits(run_static(spec_b, ins_b)[0]), wl.raw_bits(ref_b))


def test_too_large_for_the_scratch_array_is_refused():
    """Partial statistics beyond PF_STATIC_SCRATCH_BYTES: PF_ERR_NOMEM before anything is launched (the pointers passed
    are never touched, so small buffers stand in for the tensors)."""
    from paper_2307_04995_amd import binding as pf
    spec = wl.ChainSpec(inputs=[("f16", (64, 64, 64, 4096)), ("f16", (4096,)), ("f16", (4096,))])
    g = spec.op("groupnorm", 0, 1, 2, f=(1e-5, 0.0), i=(32,))
    spec.out(spec.op("silu", g), "f16")
    dummy = torch.zeros(4096, dtype=torch.float16, device="cuda")
    st = pf.pf_chain_run_static(pf.make_desc(spec), 0, [dummy.data_ptr()] * 3, [dummy.data_ptr()], torch.cuda.current_stream().cuda_stream)
    assert st == pf.PF_ERR_NOMEM, (st, pf.pf_last_error())
    assert "static scratch array" in pf.pf_last_error()
    torch.cuda.synchronize()


def test_refusals_name_the_other_entry_points():
    from paper_2307_04995_amd import binding as pf
    spec, ins = wl.x3_channel_shuffle(n=2, c=8, h=4, w=4, groups=2)
    desc = pf.make_desc(spec)
    dev = [t.cuda() for t in ins]
    outs = [torch.empty_like(dev[0]) for _ in spec.outputs]
    st = pf.pf_chain_run_static(desc, 0, [t.data_ptr() for t in dev], [o.data_ptr() for o in outs], 0)
    assert st == pf.PF_ERR_UNSUPPORTED and "pf_chain_plan" in pf.pf_last_error()
