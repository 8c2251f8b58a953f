"""Plan-time specialisation: a chain that is not in the built-in catalogue gets a kernel instantiated for its
structure when the plan is made; chains of the same structure share it; it can be switched off."""
import pytest

import workloads as wl
from pf_testlib import check_chain, env, gpu_run, SPEC_JIT

pytestmark = pytest.mark.gpu


def _chain(rows, n, dtype, scale):
    spec = wl.ChainSpec(inputs=[(dtype, (rows, n)), (dtype, (rows, n)), (dtype, (n,))])
    v = spec.op("mul", 0, 1)
    v = spec.op("add", v, 2)
    v = spec.op("scale", v, f=[scale])
    v = spec.op("softmax", v)
    spec.out(spec.op("addc", v, f=[0.25]), dtype)
    ins = [wl.random_tensor((rows, n), dtype, 901), wl.random_tensor((rows, n), dtype, 902), wl.random_tensor((n,), dtype, 903)]
    return spec, ins


def _compile_count():
    from paper_2307_04995_amd import binding as pf
    return pf.pf_jit_compile_count()


def test_unlisted_chain_gets_its_own_kernel_and_shares_it():
    spec, ins = _chain(33, 512, "f16", 0.5)
    _, info, _ = check_chain(spec, ins, what="specialised chain")
    assert info.spec_id == SPEC_JIT
    before = _compile_count()
    # same structure and launch shape, other row count and immediates: no new compilation
    spec2, ins2 = _chain(77, 512, "f16", 0.125)
    _, info2, _ = check_chain(spec2, ins2, what="specialised chain, reused")
    assert info2.spec_id == SPEC_JIT
    assert _compile_count() == before
    # another storage type is another kernel
    spec3, ins3 = _chain(9, 512, "f32", 0.5)
    _, info3, _ = check_chain(spec3, ins3, what="specialised chain, fp32")
    assert info3.spec_id == SPEC_JIT
    assert _compile_count() == before + 1


def test_specialisation_can_be_switched_off():
    spec, ins = _chain(5, 256, "f16", 0.5)
    with env(PF_JIT="0"):
        outs, info = gpu_run(spec, ins)
    assert info.spec_id == 0


def test_elementwise_and_ragged_chains_are_specialised():
    shape = (4, 9, 30)
    x = wl.random_tensor(shape, "bf16", 911)
    b = wl.random_tensor((30,), "bf16", 912)
    spec = wl.ChainSpec(inputs=[("bf16", shape), ("bf16", (30,))])
    v = spec.op("add", 0, 1)
    spec.out(spec.op("silu", v), "bf16")
    _, info, _ = check_chain(spec, [x, b], what="ragged element-wise, specialised")
    assert info.spec_id == SPEC_JIT
    x = wl.random_tensor((6, 197), "f16", 913)
    spec = wl.ChainSpec(inputs=[("f16", (6, 197))])
    spec.out(spec.op("softmax", 0), "f16")
    _, info, _ = check_chain(spec, [x], what="ragged softmax, specialised")
    assert info.spec_id == SPEC_JIT
