"""GPU parity for chains that need several kernels (section 6, graph merging): the library splits them where its
performance model says and runs the kernels in order on the caller's stream.  The tensors between the kernels are
fp32 whatever the storage type, so such a chain rounds once, on its last store, like a chain that is one kernel; it
is compared element by element with the plain fp64 oracle at the same bars."""
import numpy as np
import pytest
import torch

import workloads as wl
from pf_testlib import check_chain, env, oracle_run, compare

pytestmark = pytest.mark.gpu


def _pf():
    from paper_2307_04995_amd import binding as pf
    return pf


def _check(spec, inputs, dtype, what):
    outs, info, _ = check_chain(spec, inputs, what=what)
    assert info.n_kernels == len(info.parts) >= 1 and info.n_launches >= info.n_kernels, what  # (two row statistics alone are one row program)
    assert info.parts[0][0] == 0 and info.parts[-1][1] == len(spec.ops), what
    return outs, info


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("shape", [(2, 40, 7, 9), (1, 96, 14, 14), (3, 17, 5, 4)])
def test_layout_change_around_a_layer_normalisation(shape, dtype):
    # channels-first tensor, normalised over its channels: to channels-last, LayerNorm, back (three kernels)
    n, c, h, w = shape
    s = wl.ChainSpec(inputs=[(dtype, shape), (dtype, (c,)), (dtype, (c,))])
    v = s.op("silu", s.op("permute", 0, i=[0, 2, 3, 1]))  # (without the activation the form is one kernel: the column family)
    v = s.op("layernorm", v, 1, 2, f=[2.0 ** -20])
    v = s.op("permute", v, i=[0, 3, 1, 2])
    s.out(v, dtype)
    x = wl.random_tensor(shape, dtype, 3101)
    gam = wl.random_tensor((c,), dtype, 3102, dist="positive")
    bet = wl.random_tensor((c,), dtype, 3103, scale=0.3)
    outs, info = _check(s, [x, gam, bet], dtype, f"permute > silu > layernorm > permute {shape} {dtype}")
    assert info.n_kernels == 3 and tuple(outs[0].shape) == shape


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_softmax_then_layer_normalisation_with_steps_between(dtype):
    shape = (3, 33, 200)
    s = wl.ChainSpec(inputs=[(dtype, shape), (dtype, (200,)), (dtype, (200,)), (dtype, shape)])
    v = s.op("softmax", 0)
    v = s.op("gelu_erf", s.op("add", v, 3))
    v = s.op("layernorm", v, 1, 2, f=[2.0 ** -16])
    s.out(v, dtype)
    t = [wl.random_tensor(shape, dtype, 3111), wl.random_tensor((200,), dtype, 3112, dist="positive"),
         wl.random_tensor((200,), dtype, 3113, scale=0.3), wl.random_tensor(shape, dtype, 3114)]
    _, info = _check(s, t, dtype, f"softmax > add > gelu > layernorm {dtype}")
    assert info.n_kernels == 2


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_group_normalisation_then_global_pooling(dtype):
    shape = (2, 12, 12, 64)
    s = wl.ChainSpec(inputs=[(dtype, shape), (dtype, (64,)), (dtype, (64,))])
    v = s.op("silu", s.op("groupnorm", 0, 1, 2, f=[2.0 ** -16], i=[8]))
    v = s.op("reduce_mean", v, i=[1, 2])
    s.out(v, dtype)
    t = [wl.random_tensor(shape, dtype, 3121), wl.random_tensor((64,), dtype, 3122, dist="positive"), wl.random_tensor((64,), dtype, 3123, scale=0.3)]
    outs, info = _check(s, t, dtype, f"groupnorm > silu > mean over positions {dtype}")
    assert info.n_kernels == 2 and tuple(outs[0].shape) == (2, 1, 1, 64)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_a_value_that_is_an_output_and_feeds_the_next_kernel(dtype):
    # probabilities are an output of the chain and the input of the normalisation that follows.  fp32: the second
    # kernel reads them from the caller's output buffer.  16-bit: it reads the unrounded fp32 values the plan keeps.
    shape = (5, 16, 128)
    s = wl.ChainSpec(inputs=[(dtype, shape), (dtype, (128,))])
    p = s.op("softmax", 0)
    v = s.op("rmsnorm", p, 1, f=[2.0 ** -24])
    s.out(p, dtype)
    s.out(v, dtype)
    t = [wl.random_tensor(shape, dtype, 3131), wl.random_tensor((128,), dtype, 3132, dist="positive")]
    _, info = _check(s, t, dtype, "softmax (kept) > rmsnorm")
    assert info.n_kernels == 2
    if dtype == "f32":
        assert info.workspace_bytes == 0


def test_a_row_statistic_crosses_between_kernels():
    r, c = 96, 256
    s = wl.ChainSpec(inputs=[("f32", (r, c)), ("f32", (r, c)), ("f32", (c,))])
    m = s.op("sigmoid", s.op("reduce_max", s.op("softmax", 0)))
    s.out(s.op("rmsnorm", s.op("mul", 1, m), 2, f=[2.0 ** -20]), "f32")
    t = [wl.random_tensor((r, c), "f32", 3141), wl.random_tensor((r, c), "f32", 3142), wl.random_tensor((c,), "f32", 3143, dist="positive")]
    _check(s, t, "f32", "softmax > row maximum > scaled rmsnorm")


def test_plan_properties_repeated_runs_and_refusals():
    pf = _pf()
    shape = (2, 24, 6, 10)
    c = shape[1]
    s = wl.ChainSpec(inputs=[("f16", shape), ("f16", (c,)), ("f16", (c,))])
    v = s.op("permute", s.op("layernorm", s.op("silu", s.op("permute", 0, i=[0, 2, 3, 1])), 1, 2, f=[2.0 ** -20]), i=[0, 3, 1, 2])
    s.out(v, "f16")
    with env(PF_PARTITION="0"):
        with pytest.raises(pf.PfError) as e:
            pf.Plan(s, 0)
        assert e.value.status == pf.PF_ERR_UNSUPPORTED
    plan = pf.Plan(s, 0)
    info = plan.info()
    n = int(np.prod(shape))
    assert info.n_kernels == 3 and info.workspace_bytes >= 4 * n * 4   # input, two tensors between the kernels, output: all fp32
    assert info.compulsory_read_bytes == n * 2 + 2 * c * 2 and info.compulsory_write_bytes == n * 2
    stream = torch.cuda.current_stream().cuda_stream
    gam = wl.random_tensor((c,), "f16", 3152, dist="positive").cuda()
    bet = wl.random_tensor((c,), "f16", 3153, scale=0.3).cuda()
    out = torch.empty(shape, dtype=torch.float16, device="cuda")
    for rep in range(3):  # the tensors between the kernels are reused by every run
        x = wl.random_tensor(shape, "f16", 3160 + rep)
        xd = x.cuda()
        plan.run_ptrs([xd.data_ptr(), gam.data_ptr(), bet.data_ptr()], [out.data_ptr()], stream)
        torch.cuda.synchronize()
        wants = oracle_run(s, [x, gam.cpu(), bet.cpu()])
        compare(out.cpu(), wants[0], "f16", f"run {rep}")
    # in place is refused: the first kernel's output would be read by the second while the input is gone
    with pytest.raises(pf.PfError) as e:
        plan.run_ptrs([out.data_ptr(), gam.data_ptr(), bet.data_ptr()], [out.data_ptr()], stream)
    assert e.value.status == pf.PF_ERR_ALIAS
    assert plan.poll_error() == 0
    plan.close()


@pytest.mark.parametrize("seed", range(48))
def test_random_chains_of_several_kernels(seed):
    s, tensors, what = wl.random_multi_kernel_chain(seed)
    dtype = s.outputs[0][1]
    _check(s, tensors, dtype, what)
