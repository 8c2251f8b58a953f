"""GPU parity for reductions over the positions of a channels-last tensor (global pooling: the pool family),
through the C ABI, element by element against the fp64 oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
from pf_testlib import check_chain, compare, env, oracle_run

pytestmark = pytest.mark.gpu


def _pf():
    from paper_2307_04995_amd import binding as pf
    return pf


def _pool_chain(dtype, shape, op, pre=None, post=None):
    s = wl.ChainSpec(inputs=[(dtype, shape)])
    v = 0
    if pre:
        v = s.op(pre, v)
    v = s.op(op, v, i=list(range(1, len(shape) - 1)))
    if post:
        v = s.op(post, v)
    s.out(v, dtype)
    return s


@pytest.mark.parametrize("op", ["reduce_mean", "reduce_sum", "reduce_max"])
@pytest.mark.parametrize("shape,dtype", [((2, 7, 7, 64), "f16"), ((3, 14, 14, 240), "bf16"), ((1, 5, 96), "f32"), ((2, 64, 64, 128), "f16"),
                                         ((4, 1, 1, 8), "f32"), ((1, 3, 33, 17, 40), "f16"),
                                         # more than 512 channels: the merging workgroup's threads own several channels each
                                         ((4, 40, 40, 1024), "f16"), ((2, 30, 30, 2048), "f32"), ((3, 24, 24, 1280), "bf16")])
def test_global_pooling(shape, dtype, op):
    pf = _pf()
    positions = int(np.prod(shape[1:-1]))
    x = wl.random_tensor(shape, dtype, 2201, scale=(4.0 / positions) ** 0.5 if op == "reduce_sum" else 1.0)
    spec = _pool_chain(dtype, shape, op)
    outs, info, _ = check_chain(spec, [x], what=f"{op} over the positions of {shape} {dtype}")
    assert info.family == pf.PF_FAMILY_POOL and info.n_launches == 1
    assert tuple(outs[0].shape) == (shape[0],) + (1,) * (len(shape) - 2) + (shape[-1],)


@pytest.mark.parametrize("op", ["reduce_mean", "reduce_max"])
@pytest.mark.parametrize("shape,dtype", [((2, 7, 7, 12), "f16"), ((3, 14, 14, 100), "bf16"), ((2, 9, 9, 5), "f32"), ((2, 64, 64, 100), "f16"),
                                         ((4, 56, 56, 61), "f32"), ((2, 40, 40, 1001), "f16"), ((1, 30, 30, 3), "bf16")])
def test_channel_counts_that_are_not_whole_vectors(shape, dtype, op):
    # positions at element alignment, a partial last vector per position; slices of several workgroups included
    spec = _pool_chain(dtype, shape, op)
    _, info, _ = check_chain(spec, [wl.random_tensor(shape, dtype, 2260 + shape[-1])], what=f"ragged pooling {shape} {dtype} {op}")
    assert info.family == _pf().PF_FAMILY_POOL


def test_ragged_pooling_with_operands_on_both_sides_and_interpreted():
    # SiLU(x * s + r) -> mean -> * g + b with 100 channels: per-channel and full-shape operands gathered element by element
    # on both sides of the reduction; once specialised when the plan is made, once on the run-time-interpreted kernels
    shape, dtype, c = (3, 20, 20, 100), "f16", 100
    s = wl.ChainSpec(inputs=[(dtype, shape), (dtype, (c,)), (dtype, shape), (dtype, (c,)), (dtype, (shape[0], 1, 1, c))])
    v = s.op("mul", 0, 1)
    v = s.op("add", v, 2)
    v = s.op("silu", v)
    v = s.op("reduce_mean", v, i=[1, 2])
    v = s.op("mul", v, 3)
    v = s.op("add", v, 4)
    s.out(v, dtype)
    ins = [wl.random_tensor(shape, dtype, 2271), wl.random_tensor((c,), dtype, 2272), wl.random_tensor(shape, dtype, 2273),
           wl.random_tensor((c,), dtype, 2274), wl.random_tensor((shape[0], 1, 1, c), dtype, 2275)]
    _, info, _ = check_chain(s, ins, what="ragged pooling with operands")
    assert info.family == _pf().PF_FAMILY_POOL
    with env(PF_JIT="0"):
        _, info, _ = check_chain(s, ins, what="ragged pooling with operands, interpreted")
    assert info.spec_id == 0


def test_squeeze_step_of_a_squeeze_and_excite_block():
    # sigmoid(mean over H, W of SiLU(x * scale[c] + shift[c])): element-wise steps on both sides, broadcast operands
    n, h, w, c = 3, 12, 12, 96
    x = wl.random_tensor((n, h, w, c), "f16", 2211)
    scale = wl.random_tensor((c,), "f16", 2212, dist="positive")
    shift = wl.random_tensor((c,), "f16", 2213, scale=0.3)
    bias = wl.random_tensor((n, 1, 1, c), "f16", 2214, scale=0.3)
    s = wl.ChainSpec(inputs=[("f16", (n, h, w, c)), ("f16", (c,)), ("f16", (c,)), ("f16", (n, 1, 1, c))])
    v = s.op("silu", s.op("add", s.op("mul", 0, 1), 2))
    v = s.op("reduce_mean", v, i=[1, 2])
    s.out(s.op("sigmoid", s.op("add", v, 3)), "f16")
    check_chain(s, [x, scale, shift, bias], what="squeeze step")


@pytest.mark.parametrize("nv", [1, 2, 4, 8])
def test_every_slice_length_and_repeated_launches(nv):
    # several workgroups per sample: partial results, the counter that re-arms itself
    pf = _pf()
    shape = (3, 40, 40, 64)
    x = wl.random_tensor(shape, "f32", 2221)
    spec = _pool_chain("f32", shape, "reduce_mean", pre="relu")
    want = oracle_run(spec, [x])[0]
    with env(PF_POOL_NV=nv):
        plan = pf.Plan(spec, 0)
    assert plan.info().vectors_per_lane == nv
    dev = x.cuda()
    out = torch.empty((3, 1, 1, 64), dtype=torch.float32, device="cuda")
    for it in range(4):
        out.fill_(-1.0)
        plan.run([dev], [out])
        torch.cuda.synchronize()
        compare(out.cpu(), want, "f32", f"pooling, {nv} steps per workgroup, launch {it}")
    plan.close()


def test_maximum_keeps_a_nan_and_mean_of_constants_is_exact():
    x = wl.random_tensor((2, 9, 9, 32), "f32", 2231)
    x[1, 4, 5, 7] = float("nan")
    outs, _, _ = check_chain(_pool_chain("f32", (2, 9, 9, 32), "reduce_max"), [x], what="pooled maximum with a NaN")
    y = wl.widen(outs[0])
    assert np.isnan(y[1, 0, 0, 7]) and np.isnan(y).sum() == 1
    c = torch.full((2, 30, 30, 16), 0.625, dtype=torch.float16)
    outs, _, _ = check_chain(_pool_chain("f16", (2, 30, 30, 16), "reduce_mean"), [c], what="mean of a constant")
    assert torch.all(outs[0] == 0.625)


def test_other_sets_of_dimensions_are_refused():
    pf = _pf()
    for axes in ([1], [0, 1], [2, 3], [0]):
        s = wl.ChainSpec(inputs=[("f16", (2, 8, 8, 16))])
        s.out(s.op("reduce_sum", 0, i=axes), "f16")
        st, h = pf.pf_chain_plan(pf.make_desc(s), 0)
        assert st == pf.PF_ERR_UNSUPPORTED and h is None, axes
    s = wl.ChainSpec(inputs=[("f16", (2, 8, 8, 16))])
    s.out(s.op("reduce_sum", 0, i=[2, 1]), "f16")          # not ascending
    assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_ERR_INVALID_ARG
    # the last dimension named explicitly is the row reduction
    s = wl.ChainSpec(inputs=[("f16", (2, 8, 8, 16))])
    s.out(s.op("reduce_sum", 0, i=[3]), "f16")
    _, info, _ = check_chain(s, [wl.random_tensor((2, 8, 8, 16), "f16", 2241)], what="last dimension named")
    assert info.family == pf.PF_FAMILY_ROW


def test_bounded_wait_of_the_merging_workgroup_gives_up_instead_of_hanging():
    # with the polling limit forced to zero the sample's last workgroup does not wait for the others: the launch
    # must still end, and the plan must report it (results of such a launch are not checked)
    pf = _pf()
    shape = (4, 64, 64, 64)
    spec = _pool_chain("f16", shape, "reduce_mean")
    with env(PF_POOL_SPIN_LIMIT="0"):
        plan = pf.Plan(spec, 0)
    x = wl.random_tensor(shape, "f16", 2251).cuda()
    out = torch.empty((4, 1, 1, 64), dtype=torch.float16, device="cuda")
    for _ in range(3):
        plan.run([x], [out])
    torch.cuda.synchronize()
    assert plan.poll_error() in (0, 1)      # usually 1; 0 only if every flag happened to be up at the first look
    assert plan.poll_error() == 0           # reading clears it
    plan.close()
    # a plan with the default limit on the same shape is exact again (the flags were left in whatever state: new plan, new flags)
    check_chain(spec, [x.cpu()], what="pooling after a forced give-up")
