"""GPU parity for chains written in basic operators only (element-wise, reduce over the last dimension,
broadcast of the reduced value back over its row): the reductions become steps of one register-resident
kernel.  Through the C ABI, element by element against the fp64 oracle."""
import numpy as np
import pytest

import workloads as wl
from pf_testlib import check_chain, env, gpu_run, SPEC_JIT

pytestmark = pytest.mark.gpu


@pytest.fixture(params=["row program", "recomposed"])
def recompose(request):
    """Chains that spell out a softmax or a normalisation run twice: as the row program their basic operators
    lower to (the rewrite into the composite operator switched off), and the way the planner takes them by
    default."""
    on = request.param == "recomposed"
    with env(PF_RECOMPOSE=None if on else "0"):
        yield on


def _pf():
    from paper_2307_04995_amd import binding as pf
    return pf


def _softmax_chain(dtype, shape, scale=None, causal=False):
    s = wl.ChainSpec(inputs=[(dtype, shape)])
    v = 0
    if scale is not None:
        v = s.op("scale", v, f=[scale])
    if causal:
        v = s.op("causal_mask", v)
    m = s.op("reduce_max", v)
    d = s.op("sub", v, m)
    e = s.op("exp", d)
    t = s.op("reduce_sum", e)
    s.out(s.op("div", e, t), dtype)
    return s


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("n", [512, 200, 197, 4096])
def test_softmax_in_basic_operators(n, dtype, recompose):
    shape = (3, 7, n)
    x = wl.random_tensor(shape, dtype, 1000 + n, scale=2.0)
    spec = _softmax_chain(dtype, shape, scale=0.25)
    _, info, _ = check_chain(spec, [x], what=f"softmax in basic operators n={n} {dtype}")
    pf = _pf()
    assert info.family == pf.PF_FAMILY_ROW and info.n_launches == 1
    comp = wl.ChainSpec(inputs=[(dtype, shape)])
    comp.out(comp.op("softmax", comp.op("scale", 0, f=[0.25])), dtype)
    y0, _ = gpu_run(spec, [x])
    y1, info1 = gpu_run(comp, [x])
    if recompose:
        # planned as the composite operator: the same kernel, the same bits
        assert (info.spec_id, info.variant, info.n_micro_ops) == (info1.spec_id, info1.variant, info1.n_micro_ops)
        assert np.array_equal(wl.raw_bits(y0[0]), wl.raw_bits(y1[0]))
    else:
        assert info.spec_id == SPEC_JIT and info.n_micro_ops > info1.n_micro_ops
        # the same numbers as the composite operator, to the storage type's rounding
        np.testing.assert_allclose(wl.widen(y0[0]), wl.widen(y1[0]), atol=4e-3 if dtype != "f32" else 1e-6)


@pytest.mark.parametrize("variant", [0, 1])
def test_causal_softmax_in_basic_operators(variant, recompose):
    shape = (2, 2, 64, 64) if variant == 0 else (1, 2, 1024, 1024)
    x = wl.random_tensor(shape, "f16", 1011, scale=2.0)
    spec = _softmax_chain("f16", shape, scale=0.125, causal=True)
    _, info, _ = check_chain(spec, [x], variant=variant, what="causal softmax in basic operators")
    assert info.variant == variant


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("rows,n", [(37, 768), (5, 1000), (9, 3000)])
def test_layernorm_in_basic_operators(rows, n, dtype, recompose):
    x = wl.random_tensor((rows, n), dtype, 1021, scale=0.5)
    res = wl.random_tensor((rows, n), dtype, 1022, scale=0.5)
    gamma = wl.random_tensor((n,), dtype, 1023, dist="positive", scale=0.8)
    beta = wl.random_tensor((n,), dtype, 1024, scale=0.3)
    s = wl.ChainSpec(inputs=[(dtype, (rows, n)), (dtype, (rows, n)), (dtype, (n,)), (dtype, (n,))])
    h = s.op("add", 0, 1)
    mu = s.op("reduce_mean", h)
    c = s.op("sub", h, mu)
    var = s.op("reduce_mean", s.op("mul", c, c))
    r = s.op("rsqrt", s.op("addc", var, f=[1e-5]))
    y = s.op("mul", c, r)
    y = s.op("add", s.op("mul", y, 2), 3)
    s.out(y, dtype)
    s.out(h, dtype)                      # the residual stream as a second output
    _, info, _ = check_chain(s, [x, res, gamma, beta], what=f"layernorm in basic operators n={n} {dtype}")
    assert info.family == _pf().PF_FAMILY_ROW and info.n_launches == 1
    assert (info.n_micro_ops < 6) if recompose else (info.n_micro_ops >= 10)


def test_rmsnorm_and_l1_normalisation_in_basic_operators(recompose):
    rows, n = 11, 520
    x = wl.random_tensor((rows, n), "bf16", 1031)
    gamma = wl.random_tensor((n,), "bf16", 1032, dist="positive", scale=0.8)
    s = wl.ChainSpec(inputs=[("bf16", (rows, n)), ("bf16", (n,))])
    ms = s.op("reduce_mean", s.op("mul", 0, 0))
    r = s.op("rsqrt", s.op("addc", ms, f=[1e-6]))
    s.out(s.op("mul", s.op("mul", 0, r), 1), "bf16")
    check_chain(s, [x, gamma], what="rmsnorm in basic operators")
    # x_i -> relu(x_i) / (sum_j relu(x_j) + 1): one reduction, the reduced value transformed before its use
    s = wl.ChainSpec(inputs=[("f32", (rows, n))])
    p = s.op("relu", 0)
    t = s.op("addc", s.op("reduce_sum", p), f=[1.0])
    s.out(s.op("div", p, t), "f32")
    check_chain(s, [wl.random_tensor((rows, n), "f32", 1033)], what="l1 normalisation")


def test_three_reductions_and_row_values_combined():
    # (x - mean) / (max - min + 1): three reductions, two row values combined with each other
    rows, n = 6, 333
    x = wl.random_tensor((rows, n), "f32", 1041)
    s = wl.ChainSpec(inputs=[("f32", (rows, n))])
    mean = s.op("reduce_mean", 0)
    hi = s.op("reduce_max", 0)
    lo = s.op("neg", s.op("reduce_max", s.op("neg", 0)))
    span = s.op("addc", s.op("sub", hi, lo), f=[1.0])
    s.out(s.op("div", s.op("sub", 0, mean), span), "f32")
    check_chain(s, [x], what="three reductions")


def test_in_line_reductions_need_rows_that_fit_a_workgroup():
    pf = _pf()
    s = wl.ChainSpec(inputs=[("f32", (2, 70000))])
    s.out(s.op("div", 0, s.op("addc", s.op("reduce_max", 0), f=[1.0])), "f32")
    with env(PF_PARTITION="0"):
        st, h = pf.pf_chain_plan(pf.make_desc(s), 0)
        assert st == pf.PF_ERR_UNSUPPORTED and h is None
    # as two kernels it runs: the reduction alone has a streaming variant, the division reads one value per row
    _, info, _ = check_chain(s, [wl.random_tensor((2, 70000), "f32", 1060, scale=2.0)], what="long rows, reduction and use in two kernels")
    assert info.n_kernels == 2
    # a softmax spelled in basic operators is planned as the operator, whose streaming variant has no such limit
    with env(PF_RECOMPOSE="0", PF_PARTITION="0"):
        st, h = pf.pf_chain_plan(pf.make_desc(_softmax_chain("f32", (2, 70000))), 0)
        assert st == pf.PF_ERR_UNSUPPORTED and h is None
    x = wl.random_tensor((2, 70000), "f32", 1061, scale=2.0)
    with env(PF_RECOMPOSE="0"):  # without the rewrite: one kernel per reduction, each streaming over the row
        _, info, _ = check_chain(_softmax_chain("f32", (2, 70000)), [x], what="long softmax in basic operators, several kernels")
        assert info.n_kernels >= 2
    _, info, _ = check_chain(_softmax_chain("f32", (2, 70000)), [x], what="long softmax in basic operators")
    assert info.variant == pf.PF_VARIANT_ROW_STREAM


@pytest.mark.parametrize("n", [256, 2048])
def test_in_line_maximum_propagates_nan(n):
    # one NaN poisons its row's maximum, hence everything derived from it; other rows are untouched
    x = wl.random_tensor((4, n), "f32", 1051)
    x[2, n // 3] = float("nan")
    s = wl.ChainSpec(inputs=[("f32", (4, n))])
    s.out(s.op("sub", 0, s.op("reduce_max", 0)), "f32")
    outs, _, _ = check_chain(s, [x], what="nan through an in-line maximum")
    y = wl.widen(outs[0])
    assert np.isnan(y[2]).all() and not np.isnan(y[[0, 1, 3]]).any()
