"""GPU parity for the streaming row variant: rows longer than a workgroup keeps in registers (a workgroup
walks the row twice in chunks), also forced onto short rows so that its chunk logic meets every core."""
import numpy as np
import pytest

import workloads as wl
from pf_testlib import check_chain, gpu_run

pytestmark = pytest.mark.gpu


def _pf():
    from paper_2307_04995_amd import binding as pf
    return pf


@pytest.mark.parametrize("n,dtype", [(50257, "f16"), (40000, "bf16"), (70001, "f32"), (200, "f16"), (1024, "f32")])
def test_stream_scaled_softmax(n, dtype):
    # 50257: a vocabulary-sized row, odd length (rows start on 2-byte boundaries)
    rows = 3
    x = wl.random_tensor((rows, n), dtype, 800 + n % 97, scale=3.0)
    spec = wl.ChainSpec(inputs=[(dtype, (rows, n))])
    v = spec.op("scale", 0, f=[0.5])
    spec.out(spec.op("softmax", v), dtype)
    pf = _pf()
    _, info, _ = check_chain(spec, [x], variant=pf.PF_VARIANT_ROW_STREAM, what=f"stream softmax n={n} {dtype}")
    assert info.variant == pf.PF_VARIANT_ROW_STREAM
    if n > 40000:
        _, info, _ = check_chain(spec, [x], what=f"long softmax n={n} {dtype} (planner's choice)")
        assert info.variant == pf.PF_VARIANT_ROW_STREAM


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_stream_causal_softmax_long_keys(dtype):
    # 5 query rows against 20011 keys: the diagonal cuts the very first chunk, later chunks are never loaded
    spec, ins = wl.c2_causal_softmax(b=1, h=2, s=5, s_k=20011, dtype=dtype)
    pf = _pf()
    check_chain(spec, ins, variant=pf.PF_VARIANT_ROW_STREAM, what="stream causal softmax")
    spec, ins = wl.c2_causal_softmax(b=1, h=1, s=9001, s_k=9001, dtype=dtype)
    check_chain(spec, ins, variant=pf.PF_VARIANT_ROW_STREAM, what="stream causal softmax, square")


@pytest.mark.parametrize("rows,n,dtype", [(3, 33000, "f16"), (2, 20001, "f32"), (4, 16385, "bf16"), (5, 768, "f32")])
def test_stream_bias_residual_layernorm_two_outputs(rows, n, dtype):
    x = wl.random_tensor((rows, n), dtype, 811, scale=0.4)
    res = wl.random_tensor((rows, n), dtype, 812, scale=0.4)
    bias = wl.random_tensor((n,), dtype, 813, scale=0.4)
    gamma = wl.random_tensor((n,), dtype, 814, dist="positive", scale=0.6)
    beta = wl.random_tensor((n,), dtype, 815, scale=0.3)
    spec = wl.ChainSpec(inputs=[(dtype, (rows, n)), (dtype, (rows, n)), (dtype, (n,)), (dtype, (n,)), (dtype, (n,))])
    h = spec.op("add", 0, 1)
    h = spec.op("add", h, 2)
    y = spec.op("layernorm", h, 3, 4, f=[1e-5])
    y = spec.op("gelu_erf", y)
    spec.out(y, dtype)
    spec.out(h, dtype)
    check_chain(spec, [x, res, bias, gamma, beta], variant=_pf().PF_VARIANT_ROW_STREAM, what=f"stream layernorm n={n} {dtype}")


def test_stream_layernorm_large_offset():
    # a common offset much larger than the spread: the streamed statistics must not cancel
    rows, n = 2, 40000
    x = wl.random_tensor((rows, n), "f32", 821, scale=0.5) + 300.0
    gamma = wl.random_tensor((n,), "f32", 822, dist="positive", scale=1.0)
    beta = wl.random_tensor((n,), "f32", 823, scale=0.5)
    spec = wl.ChainSpec(inputs=[("f32", (rows, n)), ("f32", (n,)), ("f32", (n,))])
    spec.out(spec.op("layernorm", 0, 1, 2, f=[1e-5]), "f32")
    # the inputs carry 300 +- 2 in fp32 (spacing 3e-5); normalised by a spread of 0.5 the result is held to 1e-4
    outs, info = gpu_run(spec, [x, gamma, beta], variant=_pf().PF_VARIANT_ROW_STREAM)
    from pf_testlib import oracle_run
    want = oracle_run(spec, [x, gamma, beta])[0]
    assert np.abs(wl.widen(outs[0]) - want).max() < 1e-4


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_stream_rmsnorm(dtype):
    rows, n = 3, 24001
    x = wl.random_tensor((rows, n), dtype, 831)
    gamma = wl.random_tensor((n,), dtype, 832, dist="positive", scale=0.8)
    spec = wl.ChainSpec(inputs=[(dtype, (rows, n)), (dtype, (n,))])
    spec.out(spec.op("rmsnorm", 0, 1, f=[1e-6]), dtype)
    check_chain(spec, [x, gamma], variant=_pf().PF_VARIANT_ROW_STREAM, what="stream rmsnorm")


@pytest.mark.parametrize("op", ["reduce_sum", "reduce_max", "reduce_mean"])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_stream_reduce_keepdim(op, dtype):
    shape = (3, 2, 30011)
    x = wl.random_tensor(shape, dtype, 841, scale=0.01 if op == "reduce_sum" else 0.5)
    spec = wl.ChainSpec(inputs=[(dtype, shape)])
    v = spec.op("relu", 0)
    v = spec.op(op, v)
    spec.out(spec.op("scale", v, f=[0.5]), dtype)
    check_chain(spec, [x], variant=_pf().PF_VARIANT_ROW_STREAM, what=f"stream {op}")
