"""GPU parity for innermost extents that are not a multiple of a 16-byte vector (element-granular kernels of
the row, element-wise and transpose families), through the C ABI, element by element against the fp64 oracle."""
import numpy as np
import pytest

import workloads as wl
from pf_testlib import check_chain, gpu_run

pytestmark = pytest.mark.gpu


def _pf():
    from paper_2307_04995_amd import binding as pf
    return pf


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("n", [197, 50, 3, 1])
def test_ragged_scaled_softmax(n, dtype):
    # attention scores of a sequence length that is not a multiple of 8 (e.g. 196 patches + 1 class token)
    shape = (2, 3, min(n, 40), n)
    x = wl.random_tensor(shape, dtype, 700 + n, scale=2.0)
    spec = wl.ChainSpec(inputs=[(dtype, shape)])
    v = spec.op("scale", 0, f=[0.125])
    spec.out(spec.op("softmax", v), dtype)
    _, info, _ = check_chain(spec, [x], what=f"ragged softmax n={n} {dtype}")
    assert info.family == _pf().PF_FAMILY_ROW
    y, _ = gpu_run(spec, [x])
    np.testing.assert_allclose(wl.widen(y[0]).sum(-1), 1.0, atol=6e-3)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_ragged_causal_softmax(dtype):
    spec, ins = wl.c2_causal_softmax(b=1, h=2, s=50, dtype=dtype)
    check_chain(spec, ins, what="ragged causal softmax")
    spec, ins = wl.c2_causal_softmax(b=1, h=1, s=37, s_k=61, dtype=dtype)
    check_chain(spec, ins, what="ragged rectangular causal softmax")


@pytest.mark.parametrize("rows,n,dtype", [(13, 100, "f16"), (5, 770, "f32"), (3, 4099, "bf16"), (7, 1001, "f16")])
def test_ragged_bias_residual_layernorm_two_outputs(rows, n, dtype):
    # magnitudes kept below 4 so that one bf16 rounding step of the stored sum stays inside the absolute bar
    x = wl.random_tensor((rows, n), dtype, 711, scale=0.4)
    res = wl.random_tensor((rows, n), dtype, 712, scale=0.4)
    bias = wl.random_tensor((n,), dtype, 713, scale=0.4)
    gamma = wl.random_tensor((n,), dtype, 714, dist="positive", scale=0.6)
    beta = wl.random_tensor((n,), dtype, 715, scale=0.3)
    spec = wl.ChainSpec(inputs=[(dtype, (rows, n)), (dtype, (rows, n)), (dtype, (n,)), (dtype, (n,)), (dtype, (n,))])
    h = spec.op("add", 0, 1)
    h = spec.op("add", h, 2)
    y = spec.op("layernorm", h, 3, 4, f=[1e-5])
    y = spec.op("gelu_erf", y)
    spec.out(y, dtype)
    spec.out(h, dtype)
    check_chain(spec, [x, res, bias, gamma, beta], what=f"ragged layernorm n={n} {dtype}")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ragged_rmsnorm(dtype):
    rows, n = 9, 1001
    x = wl.random_tensor((rows, n), dtype, 721)
    gamma = wl.random_tensor((n,), dtype, 722, dist="positive", scale=0.8)   # |output| < 4: bf16 steps inside the bar
    spec = wl.ChainSpec(inputs=[(dtype, (rows, n)), (dtype, (n,))])
    spec.out(spec.op("rmsnorm", 0, 1, f=[1e-6]), dtype)
    check_chain(spec, [x, gamma], what="ragged rmsnorm")


@pytest.mark.parametrize("op", ["reduce_sum", "reduce_max", "reduce_mean"])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_ragged_reduce_keepdim(op, dtype):
    shape = (5, 7, 45)
    x = wl.random_tensor(shape, dtype, 731, scale=0.25)
    spec = wl.ChainSpec(inputs=[(dtype, shape)])
    v = spec.op("relu", 0)
    v = spec.op(op, v)
    spec.out(spec.op("scale", v, f=[0.5]), dtype)
    check_chain(spec, [x], what=f"ragged {op}")


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_ragged_elementwise_chain_with_broadcasts(dtype):
    shape = (3, 5, 7, 30)
    x = wl.random_tensor(shape, dtype, 741)
    y = wl.random_tensor(shape, dtype, 742, dist="positive", scale=4.0)
    bias = wl.random_tensor((30,), dtype, 743)
    plane = wl.random_tensor((7, 30), dtype, 744)
    spec = wl.ChainSpec(inputs=[(dtype, shape), (dtype, shape), (dtype, (30,)), (dtype, (7, 30))])
    v = spec.op("add", 0, 2)
    v = spec.op("div", v, 1)
    v = spec.op("sub", 3, v)
    v = spec.op("silu", v)
    v = spec.op("max", v, 2)
    spec.out(v, dtype)
    spec.out(spec.op("relu", 0), dtype)
    _, info, _ = check_chain(spec, [x, y, bias, plane], what="ragged elementwise chain")
    assert info.family == _pf().PF_FAMILY_ELEMENTWISE


def test_ragged_single_odd_row():
    # 16-bit rows of odd length: every second row starts on a 2-byte boundary only
    x = wl.random_tensor((6, 33), "f16", 751)
    spec = wl.ChainSpec(inputs=[("f16", (6, 33))])
    spec.out(spec.op("tanh", 0), "f16")
    check_chain(spec, [x], what="odd rows, element-wise")
    spec = wl.ChainSpec(inputs=[("f16", (6, 33))])
    spec.out(spec.op("softmax", 0), "f16")
    check_chain(spec, [x], what="odd rows, softmax")


# ---- transposes of extents that are not whole 16-byte vectors

@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("shape,perm", [((3, 197, 64), (0, 2, 1)), ((2, 12, 197, 197), (0, 1, 3, 2)), ((100, 50), (1, 0)),
                                        ((5, 7, 9, 11), (3, 1, 0, 2)), ((2, 67, 3, 70), (3, 2, 1, 0)), ((1, 3, 13), (2, 0, 1))])
def test_ragged_innermost_changing_permute_bit_exact(shape, perm, dtype):
    from oracle import pf_oracle as orc
    from paper_2307_04995_amd import binding as pf
    x = wl.random_tensor(shape, dtype, 2101, dist="uniform")
    s = wl.ChainSpec(inputs=[(dtype, shape)])
    s.out(s.op("permute", 0, i=list(perm)), dtype)
    for generic in (False, True):
        outs, info = gpu_run(s, [x], generic=generic)
        (want,) = orc.evaluate_layout_bits(s, [wl.raw_bits(x)])
        assert np.array_equal(wl.raw_bits(outs[0]), want), f"{shape} {perm} {dtype} generic={generic}"
        assert info.family == pf.PF_FAMILY_TRANSPOSE


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("shape,perm", [((4, 12, 197), (1, 0, 2)), ((2, 5, 3, 50), (2, 0, 1, 3)), ((3, 7, 1000), (1, 0, 2))])
def test_ragged_permute_that_keeps_the_innermost_dimension(shape, perm, dtype):
    from oracle import pf_oracle as orc
    from paper_2307_04995_amd import binding as pf
    x = wl.random_tensor(shape, dtype, 2111, dist="uniform")
    s = wl.ChainSpec(inputs=[(dtype, shape)])
    s.out(s.op("permute", 0, i=list(perm)), dtype)
    for generic in (False, True):
        outs, info = gpu_run(s, [x], generic=generic)
        (want,) = orc.evaluate_layout_bits(s, [wl.raw_bits(x)])
        assert np.array_equal(wl.raw_bits(outs[0]), want), f"{shape} {perm} {dtype} generic={generic}"
        assert info.variant == pf.PF_VARIANT_T_ROWS


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ragged_transpose_fused_with_elementwise(dtype):
    # (K [B, 197, 72] + bias [72]) * 0.125 -> [B, 72, 197]: ragged output rows; and element-wise work on the output side
    b, sq, d = 3, 197, 72
    k = wl.random_tensor((b, sq, d), dtype, 2121, dist="uniform")
    bias = wl.random_tensor((d,), dtype, 2122, dist="uniform")
    s = wl.ChainSpec(inputs=[(dtype, (b, sq, d)), (dtype, (d,))])
    s.out(s.op("permute", s.op("scale", s.op("add", 0, 1), f=[0.125]), i=[0, 2, 1]), dtype)
    check_chain(s, [k, bias], what=f"ragged bias + scale + transpose {dtype}")
    col = wl.random_tensor((sq,), dtype, 2123, dist="uniform")
    s = wl.ChainSpec(inputs=[(dtype, (b, sq, d)), (dtype, (sq,))])
    s.out(s.op("add", s.op("permute", 0, i=[0, 2, 1]), 1), dtype)
    check_chain(s, [k, col], what=f"ragged transpose + bias on the output side {dtype}")
    # a kept ragged innermost dimension with a bias along it
    x = wl.random_tensor((4, 6, 197), dtype, 2124, dist="uniform")
    bias = wl.random_tensor((197,), dtype, 2125, dist="uniform")
    s = wl.ChainSpec(inputs=[(dtype, (4, 6, 197)), (dtype, (197,))])
    s.out(s.op("permute", s.op("add", 0, 1), i=[1, 0, 2]), dtype)
    check_chain(s, [x, bias], what=f"ragged rows moved with a bias {dtype}")


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("shape,perm", [((17, 1, 256), (0, 2, 1)), ((1, 5, 40), (1, 2, 0)), ((3, 1, 1, 24), (1, 0, 2, 3)), ((6, 1, 33), (1, 0, 2))])
def test_a_permutation_that_only_moves_extents_of_1_is_a_reshape(shape, perm, dtype):
    # the order of the elements does not change: no transpose kernel, element-wise work on both sides in one launch
    from paper_2307_04995_amd import binding as pf
    out_shape = tuple(shape[p] for p in perm)
    keeps = [p for p in perm if shape[p] != 1]
    if keeps != sorted(keeps):
        pytest.skip("moves data")
    x = wl.random_tensor(shape, dtype, 6101)
    b = wl.random_tensor((shape[-1],), dtype, 6102, scale=0.3)
    s = wl.ChainSpec(inputs=[(dtype, shape), (dtype, (shape[-1],))])
    v = s.op("permute", s.op("silu", s.op("add", 0, 1)), i=list(perm))
    s.out(s.op("scale", v, f=[0.5]), dtype)
    outs, info, _ = check_chain(s, [x, b], what=f"{shape} perm {perm} {dtype}")
    assert info.family == pf.PF_FAMILY_ELEMENTWISE and tuple(outs[0].shape) == out_shape


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("shape,perm", [((3, 40, 7, 7), (0, 2, 3, 1)), ((3, 7, 7, 40), (0, 3, 1, 2)), ((2, 24, 14, 14), (0, 2, 3, 1)),
                                        ((2, 5, 3, 9, 16), (0, 4, 1, 2, 3)), ((2, 17, 3, 5), (0, 2, 3, 1))])
def test_channels_first_to_channels_last_with_few_positions(shape, perm, dtype):
    # h and w stay adjacent and in order: they transpose as one extent of h * w (49, 196) although that is not a whole
    # number of vectors; nothing in the chain looks at positions (no broadcast operand, no mask)
    from paper_2307_04995_amd import binding as pf
    x = wl.random_tensor(shape, dtype, 6201)
    s = wl.ChainSpec(inputs=[(dtype, shape)])
    s.out(s.op("scale", s.op("permute", s.op("silu", 0) if dtype == "f32" else 0, i=list(perm)), f=[0.5]), dtype)
    outs, info, _ = check_chain(s, [x], what=f"{shape} perm {perm} {dtype}")
    assert info.family == pf.PF_FAMILY_TRANSPOSE and info.variant == pf.PF_VARIANT_T_TILE
    # with a broadcast operand the extents stay apart (its vectors are told from the innermost extent)
    b = wl.random_tensor((shape[perm[-1]],), dtype, 6202, scale=0.3)
    s = wl.ChainSpec(inputs=[(dtype, shape), (dtype, (shape[perm[-1]],))])
    s.out(s.op("add", s.op("permute", 0, i=list(perm)), 1), dtype)
    check_chain(s, [x, b], what=f"{shape} perm {perm} {dtype} + bias")
