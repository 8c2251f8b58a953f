"""GPU parity for operands that broadcast the numpy way, with extents of 1 anywhere (an attention mask
[B, 1, 1, S] under scores [B, H, S, S], a per-sample bias [N, 1, 1, C] on a feature map, one value per row
[..., 1] as an input): through the C ABI, element by element against the fp64 oracle."""
import numpy as np
import pytest

import workloads as wl
from pf_testlib import check_chain

pytestmark = pytest.mark.gpu


def _pf():
    from paper_2307_04995_amd import binding as pf
    return pf


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("mask_shape", [(2, 1, 1, 72), (2, 1, 40, 72), (1, 3, 1, 72), (3, 1, 1), (2, 1, 40, 1), (2, 3, 1, 1)])
def test_softmax_with_a_broadcast_mask(mask_shape, dtype):
    B, H, Sq, S = 2, 3, 40, 72
    x = wl.random_tensor((B, H, Sq, S), dtype, 2001, scale=2.0)
    m = wl.random_tensor(mask_shape, dtype, 2002, scale=3.0)
    s = wl.ChainSpec(inputs=[(dtype, (B, H, Sq, S)), (dtype, mask_shape)])
    s.out(s.op("softmax", s.op("add", s.op("scale", 0, f=[0.125]), 1)), dtype)
    _, info, _ = check_chain(s, [x, m], what=f"softmax with mask {mask_shape} {dtype}")
    assert info.family == _pf().PF_FAMILY_ROW and info.n_launches == 1


def test_ragged_rows_with_a_padding_mask():
    # 197 tokens: the rows are not whole vectors, the mask is gathered element by element
    B, H, S = 2, 4, 197
    x = wl.random_tensor((B, H, S, S), "f16", 2011, scale=2.0)
    m = wl.random_tensor((B, 1, 1, S), "f16", 2012, scale=3.0)
    s = wl.ChainSpec(inputs=[("f16", (B, H, S, S)), ("f16", (B, 1, 1, S))])
    s.out(s.op("softmax", s.op("add", 0, 1)), "f16")
    check_chain(s, [x, m], what="ragged softmax with a padding mask")


@pytest.mark.parametrize("dtype,c", [("f16", 64), ("f32", 36), ("bf16", 36)])
def test_per_sample_bias_on_a_feature_map(dtype, c):
    # x [N, H, W, C] + t [N, 1, 1, C] -> SiLU: element-wise family (36 channels: ragged)
    n, h, w = 3, 9, 11
    x = wl.random_tensor((n, h, w, c), dtype, 2021)
    t = wl.random_tensor((n, 1, 1, c), dtype, 2022)
    s = wl.ChainSpec(inputs=[(dtype, (n, h, w, c)), (dtype, (n, 1, 1, c))])
    s.out(s.op("silu", s.op("add", 0, 1)), dtype)
    _, info, _ = check_chain(s, [x, t], what=f"per-sample bias {dtype} c={c}")
    assert info.family == _pf().PF_FAMILY_ELEMENTWISE


def test_per_sample_bias_in_front_of_groupnorm():
    # the time-embedding add of a diffusion residual block, fused into the normalisation that follows it
    pf = _pf()
    n, h, w, c, g = 3, 12, 12, 320, 32
    x = wl.random_tensor((n, h, w, c), "f16", 2031)
    t = wl.random_tensor((n, 1, 1, c), "f16", 2032)
    gamma = wl.random_tensor((c,), "f16", 2033, dist="positive", scale=0.8)
    beta = wl.random_tensor((c,), "f16", 2034, scale=0.3)
    s = wl.ChainSpec(inputs=[("f16", (n, h, w, c)), ("f16", (n, 1, 1, c)), ("f16", (c,)), ("f16", (c,))])
    s.out(s.op("silu", s.op("groupnorm", s.op("add", 0, 1), 2, 3, f=[1e-5], i=[g])), "f16")
    _, info, _ = check_chain(s, [x, t, gamma, beta], what="bias + GroupNorm + SiLU")
    assert info.family == pf.PF_FAMILY_GROUP and info.variant == pf.PF_VARIANT_GROUP_TWO_PASS


def test_one_value_per_row_as_an_input_and_three_runs_of_kept_dimensions():
    # LayerNorm of x * keep[..., 1] (a per-token factor), then a rank-6 operand with three separate kept runs
    x = wl.random_tensor((4, 25, 96), "f32", 2041)
    keep = wl.random_tensor((4, 25, 1), "f32", 2042, dist="positive")
    gamma = wl.random_tensor((96,), "f32", 2043, dist="positive")
    beta = wl.random_tensor((96,), "f32", 2044)
    s = wl.ChainSpec(inputs=[("f32", (4, 25, 96)), ("f32", (4, 25, 1)), ("f32", (96,)), ("f32", (96,))])
    s.out(s.op("layernorm", s.op("mul", 0, 1), 2, 3, f=[1e-5]), "f32")
    check_chain(s, [x, keep, gamma, beta], what="per-token factor in front of LayerNorm")

    full, part = (2, 3, 4, 5, 6, 8), (2, 1, 4, 1, 6, 8)
    a = wl.random_tensor(full, "f32", 2045)
    b = wl.random_tensor(part, "f32", 2046)
    s = wl.ChainSpec(inputs=[("f32", full), ("f32", part)])
    s.out(s.op("sub", 1, 0), "f32")
    check_chain(s, [a, b], what="three runs of kept dimensions")


def test_bias_broadcast_over_the_sequence_in_front_of_a_permutation():
    # (Q [B, S, H, D] + b [B, 1, H, D]) -> [B, H, S, D]
    B, S, H, D = 2, 24, 4, 64
    q = wl.random_tensor((B, S, H, D), "bf16", 2051)
    b = wl.random_tensor((B, 1, H, D), "bf16", 2052)
    s = wl.ChainSpec(inputs=[("bf16", (B, S, H, D)), ("bf16", (B, 1, H, D))])
    s.out(s.op("permute", s.op("add", 0, 1), i=[0, 2, 1, 3]), "bf16")
    _, info, _ = check_chain(s, [q, b], what="broadcast bias + permute")
    assert info.family == _pf().PF_FAMILY_TRANSPOSE


def test_shapes_that_do_not_broadcast_are_refused():
    pf = _pf()
    s = wl.ChainSpec(inputs=[("f32", (2, 3, 8, 8)), ("f32", (2, 2, 1, 8))])
    s.out(s.op("add", 0, 1), "f32")
    assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_ERR_SHAPE


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("small", [(6, 1), (1, 200), (200,), (1, 1)])
def test_a_value_computed_from_broadcast_inputs_alone(small, dtype):
    # x / (m + 1), x * sigmoid(g) * (a + b): the small operands are transformed before they meet the full-size value;
    # they are addressed against that value, not against their own shape
    shape = (6, 200)
    x = wl.random_tensor(shape, dtype, 5601)
    m = wl.random_tensor(small, dtype, 5602, dist="positive")
    g = wl.random_tensor(small, dtype, 5603)
    s = wl.ChainSpec(inputs=[(dtype, shape), (dtype, small)])
    s.out(s.op("div", 0, s.op("addc", 1, f=[1.0])), dtype)
    check_chain(s, [x, m], what=f"x / (m{small} + 1) {dtype}")
    s = wl.ChainSpec(inputs=[(dtype, shape), (dtype, small), (dtype, small)])
    v = s.op("mul", s.op("sigmoid", 2), s.op("add", 1, 2))
    s.out(s.op("softmax", s.op("mul", 0, v)), dtype)
    check_chain(s, [x, m, g], what=f"softmax(x * sigmoid(g) * (m + g)) {small} {dtype}")
