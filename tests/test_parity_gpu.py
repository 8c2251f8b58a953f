"""GPU parity: every kernel family, through the C ABI, element by element against the fp64 oracle on the
same seeded inputs, at sizes that span several tiles and a ragged tail."""
import numpy as np
import pytest
import torch

import workloads as wl
from pf_testlib import check_chain, compare, gpu_run, oracle_run, SPEC_JIT

pytestmark = pytest.mark.gpu


def _pf():
    from paper_2307_04995_amd import binding as pf
    return pf


# ------------------------------------------------------------------ the five benchmark chains, reduced

@pytest.mark.parametrize("generic", [False, True])
@pytest.mark.parametrize("rows,n,dtype", [(37, 768, "f32"), (5, 256, "f32"), (67, 1024, "f16"), (9, 2048, "bf16")])
def test_c1_chain(rows, n, dtype, generic):
    spec, ins = wl.c1_bias_res_layernorm_gelu(rows=rows, n=n, dtype=dtype)
    _, info, _ = check_chain(spec, ins, generic=generic, what=f"C1 {rows}x{n} {dtype}")
    assert info.family == _pf().PF_FAMILY_ROW and info.n_launches == 1
    assert (info.spec_id == 0) == generic


@pytest.mark.parametrize("generic", [False, True])
@pytest.mark.parametrize("b,h,s,dtype", [(2, 3, 64, "f16"), (1, 2, 512, "f16"), (1, 1, 136, "bf16"), (1, 2, 48, "f32")])
def test_c2_chain(b, h, s, dtype, generic):
    spec, ins = wl.c2_causal_softmax(b=b, h=h, s=s, dtype=dtype)
    outs, info, _ = check_chain(spec, ins, generic=generic, what=f"C2 {b}x{h}x{s} {dtype}")
    y = wl.widen(outs[0])
    iu = np.triu_indices(s, k=1)
    assert np.all(y[..., iu[0], iu[1]] == 0.0), "masked positions must be exactly zero"
    assert info.family == _pf().PF_FAMILY_ROW


def test_causal_softmax_with_other_prologue_steps():
    # a negative factor and a bias in front of the mask: the mask moves into the core but skipped loads may
    # not stand in as -inf; a non-positive scale is not folded into the core at all
    b, h, sq = 1, 3, 96
    x = wl.random_tensor((b, h, sq, sq), "f16", 51, scale=2.0)
    bias = wl.random_tensor((sq,), "f16", 52)
    for factor in (-0.5, 0.25):
        spec = wl.ChainSpec(inputs=[("f16", (b, h, sq, sq)), ("f16", (sq,))])
        v = spec.op("add", 0, 1)
        v = spec.op("scale", v, f=[factor])
        v = spec.op("causal_mask", v)
        v = spec.op("softmax", v)
        spec.out(v, "f16")
        check_chain(spec, [x, bias], what=f"masked softmax factor {factor}")
        check_chain(spec, [x, bias], generic=True, what=f"masked softmax factor {factor} generic")
    spec = wl.ChainSpec(inputs=[("f16", (b, h, sq, sq))])
    v = spec.op("scale", 0, f=[-1.0])
    v = spec.op("causal_mask", v)
    v = spec.op("softmax", v)
    spec.out(v, "f16")
    check_chain(spec, [x], what="masked softmax negative scale")
    # mask first, then more arithmetic: stays an ordinary prologue step
    spec = wl.ChainSpec(inputs=[("f16", (b, h, sq, sq))])
    v = spec.op("causal_mask", 0)
    v = spec.op("scale", v, f=[0.5])
    v = spec.op("softmax", v)
    spec.out(v, "f16")
    check_chain(spec, [x], what="mask then scale")


def test_full_shape_operand_after_a_causal_softmax():
    # softmax(causal(x)) * keep: the epilogue reads `keep` on the masked columns too (0 * keep, but min / add of
    # it are not 0), so columns beyond the diagonal cannot be skipped for that operand
    shape = (2, 3, 16, 64)
    x = wl.random_tensor(shape, "f32", 1601, scale=2.0)
    keep = wl.random_tensor(shape, "f32", 1602)
    for name in ("min", "add", "mul"):
        s = wl.ChainSpec(inputs=[("f32", shape), ("f32", shape)])
        s.out(s.op(name, s.op("softmax", s.op("causal_mask", s.op("scale", 0, f=[0.5]))), 1), "f32")
        check_chain(s, [x, keep], what=f"causal softmax then {name} with a full-shape operand")


def test_c2_rectangular_scores():
    # more keys than queries: the mask still compares column against row of the last two dims
    spec, ins = wl.c2_causal_softmax(b=1, h=2, s=40, s_k=72, dtype="f16")
    check_chain(spec, ins, what="C2 rectangular")


@pytest.mark.parametrize("generic", [False, True])
@pytest.mark.parametrize("rows,n,dtype", [(131, 1024, "f16"), (7, 512, "f16"), (33, 1024, "bf16"), (10, 384, "f32")])
def test_c3_chain(rows, n, dtype, generic):
    spec, ins = wl.c3_bias_res_layernorm(rows=rows, n=n, dtype=dtype)
    check_chain(spec, ins, generic=generic, what=f"C3 {rows}x{n} {dtype}")


@pytest.mark.parametrize("generic", [False, True])
@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("b,s,h,d,dtype", [(2, 48, 16, 64, "bf16"), (1, 32, 4, 32, "f16"), (3, 16, 8, 16, "f32")])
def test_c4_chain(b, s, h, d, dtype, variant, generic):
    spec, ins = wl.c4_bias_scale_permute(b=b, s=s, h=h, d=d, dtype=dtype)
    outs, info, _ = check_chain(spec, ins, variant=variant, generic=generic, what=f"C4 {dtype} v{variant}")
    assert info.family == _pf().PF_FAMILY_TRANSPOSE and info.variant == variant
    # layout part, bit-exact: the same element-wise chain without the permutation, permuted on the host
    flat = wl.ChainSpec(inputs=list(spec.inputs))
    v = flat.op("add", 0, 1)
    v = flat.op("scale", v, f=[0.125])
    flat.out(v, dtype)
    (unpermuted,), _ = gpu_run(flat, ins)
    want_bits = np.transpose(wl.raw_bits(unpermuted), (0, 2, 1, 3))
    assert np.array_equal(wl.raw_bits(outs[0]), want_bits), "fused permutation is not a bit-exact re-layout"


@pytest.mark.parametrize("generic", [False, True])
@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("n,h,w,c,g,dtype", [(2, 16, 16, 512, 32, "f16"), (3, 7, 9, 64, 4, "f16"), (1, 24, 24, 256, 8, "bf16"),
                                             (2, 5, 5, 32, 2, "f32")])
def test_c5_chain(n, h, w, c, g, dtype, variant, generic):
    pf = _pf()
    spec, ins = wl.c5_groupnorm_silu(n=n, h=h, w=w, ch=c, groups=g, dtype=dtype)
    if variant == 1 and generic:
        pytest.skip("the register-resident variant exists for catalogue chains only")
    _, info, _ = check_chain(spec, ins, variant=variant, generic=generic, what=f"C5 {dtype} v{variant}")
    assert info.family == pf.PF_FAMILY_GROUP and info.variant == variant
    assert info.n_launches == (2 if variant == 0 else 1)


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("n,h,w,c,g,dtype", [
    (2, 16, 16, 320, 32, "f16"),    # 10 channels per group: a 16-byte vector straddles two groups
    (2, 8, 8, 128, 32, "f16"),      # 4 per group: two groups per vector
    (1, 12, 12, 96, 32, "bf16"),    # 3 per group: up to four groups per vector
    (2, 6, 6, 1280, 32, "f16"),     # 40 per group: five vectors, not a power of two
    (2, 9, 9, 48, 4, "f32"),        # 12 per group in fp32: three vectors
    (1, 8, 8, 64, 64, "f16"),       # one channel per group
    (2, 5, 7, 24, 1, "f16"),        # one group over the whole sample
    (3, 40, 40, 320, 32, "f16"),    # several workgroups per sample
])
def test_groupnorm_groups_of_any_width(n, h, w, c, g, dtype, variant):
    pf = _pf()
    spec, ins = wl.c5_groupnorm_silu(n=n, h=h, w=w, ch=c, groups=g, dtype=dtype, salt=7)
    _, info, _ = check_chain(spec, ins, variant=variant, what=f"GroupNorm {c} channels / {g} groups {dtype} v{variant}")
    assert info.family == pf.PF_FAMILY_GROUP and info.variant == variant
    assert info.n_launches == (2 if variant == 0 else 1)


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("n,h,w,c,g,dtype", [
    (2, 6, 6, 12, 3, "f16"),        # 24 bytes per position: one whole vector and one of four channels
    (2, 9, 7, 100, 4, "f16"),       # 25 channels per group, last vector of four
    (3, 5, 5, 6, 2, "f32"),         # fp32, 24 bytes per position
    (1, 20, 20, 36, 36, "bf16"),    # one channel per group
    (2, 33, 33, 50, 1, "f16"),      # one group, several workgroups per sample
    (2, 4, 4, 3, 1, "f16"),         # fewer channels than one vector
])
def test_groupnorm_channel_counts_that_are_not_whole_vectors(n, h, w, c, g, dtype, variant):
    pf = _pf()
    spec, ins = wl.c5_groupnorm_silu(n=n, h=h, w=w, ch=c, groups=g, dtype=dtype, salt=13)
    _, info, _ = check_chain(spec, ins, variant=variant, what=f"GroupNorm {c} channels (ragged) / {g} groups {dtype} v{variant}")
    assert info.family == pf.PF_FAMILY_GROUP and info.variant == variant
    assert info.n_launches == (2 if variant == 0 else 1)


@pytest.mark.parametrize("c,g,dtype", [(12, 3, "f16"), (6, 2, "f32"), (100, 4, "bf16")])
def test_groupnorm_ragged_channels_on_the_interpreted_kernels(c, g, dtype):
    spec, ins = wl.c5_groupnorm_silu(n=2, h=9, w=7, ch=c, groups=g, dtype=dtype, salt=14)
    _, info, _ = check_chain(spec, ins, variant=0, generic=True, what=f"GroupNorm {c} channels (ragged), interpreted")
    assert info.spec_id == 0 and info.n_launches == 2


def test_groupnorm_with_residual_on_a_ragged_channel_count():
    # a second full-shape operand and a per-sample operand in front of the normalisation, 20 bytes per position
    c = 10
    shape = (3, 7, 5, c)
    x, res = wl.random_tensor(shape, "f16", 1901), wl.random_tensor(shape, "f16", 1902)
    gamma, beta = wl.random_tensor((c,), "f16", 1903, dist="positive"), wl.random_tensor((c,), "f16", 1904, scale=0.3)
    s = wl.ChainSpec(inputs=[("f16", shape), ("f16", shape), ("f16", (c,)), ("f16", (c,))])
    s.out(s.op("relu", s.op("groupnorm", s.op("add", 0, 1), 2, 3, f=[1e-5], i=[2])), "f16")
    check_chain(s, [x, res, gamma, beta], what="GroupNorm(x + res) on 10 channels")


def test_groupnorm_of_single_element_groups_returns_beta_exactly():
    # one position, one channel per group: every deviation is exactly zero, the result is beta (1 / sqrt(eps) would
    # amplify a one-ulp error of the mean to 3e-5)
    c = 148
    x = wl.random_tensor((1, 1, c), "f32", 1801, scale=2.0)
    gamma = wl.random_tensor((c,), "f32", 1802, dist="positive")
    beta = wl.random_tensor((c,), "f32", 1803)
    s = wl.ChainSpec(inputs=[("f32", (1, 1, c)), ("f32", (c,)), ("f32", (c,))])
    s.out(s.op("groupnorm", 0, 1, 2, f=[1e-5], i=[c]), "f32")
    for variant in (0, 1):
        outs, _, _ = check_chain(s, [x, gamma, beta], variant=variant, what=f"single-element groups, variant {variant}")
        assert torch.equal(outs[0].reshape(-1), beta)


@pytest.mark.parametrize("c,g", [(64, 8), (320, 32)])
def test_groupnorm_with_residuals_on_both_sides(c, g):
    # GroupNorm(x + res) + skip: two full-shape operands in front, one behind (two-launch variant: the fused one
    # keeps a single operand in registers)
    pf = _pf()
    shape = (2, 9, 7, c)
    x, res, skip = (wl.random_tensor(shape, "f16", 1701 + k) for k in range(3))
    gamma = wl.random_tensor((c,), "f16", 1704, dist="positive")
    beta = wl.random_tensor((c,), "f16", 1705, scale=0.3)
    s = wl.ChainSpec(inputs=[("f16", shape), ("f16", shape), ("f16", (c,)), ("f16", (c,)), ("f16", shape)])
    v = s.op("groupnorm", s.op("add", 0, 1), 2, 3, f=[1e-5], i=[g])
    s.out(s.op("add", s.op("silu", v), 4), "f16")
    _, info, _ = check_chain(s, [x, res, gamma, beta, skip], what=f"GroupNorm with residuals, {c} channels")
    assert info.family == pf.PF_FAMILY_GROUP and info.variant == pf.PF_VARIANT_GROUP_TWO_PASS
    # a single position per sample: the per-sample operand has the full shape
    shape = (4, 1, 232)
    x, t = wl.random_tensor(shape, "f16", 1711), wl.random_tensor(shape, "f16", 1712)
    gamma, beta = wl.random_tensor((232,), "f16", 1713, dist="positive"), wl.random_tensor((232,), "f16", 1714)
    s = wl.ChainSpec(inputs=[("f16", shape), ("f16", (232,)), ("f16", (232,)), ("f16", shape)])
    s.out(s.op("groupnorm", s.op("add", 0, 3), 1, 2, f=[1e-5], i=[29]), "f16")
    check_chain(s, [x, gamma, beta, t], what="GroupNorm of single positions with a second full-shape operand")


@pytest.mark.parametrize("variant", [0, 1])
def test_groupnorm_general_path_matches_the_aligned_one(variant):
    # the same chain through both statistics paths (the general one forced on a shape that does not need it)
    from pf_testlib import env
    spec, ins = wl.c5_groupnorm_silu(n=2, h=24, w=24, ch=512, groups=32, dtype="f16", salt=8)
    fast, _ = gpu_run(spec, ins, variant=variant)
    with env(PF_GROUP_GENERAL="1"):
        outs, info, _ = check_chain(spec, ins, variant=variant, what="general statistics path on an aligned shape")
    assert info.spec_id == SPEC_JIT
    diff = np.abs(wl.widen(outs[0]) - wl.widen(fast[0]))
    assert diff.max() <= 4e-3


@pytest.mark.parametrize("dtype,n", [("f16", 1024), ("f32", 200), ("bf16", 64)])
def test_normalisation_of_a_single_row(dtype, n):
    # one token: gamma and beta have as many elements as the value itself, and are parameters all the same
    x = wl.random_tensor((1, n), dtype, 1501)
    gamma = wl.random_tensor((n,), dtype, 1502, dist="positive")
    beta = wl.random_tensor((n,), dtype, 1503, scale=0.3)
    s = wl.ChainSpec(inputs=[(dtype, (1, n)), (dtype, (n,)), (dtype, (n,))])
    s.out(s.op("gelu_erf", s.op("layernorm", 0, 1, 2, f=[1e-5])), dtype)
    check_chain(s, [x, gamma, beta], what=f"LayerNorm of one row {dtype}")
    s = wl.ChainSpec(inputs=[(dtype, (1, 1, n)), (dtype, (n,))])
    s.out(s.op("rmsnorm", 0, 1, f=[1e-6]), dtype)
    check_chain(s, [x.reshape(1, 1, n), gamma], what=f"RMSNorm of one row {dtype}")


# ------------------------------------------------------------------ layout-only chains, bit-exact

@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("shape,perm", [((2, 24, 16, 64), (0, 2, 1, 3)), ((6, 5, 32), (1, 0, 2)), ((2, 3, 4, 5, 16), (3, 0, 2, 1, 4)),
                                        ((4, 8, 8), (0, 1, 2)),
                                        # two swapped dimensions around a short kept run: walked in blocks (4 x 4, 2 x 4, 8 x 2, none)
                                        ((3, 12, 6, 64), (0, 2, 1, 3)), ((40, 24, 8), (1, 0, 2)), ((2, 7, 9, 32), (0, 2, 1, 3))])
def test_permute_only_bit_exact(shape, perm, dtype):
    from oracle import pf_oracle as orc
    g = np.random.default_rng(99)
    nbits = 32 if dtype == "f32" else 16
    bits = g.integers(0, 1 << nbits, size=shape, dtype=np.uint32 if nbits == 32 else np.uint16)
    view = {"f32": torch.int32, "f16": torch.int16, "bf16": torch.int16}[dtype]
    t = torch.from_numpy(bits.view(np.int32 if nbits == 32 else np.int16)).view(wl.DTYPES[dtype])
    spec = wl.ChainSpec(inputs=[(dtype, shape)])
    spec.out(spec.op("permute", 0, i=perm), dtype)
    for variant in (None,):
        (out,), info = gpu_run(spec, [t], variant=variant)
        (want,) = orc.evaluate_layout_bits(spec, [bits])
        assert np.array_equal(wl.raw_bits(out), want)


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("shape,perm", [((3, 64, 128), (0, 2, 1)), ((72, 40), (1, 0)), ((2, 24, 3, 16), (0, 3, 2, 1)),
                                        ((2, 8, 136, 200), (1, 3, 0, 2)), ((5, 8, 8, 16), (3, 1, 0, 2))])
def test_innermost_changing_permute_bit_exact(shape, perm, dtype):
    from oracle import pf_oracle as orc
    g = np.random.default_rng(101)
    nbits = 32 if dtype == "f32" else 16
    bits = g.integers(0, 1 << nbits, size=shape, dtype=np.uint32 if nbits == 32 else np.uint16)
    t = torch.from_numpy(bits.view(np.int32 if nbits == 32 else np.int16)).view(wl.DTYPES[dtype])
    spec = wl.ChainSpec(inputs=[(dtype, shape)])
    spec.out(spec.op("permute", 0, i=perm), dtype)
    (out,), info = gpu_run(spec, [t])
    assert info.variant == _pf().PF_VARIANT_T_TILE
    (want,) = orc.evaluate_layout_bits(spec, [bits])
    assert np.array_equal(wl.raw_bits(out), want)


@pytest.mark.parametrize("generic", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_transpose_fused_with_elementwise(dtype, generic):
    # K^T-style chain: (x + bias) * scale computed on the input layout, then [b, s, d] -> [b, d, s]
    b, sq, d = 3, 200, 64
    x = wl.random_tensor((b, sq, d), dtype, 61)
    bias = wl.random_tensor((d,), dtype, 62)
    spec = wl.ChainSpec(inputs=[(dtype, (b, sq, d)), (dtype, (d,))])
    v = spec.op("add", 0, 1)
    v = spec.op("scale", v, f=[0.125])
    v = spec.op("permute", v, i=[0, 2, 1])
    spec.out(v, dtype)
    outs, info, _ = check_chain(spec, [x, bias], generic=generic, what="fused transpose, prologue side")
    assert info.variant == _pf().PF_VARIANT_T_TILE
    # compute on the output layout instead: permute first, then an operand shaped like the output rows
    col = wl.random_tensor((sq,), dtype, 63, scale=0.5)     # keeps |result| small: the 16-bit bars are absolute
    spec2 = wl.ChainSpec(inputs=[(dtype, (b, sq, d)), (dtype, (sq,))])
    v = spec2.op("permute", 0, i=[0, 2, 1])
    v = spec2.op("mul", v, 1)
    v = spec2.op("gelu_erf", v)
    spec2.out(v, dtype)
    check_chain(spec2, [x, col], generic=generic, what="fused transpose, epilogue side")


def test_transpose_fp32_computes_on_both_sides():
    b, sq, d = 2, 72, 40
    x = wl.random_tensor((b, sq, d), "f32", 64)
    bias = wl.random_tensor((d,), "f32", 65)
    col = wl.random_tensor((sq,), "f32", 66)
    spec = wl.ChainSpec(inputs=[("f32", (b, sq, d)), ("f32", (d,)), ("f32", (sq,))])
    v = spec.op("add", 0, 1)
    v = spec.op("permute", v, i=[0, 2, 1])
    v = spec.op("mul", v, 2)
    spec.out(v, "f32")
    check_chain(spec, [x, bias, col], what="fp32 transpose, both sides")


# ------------------------------------------------------------------ other cores and the element-wise family

@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_rmsnorm_and_residual(dtype):
    rows, n = 45, 640
    x = wl.random_tensor((rows, n), dtype, 1)
    res = wl.random_tensor((rows, n), dtype, 2)
    gamma = wl.random_tensor((n,), dtype, 3)
    spec = wl.ChainSpec(inputs=[(dtype, (rows, n)), (dtype, (rows, n)), (dtype, (n,))])
    v = spec.op("add", 0, 1)
    v = spec.op("rmsnorm", v, 2, f=[1e-6])
    spec.out(v, dtype)
    check_chain(spec, [x, res, gamma], what="rmsnorm")
    check_chain(spec, [x, res, gamma], generic=True, what="rmsnorm generic")


@pytest.mark.parametrize("n", [8, 200, 1024, 4096, 12288])
def test_softmax_row_lengths(n):
    rows = 11
    x = wl.random_tensor((rows, n), "f16", n, scale=3.0)
    spec = wl.ChainSpec(inputs=[("f16", (rows, n))])
    spec.out(spec.op("softmax", 0), "f16")
    _, info, _ = check_chain(spec, [x], what=f"softmax n={n}")
    y, _ = gpu_run(spec, [x])
    np.testing.assert_allclose(wl.widen(y[0]).sum(-1), 1.0, atol=4e-3)


@pytest.mark.parametrize("variant", [0, 1])
def test_layernorm_wave_and_block_variants_agree_with_oracle(variant):
    rows, n = 19, 1024
    spec, ins = wl.c3_bias_res_layernorm(rows=rows, n=n, dtype="f16", salt=3)
    _, info, _ = check_chain(spec, ins, variant=variant, what=f"LN variant {variant}")
    assert info.variant == variant


@pytest.mark.parametrize("op", ["reduce_sum", "reduce_max", "reduce_mean"])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_reduce_keepdim(op, dtype):
    rows, n = 23, 520
    x = wl.random_tensor((rows, n), dtype, 5, scale=0.5)
    spec = wl.ChainSpec(inputs=[(dtype, (rows, n))])
    v = spec.op("scale", 0, f=[0.5])
    v = spec.op(op, v)
    v = spec.op("addc", v, f=[1.0])
    spec.out(v, dtype)
    outs, info, _ = check_chain(spec, [x], what=op)
    assert tuple(outs[0].shape) == (rows, 1)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_elementwise_chain_with_broadcasts(dtype):
    shape = (3, 5, 7, 64)
    x = wl.random_tensor(shape, dtype, 11)
    y = wl.random_tensor(shape, dtype, 12, dist="positive", scale=4.0)     # in [1, 4]: keeps |result| small
    bias = wl.random_tensor((64,), dtype, 13)
    plane = wl.random_tensor((7, 64), dtype, 14)
    spec = wl.ChainSpec(inputs=[(dtype, shape), (dtype, shape), (dtype, (64,)), (dtype, (7, 64))])
    v = spec.op("add", 0, 2)          # + bias[64]
    v = spec.op("div", v, 1)          # / y
    v = spec.op("sub", 3, v)          # plane[7,64] - v   (broadcast operand on the left)
    v = spec.op("gelu_erf", v)
    v = spec.op("max", v, 2)
    spec.out(v, dtype)
    _, info, _ = check_chain(spec, [x, y, bias, plane], what="elementwise chain")
    assert info.family == _pf().PF_FAMILY_ELEMENTWISE


@pytest.mark.parametrize("name", ["relu", "sigmoid", "silu", "gelu_erf", "tanh", "exp", "neg"])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_unary_ops(name, dtype):
    # magnitudes stay O(1): the parity bars are absolute
    x = wl.random_tensor((6, 1000 if dtype == "f32" else 1024), dtype, 21, scale=0.5 if name == "exp" else 2.0)
    spec = wl.ChainSpec(inputs=[(dtype, tuple(x.shape))])
    spec.out(spec.op(name, 0), dtype)
    check_chain(spec, [x], what=name)


def test_rsqrt_and_min():
    x = wl.random_tensor((4, 256), "f32", 22, dist="positive", scale=4.0)
    spec = wl.ChainSpec(inputs=[("f32", (4, 256))])
    v = spec.op("rsqrt", 0)
    v = spec.op("min", v, 0)
    spec.out(v, "f32")
    check_chain(spec, [x], what="rsqrt/min")


def test_silu_composite_equals_decomposition():
    # SiLU given as one op and as sigmoid followed by multiply (needs a temporary) must agree
    x = wl.random_tensor((9, 512), "f32", 23, scale=3.0)
    a = wl.ChainSpec(inputs=[("f32", (9, 512))])
    a.out(a.op("silu", 0), "f32")
    b = wl.ChainSpec(inputs=[("f32", (9, 512))])
    s = b.op("sigmoid", 0)
    b.out(b.op("mul", 0, s), "f32")
    (ya,), _ = gpu_run(a, [x])
    (yb,), _ = gpu_run(b, [x])
    np.testing.assert_allclose(ya.numpy(), yb.numpy(), rtol=0, atol=1e-6)
    check_chain(b, [x], what="decomposed silu")


def test_dag_chain_with_temporaries():
    # y = (x*x + x) * tanh(x) -> LayerNorm: values reused out of order force SAVE / TMP steps
    rows, n = 13, 256
    x = wl.random_tensor((rows, n), "f32", 24)
    gamma = wl.random_tensor((n,), "f32", 25)
    beta = wl.random_tensor((n,), "f32", 26)
    spec = wl.ChainSpec(inputs=[("f32", (rows, n)), ("f32", (n,)), ("f32", (n,))])
    sq = spec.op("mul", 0, 0)
    s = spec.op("add", sq, 0)
    t = spec.op("tanh", 0)
    v = spec.op("mul", s, t)
    v = spec.op("layernorm", v, 1, 2, f=[1e-5])
    spec.out(v, "f32")
    check_chain(spec, [x, gamma, beta], what="dag chain")


def test_two_outputs_residual_stream():
    rows, n = 21, 1024
    x = wl.random_tensor((rows, n), "f16", 31)
    res = wl.random_tensor((rows, n), "f16", 32)
    gamma = wl.random_tensor((n,), "f16", 33)
    beta = wl.random_tensor((n,), "f16", 34)
    spec = wl.ChainSpec(inputs=[("f16", (rows, n)), ("f16", (rows, n)), ("f16", (n,)), ("f16", (n,))])
    h = spec.op("add", 0, 1)
    y = spec.op("layernorm", h, 2, 3, f=[1e-5])
    spec.out(y, "f16")
    spec.out(h, "f16")
    check_chain(spec, [x, res, gamma, beta], what="two outputs")


def test_reshape_is_free():
    x = wl.random_tensor((4, 6, 128), "f16", 41)
    spec = wl.ChainSpec(inputs=[("f16", (4, 6, 128))])
    v = spec.op("reshape", 0, i=[24, 128])
    v = spec.op("softmax", v)
    v = spec.op("reshape", v, i=[4, 6, 128])
    spec.out(v, "f16")
    outs, _, _ = check_chain(spec, [x], what="reshape")
    assert tuple(outs[0].shape) == (4, 6, 128)


def test_in_place_row_chain():
    pf = _pf()
    spec, ins = wl.c3_bias_res_layernorm(rows=40, n=1024, dtype="f16", salt=5)
    dev = [t.cuda() for t in ins]
    want = oracle_run(spec, ins)[0]
    plan = pf.Plan(spec, 0)
    plan.run(dev, [dev[0]])          # output aliases x exactly
    torch.cuda.synchronize()
    compare(dev[0].cpu(), want, "f16", "in place")
    plan.close()


def test_run_rejects_bad_pointers():
    pf = _pf()
    spec, ins = wl.c4_bias_scale_permute(b=1, s=16, h=4, d=32)
    dev = [t.cuda() for t in ins]
    out = torch.empty((1, 4, 16, 32), dtype=torch.bfloat16, device="cuda")
    plan = pf.Plan(spec, 0)
    st = pf.pf_chain_run(plan.handle, [dev[0].data_ptr() + 2, dev[1].data_ptr()], [out.data_ptr()], 0)
    assert st == pf.PF_ERR_ALIGNMENT
    st = pf.pf_chain_run(plan.handle, [dev[0].data_ptr(), dev[1].data_ptr()], [dev[0].data_ptr()], 0)
    assert st == pf.PF_ERR_ALIAS                      # the transpose family cannot run in place
    st = pf.pf_chain_run(plan.handle, [0, dev[1].data_ptr()], [out.data_ptr()], 0)
    assert st == pf.PF_ERR_INVALID_ARG
    plan.close()


def test_non_default_stream_and_repeated_runs():
    pf = _pf()
    spec, ins = wl.c5_groupnorm_silu(n=2, h=16, w=16, ch=512, groups=32, dtype="f16", salt=2)
    dev = [t.cuda() for t in ins]
    want = oracle_run(spec, ins)[0]
    plan = pf.Plan(spec, 0)
    out = torch.empty_like(dev[0])
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for _ in range(5):           # the resident variant's arrival counters must survive re-launches
            plan.run(dev, [out], stream.cuda_stream)
    stream.synchronize()
    compare(out.cpu(), want, "f16", "repeated runs")
    plan.close()


def test_pointer_arrays_marshalled_once_give_the_same_result():
    # Plan.run_set: the pointer arrays are built once and passed to the same C entry point
    import ctypes
    pf = _pf()
    spec, ins = wl.c1_bias_res_layernorm_gelu(rows=37, n=768, dtype="f32")
    dev = [t.cuda() for t in ins]
    plan = pf.Plan(spec, 0)
    a, b = torch.empty_like(dev[0]), torch.empty_like(dev[0])
    stream = torch.cuda.current_stream().cuda_stream
    plan.run_ptrs([t.data_ptr() for t in dev], [a.data_ptr()], stream)
    ptrs = pf.PointerSet([t.data_ptr() for t in dev], [b.data_ptr()])
    for _ in range(3):
        plan.run_set(ptrs, ctypes.c_void_p(stream))
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    compare(b.cpu(), oracle_run(spec, ins)[0], "f32", "run_set")
    plan.close()
