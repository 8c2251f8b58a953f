"""GPU parity for the stencil family: element-wise steps fused around a depthwise 3 x 3 convolution on a
channels-last tensor (the EfficientNet fragment), through the C ABI, element by element against the fp64 oracle."""
import numpy as np
import pytest

import workloads as wl
from pf_testlib import check_chain, SPEC_JIT

pytestmark = pytest.mark.gpu


def _pf():
    from paper_2307_04995_amd import binding as pf
    return pf


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("n,h,w,c,dtype", [(2, 13, 11, 64, "f16"), (1, 7, 7, 240, "f16"), (3, 5, 9, 8, "f32"), (1, 20, 3, 144, "bf16"),
                                           (1, 1, 1, 16, "f16"), (2, 6, 6, 32, "f32"), (1, 1, 40, 24, "bf16"), (1, 19, 1, 8, "f16")])
def test_relu_depthwise_conv_bias(n, h, w, c, dtype, variant):
    spec, ins = wl.x4_relu_dwconv(n=n, h=h, w=w, c=c, dtype=dtype)
    _, info, _ = check_chain(spec, ins, variant=variant, what=f"relu -> dwconv -> bias [{n},{h},{w},{c}] {dtype} variant {variant}")
    pf = _pf()
    assert info.family == pf.PF_FAMILY_STENCIL and info.n_launches == 1 and info.variant == variant
    assert info.spec_id == SPEC_JIT


@pytest.mark.parametrize("n,h,w,c,k,stride,dtype", [
    (2, 9, 11, 12, 3, 1, "f16"),     # 24 bytes per position: one whole vector and one of four channels
    (1, 7, 7, 100, 3, 1, "bf16"),    # last vector of four
    (2, 6, 5, 6, 3, 1, "f32"),       # fp32, 24 bytes per position
    (1, 10, 9, 20, 5, 1, "f16"),     # 5 x 5 kernel (staged variant)
    (2, 11, 13, 36, 3, 2, "f16"),    # down-sampling convolution
    (1, 5, 5, 3, 3, 1, "f16"),       # fewer channels than one vector
])
def test_convolution_on_channel_counts_that_are_not_whole_vectors(n, h, w, c, k, stride, dtype):
    pf = _pf()
    spec, ins = wl.x4_relu_dwconv(n=n, h=h, w=w, c=c, k=k, dtype=dtype, stride=stride, salt=3)
    variants = (None,) if (k == 5 or stride != 1) else (0, 1)
    for variant in variants:
        _, info, _ = check_chain(spec, ins, variant=variant, what=f"relu -> dwconv {k}x{k}/{stride} -> bias, {c} channels (ragged) {dtype} variant {variant}")
        assert info.family == pf.PF_FAMILY_STENCIL and info.n_launches == 1


def test_convolution_on_ragged_channels_interpreted():
    spec, ins = wl.x4_relu_dwconv(n=1, h=6, w=7, c=12, dtype="f16", salt=4)
    _, info, _ = check_chain(spec, ins, generic=True, what="relu -> dwconv -> bias, 12 channels, interpreted kernel")
    assert info.spec_id == 0


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_convolution_alone_and_asymmetric_kernel(dtype):
    # distinct weights in all nine taps, no other operator: tap order and padding show directly
    n, h, w, c = 1, 9, 10, 16
    x = wl.random_tensor((n, h, w, c), dtype, 1301)
    k = wl.quantise(np.arange(1, 10, dtype=np.float32).reshape(3, 3, 1).repeat(c, 2) / 16.0, dtype)
    spec = wl.ChainSpec(inputs=[(dtype, (n, h, w, c)), (dtype, (3, 3, c))])
    spec.out(spec.op("dwconv2d", 0, 1), dtype)
    for variant in (0, 1):
        check_chain(spec, [x, k], variant=variant, what=f"dwconv alone, variant {variant}")


def test_operands_on_both_sides_of_the_convolution():
    # y = silu(dwconv(relu(x + shift[c])) + bias[c]) + res: a broadcast operand before the convolution, a
    # broadcast and a full-shape operand after it
    dtype = "f16"
    n, h, w, c = 2, 11, 7, 48
    x = wl.random_tensor((n, h, w, c), dtype, 1311)
    shift = wl.random_tensor((c,), dtype, 1312, scale=0.5)
    k = wl.random_tensor((3, 3, c), dtype, 1313, scale=0.3)
    bias = wl.random_tensor((c,), dtype, 1314, scale=0.5)
    res = wl.random_tensor((n, h, w, c), dtype, 1315, scale=0.5)
    s = wl.ChainSpec(inputs=[(dtype, (n, h, w, c)), (dtype, (c,)), (dtype, (3, 3, c)), (dtype, (c,)), (dtype, (n, h, w, c))])
    v = s.op("relu", s.op("add", 0, 1))
    v = s.op("dwconv2d", v, 2)
    v = s.op("silu", s.op("add", v, 3))
    s.out(s.op("add", v, 4), dtype)
    # (fp16 values that went through an addition are kept in fp32: the staged variant's tile would not fit)
    for variant in (0, None):
        check_chain(s, [x, shift, k, bias, res], variant=variant, what=f"operands on both sides of a dwconv, variant {variant}")
    # the same chain in fp32 fits the tile
    ins32 = [wl.quantise(wl.widen(t).astype(np.float32), "f32") for t in (x, shift, k, bias, res)]
    s32 = wl.ChainSpec(inputs=[("f32", sh) for _, sh in s.inputs], ops=s.ops, outputs=[(v, "f32") for v, _ in s.outputs])
    _, info, _ = check_chain(s32, ins32, variant=1, what="operands on both sides of a dwconv, fp32, staged")
    assert info.variant == 1


def test_padding_comes_after_the_activation():
    # sigmoid(0) = 0.5: if the padding were applied before the activation the border would see 0.5, not 0
    dtype = "f32"
    n, h, w, c = 1, 4, 4, 8
    x = wl.random_tensor((n, h, w, c), dtype, 1321)
    k = wl.quantise(np.ones((3, 3, c), dtype=np.float32), dtype)
    s = wl.ChainSpec(inputs=[(dtype, (n, h, w, c)), (dtype, (3, 3, c))])
    s.out(s.op("dwconv2d", s.op("sigmoid", 0), 1), dtype)
    for variant in (0, 1):
        check_chain(s, [x, k], variant=variant, what=f"sigmoid -> dwconv, variant {variant}")


def test_wide_channel_counts_fall_back_to_the_direct_variant():
    # 1152 channels in fp16: the LDS tile of the staged variant would not fit
    pf = _pf()
    spec, ins = wl.x4_relu_dwconv(n=1, h=7, w=7, c=1152, dtype="f16")
    _, info, _ = check_chain(spec, ins, what="relu -> dwconv -> bias, 1152 channels")
    assert info.variant in (pf.PF_VARIANT_STENCIL_DIRECT, pf.PF_VARIANT_STENCIL_STAGED)
    spec, ins = wl.x4_relu_dwconv(n=1, h=5, w=5, c=2048, dtype="f32")
    _, info, _ = check_chain(spec, ins, what="relu -> dwconv -> bias, 2048 fp32 channels")
    assert info.variant == pf.PF_VARIANT_STENCIL_DIRECT


@pytest.mark.parametrize("n,h,w,c,dtype", [(2, 13, 11, 64, "f16"), (1, 7, 7, 240, "f16"), (2, 5, 9, 8, "f32"), (1, 9, 3, 48, "bf16"), (1, 1, 1, 16, "f16"),
                                           (1, 2, 30, 24, "f32")])
def test_five_by_five_kernels(n, h, w, c, dtype):
    spec, ins = wl.x4_relu_dwconv(n=n, h=h, w=w, c=c, k=5, dtype=dtype)
    _, info, _ = check_chain(spec, ins, what=f"relu -> 5x5 dwconv -> bias [{n},{h},{w},{c}] {dtype}")
    assert info.variant == _pf().PF_VARIANT_STENCIL_STAGED
    # asymmetric 5 x 5 kernel alone: tap order and the two-wide padding
    x = wl.random_tensor((1, 6, 7, 8), dtype, 1331)
    k = wl.quantise(np.arange(1, 26, dtype=np.float32).reshape(5, 5, 1).repeat(8, 2) / 64.0, dtype)
    s = wl.ChainSpec(inputs=[(dtype, (1, 6, 7, 8)), (dtype, (5, 5, 8))])
    s.out(s.op("dwconv2d", 0, 1), dtype)
    check_chain(s, [x, k], what="5x5 dwconv alone")


@pytest.mark.parametrize("n,h,w,c,k,stride,dtype", [(2, 14, 14, 96, 3, 2, "f16"), (1, 9, 7, 40, 5, 2, "f16"), (3, 16, 15, 32, 3, 2, "bf16"),
                                                    (1, 13, 13, 16, 3, 3, "f32"), (2, 28, 28, 144, 5, 2, "f16"), (1, 1, 1, 8, 3, 2, "f32")])
def test_strided_depthwise_convolution(n, h, w, c, k, stride, dtype):
    # the down-sampling blocks: stride 2 (3 once), even and odd image extents, both kernel sizes
    pf = _pf()
    spec, ins = wl.x4_relu_dwconv(n=n, h=h, w=w, c=c, k=k, dtype=dtype, stride=stride, salt=5)
    outs, info, _ = check_chain(spec, ins, what=f"strided dwconv {k}x{k}/{stride} {dtype}")
    assert info.family == pf.PF_FAMILY_STENCIL and info.variant == pf.PF_VARIANT_STENCIL_STRIDED and info.n_launches == 1
    assert tuple(outs[0].shape) == (n, (h - 1) // stride + 1, (w - 1) // stride + 1, c)


def test_strided_convolution_with_operands_on_both_sides():
    # silu(dwconv_stride2(relu(x + t[n,1,1,c])) + bias[c]) + res[n, h/2, w/2, c]: epilogue operands have the
    # result's shape, the prologue's the input's (and one of them broadcasts the general way)
    dtype = "f16"
    n, h, w, c = 2, 12, 10, 48
    oh, ow = (h - 1) // 2 + 1, (w - 1) // 2 + 1
    x = wl.random_tensor((n, h, w, c), dtype, 1341)
    t = wl.random_tensor((n, 1, 1, c), dtype, 1342, scale=0.5)
    k = wl.random_tensor((3, 3, c), dtype, 1343, scale=0.3)
    bias = wl.random_tensor((c,), dtype, 1344, scale=0.5)
    res = wl.random_tensor((n, oh, ow, c), dtype, 1345, scale=0.5)
    s = wl.ChainSpec(inputs=[(dtype, (n, h, w, c)), (dtype, (n, 1, 1, c)), (dtype, (3, 3, c)), (dtype, (c,)), (dtype, (n, oh, ow, c))])
    v = s.op("relu", s.op("add", 0, 1))
    v = s.op("dwconv2d", v, 2, i=[2])
    v = s.op("silu", s.op("add", v, 3))
    s.out(s.op("add", v, 4), dtype)
    check_chain(s, [x, t, k, bias, res], what="strided dwconv, operands on both sides")


def test_stride_attribute_is_checked():
    pf = _pf()
    s = wl.ChainSpec(inputs=[("f16", (1, 8, 8, 8)), ("f16", (3, 3, 8))])
    s.out(s.op("dwconv2d", 0, 1, i=[0]), "f16")
    assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_ERR_INVALID_ARG
    s = wl.ChainSpec(inputs=[("f16", (1, 8, 8, 8)), ("f16", (3, 3, 8))])
    s.out(s.op("dwconv2d", 0, 1, i=[2]), "f16")
    st, t = pf.pf_chain_infer_shape(pf.make_desc(s), 2)
    assert st == pf.PF_OK and [t.shape[q] for q in range(t.rank)] == [1, 4, 4, 8]


def test_other_kernel_sizes_are_refused():
    pf = _pf()
    s = wl.ChainSpec(inputs=[("f16", (1, 8, 8, 16)), ("f16", (7, 7, 16))])
    s.out(s.op("dwconv2d", 0, 1), "f16")
    st, h = pf.pf_chain_plan(pf.make_desc(s), 0)
    assert st == pf.PF_ERR_UNSUPPORTED and h is None
    s = wl.ChainSpec(inputs=[("f16", (1, 8, 8, 16)), ("f16", (3, 3, 8))])
    s.out(s.op("dwconv2d", 0, 1), "f16")
    assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_ERR_SHAPE
