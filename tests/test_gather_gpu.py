"""GPU parity for layout-only chains with concatenations and slices (the gather family): bit-exact against the
oracle's byte moves, through the C ABI, arbitrary bit patterns (NaN payloads included)."""
import numpy as np
import pytest
import torch

import workloads as wl
from pf_testlib import check_chain, env, gpu_run

pytestmark = pytest.mark.gpu


def _pf():
    from paper_2307_04995_amd import binding as pf
    return pf


def _random_bits(shape, dtype, seed):
    g = np.random.default_rng(seed)
    nbits = 32 if dtype == "f32" else 16
    bits = g.integers(0, 1 << nbits, size=shape, dtype=np.uint32 if nbits == 32 else np.uint16)
    t = torch.from_numpy(bits.view(np.int32 if nbits == 32 else np.int16)).view(wl.DTYPES[dtype])
    return bits, t


def _check_bits(spec, tensors, bits, what):
    from oracle import pf_oracle as orc
    outs, info = gpu_run(spec, tensors)
    wants = orc.evaluate_layout_bits(spec, bits)
    assert len(outs) == len(wants)
    for k, (o, w) in enumerate(zip(outs, wants)):
        assert tuple(o.shape) == tuple(w.shape), f"{what}: output {k} shape {tuple(o.shape)} != {w.shape}"
        assert np.array_equal(wl.raw_bits(o), w), f"{what}: output {k} differs"
    return info


@pytest.mark.parametrize("n,c,h,w,groups,dtype", [(2, 116, 28, 28, 2, "f16"), (3, 232, 14, 14, 2, "f16"), (2, 464, 7, 7, 2, "bf16"),
                                                  (1, 48, 9, 5, 4, "f32"), (2, 24, 1, 1, 2, "f16")])
def test_concat_channel_shuffle_split(n, c, h, w, groups, dtype):
    spec, _ = wl.x3_channel_shuffle(n=n, c=c, h=h, w=w, groups=groups, dtype=dtype)
    shape = (n, c // 2, h, w)
    ba, ta = _random_bits(shape, dtype, 1201)
    bb, tb = _random_bits(shape, dtype, 1202)
    info = _check_bits(spec, [ta, tb], [ba, bb], f"channel shuffle {shape} g={groups} {dtype}")
    pf = _pf()
    assert info.family == pf.PF_FAMILY_GATHER and info.n_launches == 1
    # whole channel planes move: one run per (sample, channel) of each output
    assert info.workspace_bytes == n * c * 12


def test_three_way_concat_and_offset_slices_two_outputs():
    dtype = "f16"
    ba, ta = _random_bits((4, 6, 40), dtype, 1211)
    bb, tb = _random_bits((4, 3, 40), dtype, 1212)
    bc, tc = _random_bits((4, 5, 40), dtype, 1213)
    s = wl.ChainSpec(inputs=[(dtype, (4, 6, 40)), (dtype, (4, 3, 40)), (dtype, (4, 5, 40))])
    y = s.op("concat", s.op("concat", 0, 1, i=[1]), 2, i=[1])          # [4, 14, 40]
    s.out(s.op("slice", y, i=[1, 4, 7]), dtype)                          # rows 4..10: tail of a, all of b, head of c
    s.out(s.op("slice", y, i=[2, 8, 24]), dtype)                         # a window of the innermost axis
    _check_bits(s, [ta, tb, tc], [ba, bb, bc], "three-way concat")


def test_concat_along_the_innermost_axis_and_permutes():
    dtype = "f32"
    ba, ta = _random_bits((5, 7, 12), dtype, 1221)
    bb, tb = _random_bits((5, 7, 20), dtype, 1222)
    s = wl.ChainSpec(inputs=[(dtype, (5, 7, 12)), (dtype, (5, 7, 20))])
    y = s.op("concat", 0, 1, i=[2])                                      # [5, 7, 32]: runs of 12 and 20 -> 4 elements
    y = s.op("permute", y, i=[1, 0, 2])                                  # [7, 5, 32]
    s.out(y, dtype)
    _check_bits(s, [ta, tb], [ba, bb], "innermost concat + permute")


def test_channels_last_shuffle_moves_single_elements():
    # NHWC: the shuffle interleaves channels element by element; runs of one element, still exact
    dtype = "bf16"
    n, hw, c = 2, 6, 16
    ba, ta = _random_bits((n, hw, c // 2), dtype, 1231)
    bb, tb = _random_bits((n, hw, c // 2), dtype, 1232)
    s = wl.ChainSpec(inputs=[(dtype, (n, hw, c // 2)), (dtype, (n, hw, c // 2))])
    y = s.op("concat", 0, 1, i=[2])
    y = s.op("reshape", y, i=[n, hw, 2, c // 2])
    y = s.op("permute", y, i=[0, 1, 3, 2])
    y = s.op("reshape", y, i=[n, hw, c])
    s.out(s.op("slice", y, i=[2, 0, c // 2]), dtype)
    s.out(s.op("slice", y, i=[2, c // 2, c // 2]), dtype)
    _check_bits(s, [ta, tb], [ba, bb], "channels-last shuffle")


def test_arithmetic_next_to_concat_is_refused():
    pf = _pf()
    s = wl.ChainSpec(inputs=[("f16", (4, 8)), ("f16", (4, 8))])
    s.out(s.op("relu", s.op("concat", 0, 1, i=[1])), "f16")
    with env(PF_PARTITION="0"):  # not one kernel ...
        st, h = pf.pf_chain_plan(pf.make_desc(s), 0)
        assert st == pf.PF_ERR_UNSUPPORTED and h is None
    # ... so it runs as two: the index-map copy, then the element-wise kernel
    a, b = wl.random_tensor((4, 8), "f16", 4501), wl.random_tensor((4, 8), "f16", 4502)
    _, info, _ = check_chain(s, [a, b], what="concat > relu")
    assert info.n_kernels == 2
    s = wl.ChainSpec(inputs=[("f16", (4, 8)), ("f16", (4, 9))])
    s.out(s.op("concat", 0, 1, i=[0]), "f16")
    assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_ERR_SHAPE
