"""Differential test on seeded random chains: random shapes, dtypes, operand kinds (full shape, trailing
broadcast, extents of 1, one value per row, scalar), element-wise steps on both sides of a random core.  Every
chain goes through the C ABI (as planned by default, and again on the run-time-interpreted kernels when the
default was a specialised one) and is compared element by element with the fp64 oracle."""
import pytest

import workloads as wl
from pf_testlib import check_chain

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("block", range(16))
def test_random_chains_match_the_oracle(block):
    from paper_2307_04995_amd import binding as pf
    ran = 0
    for seed in range(block * 12, block * 12 + 12):
        spec, ins, desc = wl.random_chain(seed)
        try:
            check_chain(spec, ins, what=desc)
            ran += 1
        except pf.PfError as e:
            # a chain shape the library does not take must be refused as unsupported, never mis-run
            assert e.status in (pf.PF_ERR_UNSUPPORTED, pf.PF_ERR_ALIGNMENT), f"{desc}: {e}"
            print(f"refused ({pf.pf_status_str(e.status)}): {desc}: {e}")
    assert ran >= 8, "most random chains are expected to be supported"


@pytest.mark.parametrize("block", range(6))
def test_random_chains_with_transformed_broadcast_operands(block):
    # the same chains, with about half of the broadcast operands passed through an operator of their own first
    from paper_2307_04995_amd import binding as pf
    ran = 0
    for seed in range(block * 12, block * 12 + 12):
        spec, ins, desc = wl.random_chain(seed, transform_operands=True)
        try:
            check_chain(spec, ins, what=desc + " (operands transformed)")
            ran += 1
        except pf.PfError as e:
            assert e.status in (pf.PF_ERR_UNSUPPORTED, pf.PF_ERR_ALIGNMENT), f"{desc}: {e}"
            print(f"refused ({pf.pf_status_str(e.status)}): {desc}: {e}")
    assert ran >= 8


@pytest.mark.parametrize("block", range(6))
def test_random_groupnorm_chains_match_the_oracle(block):
    # groups of any width, small and large tiles, one or several workgroups per sample; both variants
    from paper_2307_04995_amd import binding as pf
    for seed in range(block * 10, block * 10 + 10):
        spec, ins, desc = wl.random_groupnorm_chain(seed)
        _, info, _ = check_chain(spec, ins, what=desc)
        assert info.family == pf.PF_FAMILY_GROUP
        other = pf.PF_VARIANT_GROUP_TWO_PASS if info.variant == pf.PF_VARIANT_GROUP_RESIDENT else pf.PF_VARIANT_GROUP_RESIDENT
        try:
            check_chain(spec, ins, variant=other, what=desc + f" (variant {other})")
        except pf.PfError as e:
            assert e.status == pf.PF_ERR_UNSUPPORTED, f"{desc}: {e}"     # e.g. the fused variant with a per-sample operand


def _run_random(builder, seeds, allowed=()):
    from paper_2307_04995_amd import binding as pf
    ran = 0
    for seed in seeds:
        spec, ins, desc = builder(seed)
        try:
            check_chain(spec, ins, what=desc)
            ran += 1
        except pf.PfError as e:
            assert e.status in allowed, f"{desc}: {e}"
            print(f"refused ({pf.pf_status_str(e.status)}): {desc}: {e}")
    return ran


@pytest.mark.parametrize("block", range(5))
def test_random_depthwise_convolution_chains_match_the_oracle(block):
    assert _run_random(wl.random_stencil_chain, range(block * 12, block * 12 + 12)) == 12


@pytest.mark.parametrize("block", range(4))
def test_random_attention_chains_match_the_oracle(block):
    assert _run_random(wl.random_attention_chain, range(block * 10, block * 10 + 10)) == 10


@pytest.mark.parametrize("block", range(5))
def test_random_permutation_chains_match_the_oracle(block):
    from paper_2307_04995_amd import binding as pf
    # (a permutation that leaves the layout as it is has nothing to do and is refused)
    ran = _run_random(wl.random_permute_chain, range(block * 12, block * 12 + 12), allowed=(pf.PF_ERR_UNSUPPORTED,))
    assert ran >= 9


@pytest.mark.parametrize("block,vectors_per_lane", [(b, 0) for b in range(5)] + [(5, 2), (6, 4)])
def test_random_layout_chains_are_bit_exact(block, vectors_per_lane):
    # joins, slices, permutations and reshapes at random: every output bit pattern must come from the right place
    # (the last two blocks force the copy kernels that move two and four vectors per lane, which the planner itself
    # takes for large tensors only, onto these small, ragged cases)
    import numpy as np
    import torch
    from oracle import pf_oracle as orc
    from paper_2307_04995_amd import binding as pf
    from pf_testlib import env, gpu_run
    ran = 0
    with env(PF_GATHER_K=str(vectors_per_lane) if vectors_per_lane else None):
        ran = _layout_block(block, np, torch, orc, pf, gpu_run)
    assert ran >= 12


def _layout_block(block, np, torch, orc, pf, gpu_run):
    ran = 0
    for seed in range(block * 16, block * 16 + 16):
        spec, desc = wl.random_layout_chain(seed)
        g = np.random.default_rng(9000 + seed)
        bits, tensors = [], []
        for dt, shape in spec.inputs:
            wide = dt == "f32"
            b = g.integers(0, 1 << (32 if wide else 16), size=shape, dtype=np.uint32 if wide else np.uint16)
            bits.append(b)
            tensors.append(torch.from_numpy(b.view(np.int32 if wide else np.int16)).view(wl.DTYPES[dt]))
        try:
            outs, info = gpu_run(spec, tensors)
        except pf.PfError as e:
            assert e.status in (pf.PF_ERR_UNSUPPORTED, pf.PF_ERR_ALIGNMENT), f"{desc}: {e}"
            print(f"refused ({pf.pf_status_str(e.status)}): {desc}: {e}")
            continue
        wants = orc.evaluate_layout_bits(spec, bits)
        for k, (o, w) in enumerate(zip(outs, wants)):
            assert tuple(o.shape) == tuple(w.shape), f"{desc}: output {k} shape"
            assert np.array_equal(wl.raw_bits(o), w), f"{desc}: output {k} differs"
        ran += 1
    return ran


@pytest.mark.parametrize("block", range(4))
def test_random_pooling_chains_match_the_oracle(block):
    assert _run_random(wl.random_pool_chain, range(block * 12, block * 12 + 12)) == 12
