"""GPU parity for the attention family: one new token against cached keys and values in one kernel
(concat -> matrix-vector -> scale -> softmax -> concat -> vector-matrix), through the C ABI, element by element
against the fp64 oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
from pf_testlib import check_chain, compare, env, gpu_run, oracle_run

pytestmark = pytest.mark.gpu


def _pf():
    from paper_2307_04995_amd import binding as pf
    return pf


@pytest.mark.parametrize("b,h,t,d,dtype", [(1, 12, 1023, 64, "f16"), (2, 3, 37, 64, "bf16"), (1, 2, 129, 128, "f16"),
                                           (1, 4, 300, 64, "f32"), (1, 1, 1, 64, "f16"), (2, 2, 515, 32, "f32"),
                                           (1, 3, 2049, 256, "bf16")])
def test_one_token_attention(b, h, t, d, dtype):
    spec, ins = wl.x2_decode_attention(b=b, h=h, t=t, d=d, dtype=dtype)
    _, info, _ = check_chain(spec, ins, what=f"attention b={b} h={h} t={t} d={d} {dtype}")
    pf = _pf()
    assert info.family == pf.PF_FAMILY_ATTENTION and info.n_launches == 1
    assert info.grid[1] == b * h


@pytest.mark.parametrize("nv", [1, 2, 4, 8])
def test_every_split_shape_gives_the_same_answer(nv):
    # t + 1 = 200 rows: 7 slices of 32 rows, 4 of 64, 2 of 128, one of 256 (no merge at all)
    spec, ins = wl.x2_decode_attention(b=1, h=5, t=199, d=64, dtype="f16")
    with env(PF_ATTN_NV=nv):
        _, info, _ = check_chain(spec, ins, what=f"attention, {nv} steps per workgroup")
    assert info.vectors_per_lane == nv
    assert info.grid[0] == -(-200 // (32 * nv))


@pytest.mark.parametrize("b,h,t,d,dtype", [(1, 12, 1023, 64, "f16"), (2, 3, 37, 64, "bf16"), (1, 2, 129, 128, "f16"),
                                           (1, 4, 300, 64, "f32"), (1, 1, 1, 64, "f16"), (1, 3, 2049, 256, "bf16")])
@pytest.mark.parametrize("chunks", [2, 3, 8])
def test_streaming_walk_over_longer_slices(b, h, t, d, dtype, chunks):
    # the variant that walks its slice in chunks with running (maximum, sum, weighted values) per lane; slices
    # that end inside a chunk, lanes and waves that never see a row, a single slice (no merge) all occur here
    pf = _pf()
    spec, ins = wl.x2_decode_attention(b=b, h=h, t=t, d=d, dtype=dtype)
    with env(PF_ATTN_CHUNKS=chunks):
        _, info, _ = check_chain(spec, ins, variant=pf.PF_VARIANT_ATTN_STREAM, what=f"streamed attention t={t} d={d} {dtype} chunks={chunks}")
    assert info.variant == pf.PF_VARIANT_ATTN_STREAM and info.n_launches == 1
    rows_per_wg = (256 // (d * (4 if dtype == "f32" else 2) // 16)) * info.vectors_per_lane * chunks
    assert info.grid[0] == -(-(t + 1) // rows_per_wg)


def test_many_heads_take_the_streaming_walk_by_default():
    # enough heads that one slice per head fills the device: no partial results, no merge
    pf = _pf()
    spec, ins = wl.x2_decode_attention(b=32, h=25, t=511, d=64, dtype="f16")
    _, info, _ = check_chain(spec, ins, what="attention, 800 heads")
    assert info.variant == pf.PF_VARIANT_ATTN_STREAM and tuple(info.grid)[:2] == (1, 800)


def test_streaming_walk_with_cache_outputs_and_peaked_scores():
    pf = _pf()
    spec, ins = wl.x2_decode_attention(b=2, h=3, t=333, d=64, dtype="bf16", cache_outputs=True)
    q, k, v, K, V = ins
    K = K.clone()
    K[1, 1, 300] = q[1, 1] * 6.0          # a late row dominates: every earlier running sum is rescaled away
    outs, info, _ = check_chain(spec, [q, k, v, K, V], variant=pf.PF_VARIANT_ATTN_STREAM, what="streamed attention, cache outputs")
    assert info.variant == pf.PF_VARIANT_ATTN_STREAM
    assert torch.equal(outs[1].view(torch.int16), torch.cat([K, k[:, :, None, :]], dim=2).view(torch.int16))
    assert torch.equal(outs[2].view(torch.int16), torch.cat([V, v[:, :, None, :]], dim=2).view(torch.int16))


def test_grown_caches_as_outputs_are_bit_exact():
    spec, ins = wl.x2_decode_attention(b=2, h=3, t=77, d=64, dtype="bf16", cache_outputs=True)
    outs, info, _ = check_chain(spec, ins, what="attention with cache outputs")
    q, k, v, K, V = ins
    assert torch.equal(outs[1].view(torch.int16), torch.cat([K, k[:, :, None, :]], dim=2).view(torch.int16))
    assert torch.equal(outs[2].view(torch.int16), torch.cat([V, v[:, :, None, :]], dim=2).view(torch.int16))


def test_caches_that_already_hold_the_new_rows():
    b, h, t, d = 2, 4, 140, 64
    q = wl.random_tensor((b, h, d), "f16", 1101)
    K = wl.random_tensor((b, h, t, d), "f16", 1102)
    V = wl.random_tensor((b, h, t, d), "f16", 1103)
    spec = wl.ChainSpec(inputs=[("f16", (b, h, d)), ("f16", (b, h, t, d)), ("f16", (b, h, t, d))])
    s = spec.op("matvec", 1, 0)
    p = spec.op("softmax", spec.op("scale", s, f=[0.125]))
    spec.out(spec.op("vecmat", p, 2), "f16")
    check_chain(spec, [q, K, V], what="attention without concatenation")
    # and without the scale
    spec = wl.ChainSpec(inputs=[("f16", (b, h, d)), ("f16", (b, h, t, d)), ("f16", (b, h, t, d))])
    p = spec.op("softmax", spec.op("matvec", 1, 0))
    spec.out(spec.op("vecmat", p, 2), "f16")
    check_chain(spec, [wl.random_tensor((b, h, d), "f16", 1104, scale=0.2), K, V], what="attention, unscaled")


def test_a_plan_can_run_again_and_again():
    # the per-head arrival counters re-arm themselves: every launch of one plan merges correctly
    pf = _pf()
    spec, ins = wl.x2_decode_attention(b=1, h=7, t=700, d=64, dtype="f16")
    want = oracle_run(spec, ins)[0]
    dev = [t.cuda() for t in ins]
    plan = pf.Plan(spec, 0)
    out = torch.empty((1, 7, 64), dtype=torch.float16, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    for it in range(5):
        out.fill_(float("nan"))
        plan.run_ptrs([t.data_ptr() for t in dev], [out.data_ptr()], stream)
        torch.cuda.synchronize()
        compare(out.cpu(), want, "f16", f"attention, launch {it}")
    plan.close()


def test_peaked_scores_and_large_magnitudes():
    # one key dominates in some heads (softmax close to one-hot), scores of a few hundred before scaling
    b, h, t, d = 1, 6, 260, 64
    spec, ins = wl.x2_decode_attention(b=b, h=h, t=t, d=d, dtype="f32")
    q, k, v, K, V = ins
    K = K.clone()
    K[0, 2, 100] = q[0, 2] * 8.0
    K[0, 4, 259] = q[0, 4] * 20.0
    check_chain(spec, [q, k, v, K, V], what="attention, peaked")


def test_other_arrangements_of_the_contractions_are_refused():
    pf = _pf()
    b, h, t, d = 1, 2, 16, 64
    # matvec alone
    s = wl.ChainSpec(inputs=[("f16", (b, h, d)), ("f16", (b, h, t, d))])
    s.out(s.op("matvec", 1, 0), "f16")
    st, hd = pf.pf_chain_plan(pf.make_desc(s), 0)
    assert st == pf.PF_ERR_UNSUPPORTED and hd is None
    # an element-wise step between softmax and vecmat
    s = wl.ChainSpec(inputs=[("f16", (b, h, d)), ("f16", (b, h, t, d)), ("f16", (b, h, t, d))])
    p = s.op("relu", s.op("softmax", s.op("matvec", 1, 0)))
    s.out(s.op("vecmat", p, 2), "f16")
    st, hd = pf.pf_chain_plan(pf.make_desc(s), 0)
    assert st == pf.PF_ERR_UNSUPPORTED and hd is None
    # shapes that do not fit
    s = wl.ChainSpec(inputs=[("f16", (b, h, d + 8)), ("f16", (b, h, t, d))])
    s.out(s.op("matvec", 1, 0), "f16")
    assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_ERR_SHAPE


def test_bounded_wait_of_the_merging_slice_gives_up_instead_of_hanging():
    # with the re-read limit forced to zero the head's last slice does not wait for the others: the launch must still
    # end, and the plan must report it (results of such a launch are not checked); a plan with the default limit on the
    # same shape is exact again, and so is the counted merge
    pf = _pf()
    spec, ins = wl.x2_decode_attention(b=2, h=5, t=1500, d=64, dtype="f16")
    dev = [t.cuda() for t in ins]
    out = torch.empty((2, 5, 64), dtype=torch.float16, device="cuda")
    with env(PF_ATTN_SPIN_LIMIT="0"):
        plan = pf.Plan(spec, 0)
    for _ in range(3):
        plan.run(dev, [out])
    torch.cuda.synchronize()
    assert plan.poll_error() in (0, 1)      # usually 1; 0 only if every word happened to be there at the first look
    assert plan.poll_error() == 0           # reading clears it (and puts the words back to "empty")
    plan.close()
    check_chain(spec, ins, what="attention after a forced give-up")
    with env(PF_ATTN_POLLED="0"):
        _, info, _ = check_chain(spec, ins, what="attention, counted merge")
    assert info.n_launches == 1
