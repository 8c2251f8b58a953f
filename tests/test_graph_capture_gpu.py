"""Launches of a plan recorded into a HIP graph: pf_chain_run only enqueues kernels on the caller's stream (no
allocation, no memset, no synchronisation), so launch-bound chains can be replayed from a graph.  Every replay
is checked against the eager result, with eager work and synchronisations between replays."""
import numpy as np
import pytest
import torch

import workloads as wl
from pf_testlib import compare, oracle_run

pytestmark = pytest.mark.gpu


def _capture_and_replay(spec, ins, what):
    from paper_2307_04995_amd import binding as pf
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
    plan = pf.Plan(spec, 0)
    dev = [t.cuda() for t in ins]
    shapes = plan.output_shapes()
    outs = [torch.empty(s, dtype=tdt[dt], device="cuda") for s, (_, dt) in zip(shapes, spec.outputs)]
    # eager reference
    plan.run(dev, outs)
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    want = oracle_run(spec, ins)
    for o, w, (_, dt) in zip(eager, want, spec.outputs):
        compare(o.cpu(), w, dt, what + " (eager)")
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        plan.run(dev, outs)                       # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            stream = torch.cuda.current_stream().cuda_stream
            for _ in range(3):                    # three launches per replay
                plan.run_ptrs([t.data_ptr() for t in dev], [o.data_ptr() for o in outs], stream)
    for it in range(4):
        for o in outs:
            o.fill_(float("nan"))                 # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, e in zip(outs, eager):
            assert torch.equal(o.view(torch.int16 if o.element_size() == 2 else torch.int32),
                               e.view(torch.int16 if e.element_size() == 2 else torch.int32)), f"{what}: replay {it} differs from eager"
    plan.close()


def test_row_chain_replays_from_a_graph():
    _capture_and_replay(*wl.c1_bias_res_layernorm_gelu(rows=64, n=768), "C1 in a graph")


def test_specialised_and_attention_chains_replay_from_a_graph():
    # a plan-time specialised kernel (module launch) and the attention family (self re-arming counters)
    shape = (6, 197)
    spec = wl.ChainSpec(inputs=[("f16", shape)])
    m = spec.op("reduce_max", 0)
    e = spec.op("exp", spec.op("sub", 0, m))
    spec.out(spec.op("div", e, spec.op("reduce_sum", e)), "f16")
    _capture_and_replay(spec, [wl.random_tensor(shape, "f16", 1401, scale=2.0)], "row program in a graph")
    _capture_and_replay(*wl.x2_decode_attention(b=1, h=6, t=300, d=64), "attention in a graph")


def test_fused_groupnorm_refuses_capture_and_the_two_launch_variant_replays():
    from paper_2307_04995_amd import binding as pf
    spec, ins = wl.c5_groupnorm_silu(n=2, h=16, w=16, ch=128, groups=8)
    dev = [t.cuda() for t in ins]
    out = torch.empty_like(dev[0])
    plan = pf.Plan(spec, 0, pf.PF_VARIANT_GROUP_RESIDENT)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        plan.run(dev, [out])
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            st = pf.pf_chain_run(plan.handle, [t.data_ptr() for t in dev], [out.data_ptr()], torch.cuda.current_stream().cuda_stream)
    assert st == pf.PF_ERR_UNSUPPORTED
    plan.close()
    # the two-launch variant has no launch-numbered state
    spec2 = spec
    plan2 = pf.Plan(spec2, 0, pf.PF_VARIANT_GROUP_TWO_PASS)
    plan2.run(dev, [out])
    torch.cuda.synchronize()
    eager = out.clone()
    graph2 = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph2, stream=side):
            plan2.run_ptrs([t.data_ptr() for t in dev], [out.data_ptr()], torch.cuda.current_stream().cuda_stream)
    for _ in range(3):
        out.fill_(0)
        torch.cuda.synchronize()
        graph2.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16))
    plan2.close()


def test_a_chain_of_several_kernels_replays_from_a_graph():
    # three kernels per run, tensors between them in the plan's arena: nine kernel nodes per replay
    n, c, h, w = 2, 24, 6, 10
    spec = wl.ChainSpec(inputs=[("f32", (n, c, h, w)), ("f32", (c,)), ("f32", (c,))])
    # (the activation keeps the chain from being the one-kernel form of the column family)
    v = spec.op("permute", spec.op("layernorm", spec.op("silu", spec.op("permute", 0, i=[0, 2, 3, 1])), 1, 2, f=[2.0 ** -20]), i=[0, 3, 1, 2])
    spec.out(v, "f32")
    ins = [wl.random_tensor((n, c, h, w), "f32", 1411), wl.random_tensor((c,), "f32", 1412, dist="positive"), wl.random_tensor((c,), "f32", 1413, scale=0.3)]
    _capture_and_replay(spec, ins, "channels-first layer normalisation in a graph")
