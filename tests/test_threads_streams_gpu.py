"""Plans made and run from several host threads at once, and launches on several streams: the plan-time
compile cache is shared by all threads, the error text is per thread, plans without workspace may run on any
number of streams."""
import threading

import numpy as np
import pytest
import torch

import workloads as wl
from pf_testlib import compare, oracle_run

pytestmark = pytest.mark.gpu


def test_planning_and_running_from_many_threads():
    from paper_2307_04995_amd import binding as pf
    torch.cuda.init()
    errors = []

    def worker(tid):
        try:
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()
            for rep in range(4):
                # half of the threads share chain structures (one compilation, many waiters), half have their own
                seed = (tid % 4) * 7 + rep if tid < 4 else 200 + tid * 10 + rep
                spec, ins, desc = wl.random_chain(seed)
                plan = pf.Plan(spec, 0)
                with torch.cuda.stream(stream):
                    dev = [t.cuda() for t in ins]
                    outs = [torch.empty(s, dtype=wl.DTYPES[dt], device="cuda") for s, (_, dt) in zip(plan.output_shapes(), spec.outputs)]
                    plan.run_ptrs([t.data_ptr() for t in dev], [o.data_ptr() for o in outs], stream.cuda_stream)
                stream.synchronize()
                want = oracle_run(spec, ins)
                for o, w, (_, dt) in zip(outs, want, spec.outputs):
                    compare(o.cpu(), w, dt, f"thread {tid}: {desc}")
                plan.close()
                # an error raised in this thread is reported with this thread's text
                bad = wl.ChainSpec(inputs=[("f32", (4, 8))])
                bad.out(bad.op("permute", 0, i=[0, 0]), "f32")
                assert pf.pf_chain_validate(pf.make_desc(bad)) == pf.PF_ERR_INVALID_ARG
                assert "permutation" in pf.pf_last_error()
        except Exception as e:  # noqa: BLE001 (collected and re-raised in the main thread)
            errors.append((tid, repr(e)))

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(8)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_one_plan_on_several_streams_at_once():
    # a row-family plan owns no workspace: the same plan may be in flight on any number of streams
    from paper_2307_04995_amd import binding as pf
    spec, ins = wl.c3_bias_res_layernorm(rows=2048, n=1024)
    plan = pf.Plan(spec, 0)
    assert plan.info().workspace_bytes == 0
    want = oracle_run(spec, ins)[0]
    streams = [torch.cuda.Stream() for _ in range(4)]
    outs = []
    for s in streams:
        with torch.cuda.stream(s):
            dev = [t.cuda() for t in ins]
            out = torch.empty_like(dev[0])
            for _ in range(5):
                plan.run_ptrs([t.data_ptr() for t in dev], [out.data_ptr()], s.cuda_stream)
            outs.append((dev, out))
    torch.cuda.synchronize()
    for _, out in outs:
        compare(out.cpu(), want, "f16", "LayerNorm on concurrent streams")
    plan.close()
