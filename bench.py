#!/usr/bin/env python3
"""Benchmark of the fused-chain hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch: one `pf_chain_run` of each of the five benchmark
chains (benchmark configs C1 .. C5 at full size), inputs already resident in HBM.  Every chain rotates over
several buffer sets and a step moves 380 MB, so no launch finds its data in the 256 MB last-level cache: the
numbers printed are the cold, HBM-bound ones.

One JSON line is printed.  `value` is GB/s of the bytes the five chains have to move (inputs once + outputs once;
for the causal chain the 16-byte vectors that lie wholly above the diagonal are never needed and are not
counted) over the wall time of a step.  `roofline` prices the dominant kernel of the step -- the chain that takes
longest, C5 -- against the 8 TB/s HBM peak from its average launch duration, measured with HIP events around its
launches inside the timed region.  `cpu_baseline` is the fp64 oracle timed on the host cores on whole passes over the
same five chains.  `chains` has every chain timed on its own (at least 200 launches each, whatever --steps says) and
a plain copy kernel, for context.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
ROTATE_BYTES = 640 * 1024 * 1024


def causal_needed_read_bytes(b, h, s, s_k, esize):
    """Bytes of the score tensor that are not wholly masked 16-byte vectors."""
    vec = 16 // esize
    per_matrix = 0
    for i in range(s):
        keep = min(s_k, i + 1)
        per_matrix += ((keep + vec - 1) // vec) * 16
    return b * h * per_matrix


def full_size_chain(name):
    """(spec, inputs, algorithmic bytes, nominal bytes, label) at the benchmark's full size."""
    import workloads as wl
    if name == "C1x256":
        # the C1 chain and kernel with 256 times the rows: what that kernel does when it is not launch-bound
        spec, ins = wl.c1_bias_res_layernorm_gelu(rows=65536)
    else:
        spec, ins = wl.CONFIGS[name]()
    esz = {"f32": 4, "f16": 2, "bf16": 2}
    nominal = sum(t.numel() * t.element_size() for t in ins)
    out_bytes = 0
    import numpy as np
    from paper_2307_04995_amd import binding as pf
    plan = pf.Plan(spec, 0)
    for shape, (_, dt) in zip(plan.output_shapes(), spec.outputs):
        out_bytes += int(np.prod(shape)) * esz[dt]
    plan.close()
    nominal += out_bytes
    algorithmic = nominal
    if name == "C2":
        b, h, s, s_k = spec.inputs[0][1]
        algorithmic = causal_needed_read_bytes(b, h, s, s_k, 2) + out_bytes
    labels = {
        "C1": "C1 fp32 x+res+bias -> LayerNorm -> GELU(erf) [256x768]",
        "C1x256": "the C1 chain at [65536x768] (same kernel, 256 x the rows: its bandwidth when not launch-bound; not a BASELINE config)",
        "C2": "C2 fp16 scale -> causal mask -> softmax [8,12,512,512]",
        "C3": "C3 fp16 x+bias+res -> LayerNorm [16384x1024]",
        "C4": "C4 bf16 (Q+bias)*0.125 -> permute [32,512,16,64]->[32,16,512,64]",
        "C5": "C5 fp16 NHWC GroupNorm(32)+SiLU [16,64,64,512]",
        "X1": "X1 bf16 (K+bias)*0.125 -> transpose [32,512,1024]->[32,1024,512] (not a BASELINE config)",
        "X4": "X4 fp16 RELU -> depthwise 3x3 conv -> +bias, NHWC [32,56,56,240] (not a BASELINE config)",
        "X3": "X3 fp16 concat -> channel shuffle (2 groups) -> split, NCHW [128,232,28,28] (not a BASELINE config)",
        "X2": "X2 fp16 one-token attention, 8x25 heads, 1023 cached rows + 1, d=64 (not a BASELINE config)",
        "X5": "X5 fp16 NHWC GroupNorm(32)+SiLU [16,64,64,320], 10 channels per group (not a BASELINE config)",
        "X6": "X6 fp16 SiLU -> mean over H, W, NHWC [32,56,56,240] (not a BASELINE config)",
        "X7": "X7 fp16 LayerNorm over the channels of NCHW [64,96,56,56], written permute -> LayerNorm -> permute (not a BASELINE config)",
    }
    return spec, ins, algorithmic, nominal, labels[name]


def time_chain(spec, ins, steps, warmup, variant=None, hot=None, graph=None):
    """Returns (ms per step from host clock, ms per launch from HIP events, plan info).  The timed launches
    rotate over the buffer sets (cold).  If `hot` is a list, the average launch duration of the same number
    of launches on ONE buffer set (data resident in the last-level cache where it fits) is appended to it.
    If `graph` is a list, the launches are also recorded into a HIP graph (one launch per buffer set) and the
    average launch duration under graph replay is appended: what a launch-bound chain gains from it."""
    import numpy as np
    import torch
    from paper_2307_04995_amd import binding as pf
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
    plan = pf.Plan(spec, 0, variant)
    info = plan.info()
    shapes = plan.output_shapes()
    per_set = sum(t.numel() * t.element_size() for t in ins)
    per_set += sum(int(np.prod(s)) * {"f32": 4, "f16": 2, "bf16": 2}[dt] for s, (_, dt) in zip(shapes, spec.outputs))
    n_sets = max(3, min(64, -(-ROTATE_BYTES // per_set)))
    base = [t.cuda() for t in ins]
    sets = []
    for k in range(n_sets):
        # broadcast operands (a few KB) are shared; streamed tensors get their own copy per set
        i_k = [t if t.numel() * t.element_size() < 65536 else t.clone() for t in base]
        o_k = [torch.empty(s, dtype=tdt[dt], device="cuda") for s, (_, dt) in zip(shapes, spec.outputs)]
        sets.append(([t.data_ptr() for t in i_k], [t.data_ptr() for t in o_k], i_k, o_k))
    stream = torch.cuda.current_stream().cuda_stream
    # the pointer arrays of every buffer set are marshalled once: the timed loop is one foreign call per launch
    import ctypes
    cstream = ctypes.c_void_p(stream)
    psets = [pf.PointerSet(ip, op) for ip, op, _, _ in sets]
    for k in range(warmup):
        plan.run_set(psets[k % n_sets], cstream)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for k in range(steps):
        plan.run_set(psets[k % n_sets], cstream)
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    host_ms = (t1 - t0) * 1e3 / steps
    event_ms = ev0.elapsed_time(ev1) / steps
    if hot is not None:
        ip, op, _, _ = sets[0]
        for k in range(warmup):
            plan.run_ptrs(ip, op, stream)
        ev0.record()
        for k in range(steps):
            plan.run_ptrs(ip, op, stream)
        ev1.record()
        torch.cuda.synchronize()
        hot.append(ev0.elapsed_time(ev1) / steps)
    if graph is not None:
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            plan.run_ptrs(sets[0][0], sets[0][1], side.cuda_stream)
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                cs = torch.cuda.current_stream().cuda_stream
                for k in range(n_sets):
                    plan.run_ptrs(sets[k][0], sets[k][1], cs)
        reps = max(1, steps // n_sets)
        g.replay()
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(reps):
            g.replay()
        ev1.record()
        torch.cuda.synchronize()
        graph.append(ev0.elapsed_time(ev1) / (reps * n_sets))
    plan.close()
    del sets
    torch.cuda.empty_cache()
    return host_ms, event_ms, info


def time_copy(nbytes, steps, warmup, variant=2, graph=False):
    """Average duration of a launch of the library's plain copy kernel over rotating buffers, launched back to back
    from Python, or (graph=True) replayed from a HIP graph, where the host's launch rate plays no part."""
    import torch
    from paper_2307_04995_amd import binding as pf
    n_sets = min(64 if graph else 512, max(3, -(-ROTATE_BYTES // (2 * nbytes))))
    bufs = [(torch.empty(nbytes, dtype=torch.uint8, device="cuda"), torch.empty(nbytes, dtype=torch.uint8, device="cuda"))
            for _ in range(n_sets)]
    for a, _ in bufs:
        a.fill_(1)
    if graph:
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            pf.pf_copy_probe(bufs[0][0].data_ptr(), bufs[0][1].data_ptr(), nbytes, variant, side.cuda_stream)
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                cs = torch.cuda.current_stream().cuda_stream
                for a, b in bufs:
                    if pf.pf_copy_probe(a.data_ptr(), b.data_ptr(), nbytes, variant, cs) != 0:
                        raise RuntimeError(pf.pf_last_error())
        reps = max(1, steps // n_sets)
        g.replay()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(reps):
            g.replay()
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / (reps * n_sets)
    stream = torch.cuda.current_stream().cuda_stream
    for k in range(warmup):
        a, b = bufs[k % n_sets]
        pf.pf_copy_probe(a.data_ptr(), b.data_ptr(), nbytes, variant, stream)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for k in range(steps):
        a, b = bufs[k % n_sets]
        st = pf.pf_copy_probe(a.data_ptr(), b.data_ptr(), nbytes, variant, stream)
        if st != 0:
            raise RuntimeError(pf.pf_last_error())
    ev1.record()
    torch.cuda.synchronize()
    return ev0.elapsed_time(ev1) / steps


BENCH_CHAINS = ["C1", "C2", "C3", "C4", "C5"]


def time_pass(steps, warmup):
    """One step = C1 .. C5 once each, back to back on one stream.  Returns (ms per step from the host clock, ms per
    step from HIP events, {name: average launch ms of that chain inside the timed region, from HIP events recorded
    around its launches}, {name: plan info}, {name: (algorithmic bytes, nominal bytes, label)})."""
    import numpy as np
    import torch
    from paper_2307_04995_amd import binding as pf
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
    esz = {"f32": 4, "f16": 2, "bf16": 2}
    plans, sets, infos, meta = {}, {}, {}, {}
    for name in BENCH_CHAINS:
        spec, ins, alg, nom, label = full_size_chain(name)
        plan = pf.Plan(spec, 0)
        shapes = plan.output_shapes()
        per_set = sum(t.numel() * t.element_size() for t in ins) + sum(int(np.prod(sh)) * esz[dt] for sh, (_, dt) in zip(shapes, spec.outputs))
        n_sets = max(3, min(8, -(-ROTATE_BYTES // per_set)))
        base = [t.cuda() for t in ins]
        ss = []
        for k in range(n_sets):
            i_k = [t if t.numel() * t.element_size() < 65536 else t.clone() for t in base]
            o_k = [torch.empty(sh, dtype=tdt[dt], device="cuda") for sh, (_, dt) in zip(shapes, spec.outputs)]
            ss.append((pf.PointerSet([t.data_ptr() for t in i_k], [t.data_ptr() for t in o_k]), i_k, o_k))
        plans[name], sets[name], infos[name], meta[name] = plan, ss, plan.info(), (alg, nom, label)
    import ctypes
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def one_step(k, marks=None):
        for name in BENCH_CHAINS:
            ss = sets[name]
            ps = ss[k % len(ss)][0]
            if marks is not None:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                plans[name].run_set(ps, stream)
                e1.record()
                marks[name].append((e0, e1))
            else:
                plans[name].run_set(ps, stream)

    for k in range(warmup):
        one_step(k)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for k in range(steps):
        one_step(k)
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    host_ms = (t1 - t0) * 1e3 / steps
    event_ms = ev0.elapsed_time(ev1) / steps
    # the same K steps once more with an event pair around every launch: the per-kernel durations of the timed
    # region (kept out of the first loop so that the events' own cost is not in `value`)
    marks = {name: [] for name in BENCH_CHAINS}
    for k in range(steps):
        one_step(k, marks)
    torch.cuda.synchronize()
    per_kernel = {name: sum(a.elapsed_time(b) for a, b in marks[name]) / len(marks[name]) for name in BENCH_CHAINS}
    for plan in plans.values():
        plan.close()
    del sets
    torch.cuda.empty_cache()
    return host_ms, event_ms, per_kernel, infos, meta


def cpu_baseline(budget_s=12.0):
    """The oracle as it stands, on the host cores: whole passes over the five benchmark chains at full size (the same
    work as one step), repeated until about `budget_s` seconds of CPU work."""
    import workloads as wl
    from oracle import pf_oracle as orc
    threads = orc.max_threads()
    orc.set_threads(threads)
    work, nbytes = [], 0
    for name in BENCH_CHAINS:
        spec, ins = wl.CONFIGS[name]()
        work.append((name, spec, [wl.widen(t) for t in ins]))
    nbytes = None
    per_chain = {name: 0.0 for name in BENCH_CHAINS}
    passes, total = 0, 0.0
    while total < budget_s and passes < 200:
        for name, spec, wide in work:
            t0 = time.perf_counter()
            orc.evaluate_outputs(spec, wide)
            dt = time.perf_counter() - t0
            per_chain[name] += dt
            total += dt
        passes += 1
    return {"unit": "GB/s", "cores": int(threads), "kind": "oracle", "passes": passes, "seconds": round(total, 2),
            "ms_per_chain": {name: round(per_chain[name] * 1e3 / passes, 2) for name in BENCH_CHAINS},
            "sample": f"{passes} whole passes over C1..C5 at full size (the work of {passes} steps) in {total:.1f} s, fp64 unfused, "
                      f"{threads} OpenMP threads"}


def read_traffic(name):
    """HBM bytes per launch from the committed counter summary (profiles/), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as fh:
            return json.load(fh).get(name, {}).get("traffic_bytes_per_launch")
    except (OSError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--only", default="", help="comma-separated subset of chains for the context block")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-context", action="store_true", help="time the five-chain step only")
    ap.add_argument("--hot", action="store_true",
                    help="also time every chain on ONE buffer set (cache-resident where it fits); adds launches of the "
                         "same kernels, so leave it off under a kernel trace")
    ap.add_argument("--variant", default="", help="force a kernel variant for chains of the context block, e.g. C4=1,C5=0")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (every chain shards by rows with no exchange); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)

    host_ms, event_ms, per_kernel, infos, meta = time_pass(args.steps, args.warmup)
    alg_total = sum(meta[n][0] for n in BENCH_CHAINS)
    nom_total = sum(meta[n][1] for n in BENCH_CHAINS)
    dominant = max(BENCH_CHAINS, key=lambda n: per_kernel[n])
    dom_alg = meta[dominant][0]
    # The dominant kernel's launch duration: its launches back to back on the stream between two HIP events (what a
    # kernel trace reports as its duration; an event pair around a single launch inside a step adds about 1 us of
    # dispatch gap, kept below as in_step_kernel_us).
    ctx_steps, ctx_warm = max(200, args.steps), max(20, args.warmup)   # enough launches for a 5 us kernel to time stably
    dom_spec, dom_ins, _, _, _ = full_size_chain(dominant)
    _, dom_ms, _ = time_chain(dom_spec, dom_ins, ctx_steps, ctx_warm)
    del dom_spec, dom_ins
    achieved = dom_alg / (dom_ms * 1e-3) / 1e9
    result = {
        "metric": "achieved HBM GB/s (fraction of MI355X peak) per fused chain; us per call",
        "value": round(alg_total / (host_ms * 1e-3) / 1e9, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(host_ms, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "one pass over the five BASELINE chains at full size: " + "; ".join(meta[n][2] for n in BENCH_CHAINS),
                   "storage": "fp32 (C1), fp16 (C2, C3, C5), bf16 (C4)", "bytes_per_step": alg_total, "nominal_bytes_per_step": nom_total,
                   "us_per_step": round(host_ms * 1e3, 3), "event_us_per_step": round(event_ms * 1e3, 3),
                   "buffers": "rotating sets per chain, 380 MB moved per step (cold)"},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": read_traffic(dominant),
                     "traffic_source": "profiles/hbm_traffic.json (rocprofv3 FETCH_SIZE / WRITE_SIZE runs, not measured in this run)",
                     "kernel": dominant + ": " + meta[dominant][2], "kernel_us": round(dom_ms * 1e3, 3),
                     "bytes_per_launch": dom_alg,
                     "in_step_kernel_us": {n: round(per_kernel[n] * 1e3, 3) for n in BENCH_CHAINS}},
    }
    if not args.no_context:
        chains = {}
        wanted = [c for c in (args.only.split(",") if args.only else ["C1", "C1x256", "C2", "C3", "C4", "C5", "X1", "X2", "X3", "X4", "X5", "X6", "X7"]) if c]
        forced = dict((kv.split("=")[0], int(kv.split("=")[1])) for kv in args.variant.split(",") if "=" in kv)
        for name in wanted:
            s2, i2, alg2, nom2, lab2 = full_size_chain(name)
            hot2 = [] if args.hot else None
            gr2 = [] if name == "C1" else None   # the launch-bound chain, also replayed from a HIP graph
            h2, e2, inf2 = time_chain(s2, i2, ctx_steps, ctx_warm, forced.get(name), hot=hot2, graph=gr2)
            chains[name] = {"workload": lab2, "us_per_call": round(e2 * 1e3, 3),
                            "host_us_per_call": round(h2 * 1e3, 3), "gbps": round(alg2 / (e2 * 1e-3) / 1e9, 1),
                            "frac_of_peak": round(alg2 / (e2 * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4), "bytes": alg2, "nominal_bytes": nom2,
                            "variant": inf2.variant, "spec_id": inf2.spec_id, "launches": inf2.n_launches,
                            "traffic": read_traffic(name)}
            if hot2:
                chains[name]["hot_us_per_call"] = round(hot2[0] * 1e3, 3)
            if gr2:
                chains[name]["graph_replay_us_per_call"] = round(gr2[0] * 1e3, 3)
            del s2, i2
        nbytes = 64 * 1024 * 1024
        best = None
        for variant in (1, 2, 4):
            ms = time_copy(nbytes, 100, 10, variant)
            g = 2 * nbytes / (ms * 1e-3) / 1e9
            if best is None or g > best[0]:
                best = (g, variant, ms)
        # what a launch costs before it moves anything, and what a plain copy of C1's 2.4 MB costs: the floor under
        # the launch-bound chain (a 16-byte write-only launch stands in for an empty kernel)
        small = 1184256  # bytes in (and out): C1's algorithmic 2 368 512 bytes
        chains["launch_floor"] = {"workload": "one-wave 16-byte store / plain copy 1.18 MB in + 1.18 MB out; launched from Python "
                                              "back to back, and replayed from a HIP graph (no host in the loop)",
                                  "null_us_per_call": round(time_copy(16, 400, 40, 64 | 1) * 1e3, 3),
                                  "copy_2p4MB_us_per_call": round(min(time_copy(small, 400, 40, v) for v in (1, 2)) * 1e3, 3),
                                  "null_graph_replay_us_per_call": round(time_copy(16, 640, 0, 64 | 1, graph=True) * 1e3, 3),
                                  "copy_2p4MB_graph_replay_us_per_call": round(min(time_copy(small, 640, 0, v, graph=True) for v in (1, 2)) * 1e3, 3)}
        chains["copy_probe"] = {"workload": "plain 16-byte copy, 64 MiB in + 64 MiB out", "gbps": round(best[0], 1),
                                "frac_of_peak": round(best[0] / HBM_PEAK_GBPS, 4), "us_per_call": round(best[2] * 1e3, 3),
                                "unroll": best[1]}
        result["chains"] = chains
    if not args.no_cpu:
        cb = cpu_baseline()
        cb["value"] = round(alg_total * cb["passes"] / cb["seconds"] / 1e9, 4)
        result["cpu_baseline"] = cb
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
