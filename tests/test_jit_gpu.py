"""Plan-time specialisation: a chain that is not in the built-in catalogue gets a kernel instantiated for its
structure when the plan is made; chains of the same structure share it; it can be switched off."""
import pytest

import workloads as wl
from pf_testlib import check_chain, env, gpu_run, SPEC_JIT

pytestmark = pytest.mark.gpu


def _chain(rows, n, dtype, scale):
    spec = wl.ChainSpec(inputs=[(dtype, (rows, n)), (dtype, (rows, n)), (dtype, (n,))])
    v = spec.op("mul", 0, 1)
    v = spec.op("add", v, 2)
    v = spec.op("scale", v, f=[scale])
    v = spec.op("softmax", v)
    spec.out(spec.op("addc", v, f=[0.25]), dtype)
    ins = [wl.random_tensor((rows, n), dtype, 901), wl.random_tensor((rows, n), dtype, 902), wl.random_tensor((n,), dtype, 903)]
    return spec, ins


def _compile_count():
    # kernels this process made its own: compiled, or (with PF_JIT_CACHE in the environment) taken from disk
    from paper_2307_04995_amd import binding as pf
    return pf.pf_jit_compile_count() + pf.pf_jit_cache_hits()


def test_unlisted_chain_gets_its_own_kernel_and_shares_it():
    spec, ins = _chain(33, 512, "f16", 0.5)
    _, info, _ = check_chain(spec, ins, what="specialised chain")
    assert info.spec_id == SPEC_JIT
    before = _compile_count()
    # same structure and launch shape, other row count and immediates: no new compilation
    spec2, ins2 = _chain(77, 512, "f16", 0.125)
    _, info2, _ = check_chain(spec2, ins2, what="specialised chain, reused")
    assert info2.spec_id == SPEC_JIT
    assert _compile_count() == before
    # another storage type is another kernel
    spec3, ins3 = _chain(9, 512, "f32", 0.5)
    _, info3, _ = check_chain(spec3, ins3, what="specialised chain, fp32")
    assert info3.spec_id == SPEC_JIT
    assert _compile_count() == before + 1


def test_specialisation_can_be_switched_off():
    spec, ins = _chain(5, 256, "f16", 0.5)
    with env(PF_JIT="0"):
        outs, info = gpu_run(spec, ins)
    assert info.spec_id == 0


def test_elementwise_and_ragged_chains_are_specialised():
    shape = (4, 9, 30)
    x = wl.random_tensor(shape, "bf16", 911)
    b = wl.random_tensor((30,), "bf16", 912)
    spec = wl.ChainSpec(inputs=[("bf16", shape), ("bf16", (30,))])
    v = spec.op("add", 0, 1)
    spec.out(spec.op("silu", v), "bf16")
    _, info, _ = check_chain(spec, [x, b], what="ragged element-wise, specialised")
    assert info.spec_id == SPEC_JIT
    x = wl.random_tensor((6, 197), "f16", 913)
    spec = wl.ChainSpec(inputs=[("f16", (6, 197))])
    spec.out(spec.op("softmax", 0), "f16")
    _, info, _ = check_chain(spec, [x], what="ragged softmax, specialised")
    assert info.spec_id == SPEC_JIT


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_groupnorm_relu_gets_the_fused_kernel(dtype):
    # GroupNorm -> ReLU is not a catalogue entry: the fused (register-resident) kernel is specialised for it
    from paper_2307_04995_amd import binding as pf
    n, h, w, c, g = 2, 12, 12, 128, 8
    x = wl.random_tensor((n, h, w, c), dtype, 921)
    gamma = wl.random_tensor((c,), dtype, 922, dist="positive", scale=1.0)
    beta = wl.random_tensor((c,), dtype, 923, scale=0.5)
    bias = wl.random_tensor((c,), dtype, 924, scale=0.5)
    spec = wl.ChainSpec(inputs=[(dtype, (n, h, w, c)), (dtype, (c,)), (dtype, (c,)), (dtype, (c,))])
    v = spec.op("add", 0, 3)
    v = spec.op("groupnorm", v, 1, 2, f=[1e-5], i=[g])
    spec.out(spec.op("relu", v), dtype)
    _, info, _ = check_chain(spec, [x, gamma, beta, bias], what="groupnorm + relu, specialised")
    assert info.spec_id == SPEC_JIT
    assert info.variant == pf.PF_VARIANT_GROUP_RESIDENT and info.n_launches == 1
    _, info, _ = check_chain(spec, [x, gamma, beta, bias], variant=pf.PF_VARIANT_GROUP_TWO_PASS, what="groupnorm + relu, two launches")
    assert info.spec_id == SPEC_JIT and info.n_launches == 2


def test_transposes_with_unlisted_elementwise_steps():
    from paper_2307_04995_amd import binding as pf
    # innermost dimension kept
    x = wl.random_tensor((2, 24, 8, 64), "f16", 931)
    spec = wl.ChainSpec(inputs=[("f16", (2, 24, 8, 64))])
    v = spec.op("tanh", 0)
    v = spec.op("permute", v, i=[0, 2, 1, 3])
    spec.out(spec.op("scale", v, f=[0.5]), "f16")
    for variant in (pf.PF_VARIANT_T_ROWS, pf.PF_VARIANT_T_LDS_ROWS):
        _, info, _ = check_chain(spec, [x], variant=variant, what=f"tanh -> permute -> scale, variant {variant}")
        assert info.spec_id == SPEC_JIT and info.variant == variant
    # innermost dimension changed
    x = wl.random_tensor((3, 64, 128), "f32", 932)
    b = wl.random_tensor((64,), "f32", 933)
    spec = wl.ChainSpec(inputs=[("f32", (3, 64, 128)), ("f32", (64,))])
    v = spec.op("relu", 0)
    v = spec.op("permute", v, i=[0, 2, 1])
    spec.out(spec.op("add", v, 1), "f32")
    _, info, _ = check_chain(spec, [x, b], what="relu -> transpose -> + bias")
    assert info.spec_id == SPEC_JIT and info.variant == pf.PF_VARIANT_T_TILE


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("n", [197, 200, 64, 24, 100])
def test_short_rows_sit_side_by_side_in_a_wave(n, dtype):
    # rows of at most 32 vectors: 2, 4 or 8 rows share a wave (specialised kernels only); causal mask, ragged
    # widths and a row count that does not fill the last wave included
    from paper_2307_04995_amd import binding as pf
    rows_shape = (3, 5, 23, n)                      # 345 rows
    x = wl.random_tensor(rows_shape, dtype, 1500 + n, scale=2.0)
    spec = wl.ChainSpec(inputs=[(dtype, rows_shape)])
    spec.out(spec.op("softmax", spec.op("scale", 0, f=[0.25])), dtype)
    _, info, _ = check_chain(spec, [x], what=f"short-row softmax n={n} {dtype}")
    vec = 4 if dtype == "f32" else 8
    vpr = -(-n // vec)
    if vpr <= 32:
        lanes = max(8, 1 << (vpr - 1).bit_length())
        assert info.spec_id == SPEC_JIT
        # 64 / lanes rows side by side: the grid covers the 345 rows with that many rows per wave (times the
        # rows a wave holds one after the other in registers)
        waves = info.grid[0] * (info.block[0] // 64)
        assert waves * (64 // lanes) >= 345 // 4
        assert waves * (64 // lanes) <= 345 + 64
    # bias + residual + LayerNorm on the same short rows
    g = wl.random_tensor((n,), dtype, 1511, dist="positive", scale=0.8)
    b = wl.random_tensor((n,), dtype, 1512, scale=0.3)
    res = wl.random_tensor(rows_shape, dtype, 1513, scale=0.5)
    spec = wl.ChainSpec(inputs=[(dtype, rows_shape), (dtype, rows_shape), (dtype, (n,)), (dtype, (n,))])
    spec.out(spec.op("layernorm", spec.op("add", 0, 1), 2, 3, f=[1e-5]), dtype)
    check_chain(spec, [wl.random_tensor(rows_shape, dtype, 1514, scale=0.5), res, g, b], what=f"short-row layernorm n={n} {dtype}")


def test_short_causal_rows_side_by_side():
    spec, ins = wl.c2_causal_softmax(b=2, h=4, s=48, dtype="f16")      # 384 rows of 6 vectors: 8 lanes each
    _, info, _ = check_chain(spec, ins, what="short causal rows")
    assert info.spec_id == SPEC_JIT
    spec, ins = wl.c2_causal_softmax(b=1, h=3, s=100, s_k=197, dtype="bf16")
    check_chain(spec, ins, what="short ragged causal rows")


def test_a_plan_that_falls_back_to_the_interpreter_says_so(tmp_path):
    """With the kernel headers out of reach the chain cannot be specialised: the plan is still made and still right,
    but it reports that it runs on the interpreted kernels, and why."""
    from paper_2307_04995_amd import binding as pf
    # (a structure of its own, so that no kernel made for another test is waiting in the cache)
    spec = wl.ChainSpec(inputs=[("f16", (21, 384)), ("f16", (384,))])
    spec.out(spec.op("neg", spec.op("softmax", spec.op("tanh", spec.op("sub", 0, 1)))), "f16")
    ins = [wl.random_tensor((21, 384), "f16", 911), wl.random_tensor((384,), "f16", 912)]
    with env(PF_JIT_INCLUDE=str(tmp_path)):
        plan = pf.Plan(spec, 0)
        reason = pf.pf_last_error()
        info = plan.info()
        plan.close()
        assert info.spec_id == 0 and info.interpreter_fallback == 1
        assert "headers not found" in reason
        check_chain(spec, ins, what="interpreter fallback")
    # a passing condition is not remembered: with the headers back, the same chain gets its kernel
    _, info2, _ = check_chain(spec, ins, what="specialised after the headers came back")
    assert info2.spec_id == SPEC_JIT and info2.interpreter_fallback == 0
    # asking for the interpreter is no fallback
    with env(PF_JIT="0"):
        _, info3 = gpu_run(spec, ins)
    assert info3.spec_id == 0 and info3.interpreter_fallback == 0


def _shape_const_cases():
    cases = []
    cases.append(("C1 block variant, rows not a whole workgroup count", lambda: wl.c1_bias_res_layernorm_gelu(rows=37, n=768, dtype="f32")))
    cases.append(("C1 two waves per row", lambda: wl.c1_bias_res_layernorm_gelu(rows=21, n=1024, dtype="f16")))
    cases.append(("C2 causal, two rows per wave", lambda: wl.c2_causal_softmax(b=2, h=3, s=512, dtype="f16")))
    cases.append(("C2 causal, rectangular scores", lambda: wl.c2_causal_softmax(b=1, h=2, s=40, dtype="f16", s_k=256)))
    cases.append(("C2 causal bf16, odd row count", lambda: wl.c2_causal_softmax(b=1, h=3, s=24, dtype="bf16", s_k=128)))
    cases.append(("C3 wave per row", lambda: wl.c3_bias_res_layernorm(rows=131, n=1024, dtype="f16")))
    cases.append(("C3 rows that do not fill the lanes", lambda: wl.c3_bias_res_layernorm(rows=50, n=640, dtype="bf16")))
    cases.append(("C3 ragged row length", lambda: wl.c3_bias_res_layernorm(rows=33, n=197, dtype="f16")))
    cases.append(("short rows side by side", lambda: wl.c3_bias_res_layernorm(rows=300, n=128, dtype="f16")))
    return cases


@pytest.mark.parametrize("idx", range(9))
def test_row_kernels_compiled_for_their_shape(idx):
    # the shape-constant form is planned by itself for tensors of half a megabyte and more; forced here on small ones
    what, make = _shape_const_cases()[idx]
    spec, ins = make()
    with env(PF_ROW_CONST="2"):
        outs, info, _ = check_chain(spec, ins, what=what + ", shape as constants")
    assert info.spec_id == SPEC_JIT
    with env(PF_ROW_CONST="0"):
        plain, _ = gpu_run(spec, ins)
    # (not bit for bit: with constants in place of arguments the compiler contracts other multiply-adds)
    diff = (outs[0].double() - plain[0].double()).abs().max().item()
    assert diff <= (4e-6 if spec.outputs[0][1] == "f32" else 8e-3), f"the shape-constant kernel and the run-time one disagree by {diff}"


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape,perm", [((3, 24, 16, 64), (0, 2, 1, 3)), ((6, 5, 32), (1, 0, 2)), ((2, 3, 4, 5, 16), (3, 0, 2, 1, 4)),
                                        ((5, 12, 6, 64), (0, 2, 1, 3)), ((40, 24, 8), (1, 0, 2))])
def test_permutation_kernels_compiled_for_their_geometry(shape, perm, dtype):
    # planned by itself for tensors of 16 MB and more (full-size C4); forced here on small ones: a bias in front of the
    # permutation, a full-shape operand and a bias behind it, every index of both layouts in play
    import numpy as np
    out_shape = tuple(shape[i] for i in perm)
    x = wl.random_tensor(shape, dtype, 2101)
    b_in = wl.random_tensor(shape[-2:], dtype, 2102, scale=0.5)
    res = wl.random_tensor(out_shape, dtype, 2103, scale=0.5)
    b_out = wl.random_tensor((out_shape[-1],), dtype, 2104, scale=0.5)
    s = wl.ChainSpec(inputs=[(dtype, shape), (dtype, tuple(shape[-2:])), (dtype, out_shape), (dtype, (out_shape[-1],))])
    v = s.op("scale", s.op("add", 0, 1), f=[0.125])
    v = s.op("permute", v, i=list(perm))
    v = s.op("add", s.op("add", v, 2), 3)
    s.out(v, dtype)
    with env(PF_PERM_CONST="2"):
        outs, info, _ = check_chain(s, [x, b_in, res, b_out], what=f"permutation {perm} of {shape} {dtype}, geometry as constants")
    assert info.spec_id == SPEC_JIT and info.vectors_per_lane == 8
    with env(PF_PERM_CONST="0"):
        plain, info0 = gpu_run(s, [x, b_in, res, b_out])
    assert info0.vectors_per_lane <= 2
    import torch
    assert torch.equal(outs[0], plain[0])
    # layout only: the raw bits travel
    lay = wl.ChainSpec(inputs=[(dtype, shape)])
    lay.out(lay.op("permute", 0, i=list(perm)), dtype)
    with env(PF_PERM_CONST="2"):
        (moved,), _ = gpu_run(lay, [x])
    assert torch.equal(moved, x.permute(*perm).contiguous())


_DISK_CACHE_SCRIPT = r"""
import hashlib, sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {root!r} + "/tests")
import torch
import workloads as wl
from paper_2307_04995_amd import binding as pf
# (a structure of its own: nothing in the catalogue, nothing another test compiles)
spec = wl.ChainSpec(inputs=[("f16", (37, 264)), ("f16", (264,))])
spec.out(spec.op("sigmoid", spec.op("softmax", spec.op("silu", spec.op("mul", 0, 1)))), "f16")
ins = [wl.random_tensor((37, 264), "f16", 931).cuda(), wl.random_tensor((264,), "f16", 932).cuda()]
out = torch.empty((37, 264), dtype=torch.float16, device="cuda")
plan = pf.Plan(spec, 0)
info = plan.info()
plan.run(ins, [out])
torch.cuda.synchronize()
plan.close()
digest = hashlib.sha256(out.cpu().numpy().tobytes()).hexdigest()
print("RESULT", pf.pf_jit_compile_count(), pf.pf_jit_cache_hits(), info.spec_id, digest)
"""


def test_kernels_kept_on_disk_are_loaded_by_the_next_process(tmp_path):
    """PF_JIT_CACHE: the first process compiles and keeps the kernel, the second loads it and computes the same bits; a
    file that does not load is compiled over."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    script = _DISK_CACHE_SCRIPT.format(root=root)
    child_env = dict(os.environ, PF_JIT_CACHE=str(tmp_path))

    def run():
        r = subprocess.run([sys.executable, "-c", script], env=child_env, capture_output=True, text=True, timeout=110)
        assert r.returncode == 0, r.stderr[-2000:]
        line = [l for l in r.stdout.splitlines() if l.startswith("RESULT")][-1].split()
        return int(line[1]), int(line[2]), int(line[3]), line[4]

    compiles, hits, spec_id, first = run()
    assert compiles >= 1 and hits == 0 and spec_id == SPEC_JIT
    files = sorted(p for p in os.listdir(tmp_path) if p.endswith(".co"))
    assert len(files) == compiles and not [p for p in os.listdir(tmp_path) if p.endswith(".tmp")]
    compiles2, hits2, spec_id2, second = run()
    assert compiles2 == 0 and hits2 == compiles and spec_id2 == SPEC_JIT and second == first
    # a damaged file is no obstacle
    for name in files:
        with open(os.path.join(tmp_path, name), "r+b") as fh:
            fh.truncate(100)
    compiles3, hits3, _, third = run()
    assert compiles3 == compiles and hits3 == 0 and third == first
