"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, validates descriptions,
infers shapes and maps chains to kernel families.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads as wl
from paper_2307_04995_amd import binding as pf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "pf_chain.h")).read()
    declared = set(re.findall(r"^\s*(?:pf_status|void|uint64_t|const char \*)\s*\*?(pf_[a-z_]+)\s*\(", header, flags=re.M))
    assert {"pf_chain_validate", "pf_chain_infer_shape", "pf_chain_plan", "pf_chain_plan_variant", "pf_chain_recompose",
            "pf_chain_plan_get_info", "pf_chain_run", "pf_chain_plan_poll_error", "pf_chain_plan_destroy", "pf_status_str",
            "pf_last_error", "pf_copy_probe"} <= declared
    lib = ctypes.CDLL(pf.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in pf_chain.h but not exported"
    assert set(pf.EXPORTS) == declared


def test_struct_layout_matches_header_constants():
    d = pf.make_desc(wl.c3_bias_res_layernorm(rows=8, n=64)[0])
    assert d.struct_size == ctypes.sizeof(pf.pf_chain_desc)
    assert pf.pf_chain_validate(d) == pf.PF_OK
    d.struct_size += 4
    assert pf.pf_chain_validate(d) == pf.PF_ERR_INVALID_ARG
    assert "struct_size" in pf.pf_last_error()


def test_status_strings():
    assert pf.pf_status_str(pf.PF_OK) == "PF_OK"
    assert pf.pf_status_str(pf.PF_ERR_ALIAS) == "PF_ERR_ALIAS"
    assert pf.pf_status_str(99) == "PF_ERR_UNKNOWN"


def _plan_info(spec, variant=None):
    plan = pf.Plan(spec, 0, variant)
    info = plan.info()
    shapes = plan.output_shapes()
    plan.close()
    return info, shapes


def test_benchmark_chains_map_to_their_families():
    info, shapes = _plan_info(wl.c1_bias_res_layernorm_gelu()[0])
    assert (info.family, info.variant, info.n_launches) == (pf.PF_FAMILY_ROW, pf.PF_VARIANT_ROW_BLOCK, 1)
    assert info.spec_id > 0 and list(info.block)[0] == 192 and list(info.grid)[0] == 256
    assert info.compulsory_read_bytes + info.compulsory_write_bytes == 2368512
    assert shapes == [(256, 768)]

    info, shapes = _plan_info(wl.c2_causal_softmax(b=8, h=12, s=512)[0].__class__(
        inputs=[("f16", (8, 12, 512, 512))], ops=wl.c2_causal_softmax(b=1, h=1, s=8)[0].ops,
        outputs=wl.c2_causal_softmax(b=1, h=1, s=8)[0].outputs))
    assert (info.family, info.variant) == (pf.PF_FAMILY_ROW, pf.PF_VARIANT_ROW_WAVE)
    assert info.spec_id > 0 and info.vectors_per_lane == 1
    assert info.compulsory_read_bytes + info.compulsory_write_bytes == 100663296

    spec = wl.ChainSpec(inputs=[("f16", (16384, 1024)), ("f16", (16384, 1024)), ("f16", (1024,)), ("f16", (1024,)),
                                ("f16", (1024,))])
    v = spec.op("add", 0, 2)
    v = spec.op("add", v, 1)
    v = spec.op("layernorm", v, 3, 4, f=[1e-5])
    spec.out(v, "f16")
    info, _ = _plan_info(spec)
    assert (info.family, info.variant, info.vectors_per_lane) == (pf.PF_FAMILY_ROW, pf.PF_VARIANT_ROW_WAVE, 2)
    assert info.compulsory_read_bytes + info.compulsory_write_bytes == 100669440

    spec = wl.ChainSpec(inputs=[("bf16", (32, 512, 16, 64)), ("bf16", (16, 64))])
    v = spec.op("add", 0, 1)
    v = spec.op("scale", v, f=[0.125])
    v = spec.op("permute", v, i=[0, 2, 1, 3])
    spec.out(v, "bf16")
    info, shapes = _plan_info(spec)
    assert info.family == pf.PF_FAMILY_TRANSPOSE and info.spec_id > 0
    assert shapes == [(32, 16, 512, 64)]
    assert info.compulsory_read_bytes + info.compulsory_write_bytes == 67110912
    info, _ = _plan_info(spec, variant=pf.PF_VARIANT_T_LDS_ROWS)
    assert info.variant == pf.PF_VARIANT_T_LDS_ROWS and 0 < info.lds_bytes <= 48 * 1024


def test_generic_chain_uses_interpreter():
    spec = wl.ChainSpec(inputs=[("f32", (10, 256)), ("f32", (256,))])
    v = spec.op("tanh", 0)
    v = spec.op("mul", v, 1)
    v = spec.op("softmax", v)
    v = spec.op("relu", v)
    spec.out(v, "f32")
    info, _ = _plan_info(spec)
    assert info.family == pf.PF_FAMILY_ROW and info.spec_id == 0 and info.n_micro_ops == 4


def test_infer_shape():
    spec, _ = wl.c4_bias_scale_permute(b=2, s=3, h=4, d=8)
    d = pf.make_desc(spec)
    st, t = pf.pf_chain_infer_shape(d, 4)          # the permute result
    assert st == pf.PF_OK and [t.shape[k] for k in range(t.rank)] == [2, 4, 3, 8]
    st, t = pf.pf_chain_infer_shape(d, 1)          # bias input
    assert st == pf.PF_OK and t.dtype == pf.PF_BF16 and t.rank == 2
    st, t = pf.pf_chain_infer_shape(d, 9)
    assert st == pf.PF_ERR_INVALID_ARG and t is None
    red = wl.ChainSpec(inputs=[("f32", (3, 5, 8))])
    red.out(red.op("reduce_max", 0), "f32")
    st, t = pf.pf_chain_infer_shape(pf.make_desc(red), 1)
    assert [t.shape[k] for k in range(t.rank)] == [3, 5, 1]


def _status_of(spec):
    return pf.pf_chain_validate(pf.make_desc(spec))


def test_validation_errors():
    s = wl.ChainSpec(inputs=[("f32", (4, 8)), ("f32", (4,))])
    s.out(s.op("add", 0, 1), "f32")                      # [4] is not a trailing shape of [4, 8]
    assert _status_of(s) == pf.PF_ERR_SHAPE

    s = wl.ChainSpec(inputs=[("f32", (4, 8))])
    s.ops.append(wl.OpSpec("add", (0,)))                 # wrong arity
    s.out(1, "f32")
    assert _status_of(s) == pf.PF_ERR_INVALID_ARG

    s = wl.ChainSpec(inputs=[("f32", (4, 8))])
    s.ops.append(wl.OpSpec("relu", (3,)))                # operand id in the future
    s.out(1, "f32")
    assert _status_of(s) == pf.PF_ERR_INVALID_ARG

    s = wl.ChainSpec(inputs=[("f32", (4, 8))])
    s.out(s.op("permute", 0, i=[0, 0]), "f32")
    assert _status_of(s) == pf.PF_ERR_INVALID_ARG

    s = wl.ChainSpec(inputs=[("f32", (4, 8)), ("f32", (4,)), ("f32", (8,))])
    s.out(s.op("layernorm", 0, 1, 2, f=[1e-5]), "f32")   # gamma has the wrong length
    assert _status_of(s) == pf.PF_ERR_SHAPE

    s = wl.ChainSpec(inputs=[("f32", (2, 4, 12)), ("f32", (12,)), ("f32", (12,))])
    s.out(s.op("groupnorm", 0, 1, 2, f=[1e-5], i=[5]), "f32")   # 5 does not divide 12
    assert _status_of(s) == pf.PF_ERR_INVALID_ARG

    s = wl.ChainSpec(inputs=[("f32", (4, 8))])
    s.out(s.op("reshape", 0, i=[5, 8]), "f32")
    assert _status_of(s) == pf.PF_ERR_SHAPE

    s = wl.ChainSpec(inputs=[("f32", (4, 8))])
    s.op("relu", 0)
    s.out(0, "f32")                                      # an input is not an output
    assert _status_of(s) == pf.PF_ERR_INVALID_ARG

    s = wl.ChainSpec(inputs=[("f32", (8,))])
    s.out(s.op("causal_mask", 0), "f32")
    assert _status_of(s) == pf.PF_ERR_SHAPE

    d = pf.make_desc(wl.c3_bias_res_layernorm(rows=8, n=64)[0])
    d.inputs[0].dtype = 7
    assert pf.pf_chain_validate(d) == pf.PF_ERR_DTYPE
    d = pf.make_desc(wl.c3_bias_res_layernorm(rows=8, n=64)[0])
    d.ops[2].f[0] = -1.0
    assert pf.pf_chain_validate(d) == pf.PF_ERR_INVALID_ARG


def _plan_status(spec, variant=None):
    d = pf.make_desc(spec)
    st, h = (pf.pf_chain_plan(d, 0) if variant is None else pf.pf_chain_plan_variant(d, 0, variant))
    if h is not None:
        pf.pf_chain_plan_destroy(h)
    return st


def test_plan_errors():
    # a ragged innermost extent is fine in the row and element-wise families (element-granular kernels) ...
    s = wl.ChainSpec(inputs=[("f16", (4, 12))])
    s.out(s.op("softmax", 0), "f16")
    assert _plan_status(s) == pf.PF_OK
    # ... and a channel count that is not a whole number of vectors in the pool family
    s = wl.ChainSpec(inputs=[("f16", (2, 4, 4, 12))])
    s.out(s.op("reduce_mean", 0, i=[1, 2]), "f16")
    assert _plan_status(s) == pf.PF_OK
    # two cores
    s = wl.ChainSpec(inputs=[("f16", (4, 16))])
    v = s.op("softmax", 0)
    s.out(s.op("softmax", v), "f16")
    assert _plan_status(s) == pf.PF_ERR_UNSUPPORTED
    assert "one reduce" in pf.pf_last_error()
    # mixed dtypes
    s = wl.ChainSpec(inputs=[("f16", (4, 16)), ("f32", (16,))])
    s.out(s.op("add", 0, 1), "f16")
    assert _plan_status(s) == pf.PF_ERR_DTYPE
    # a row too long for one workgroup's registers takes the streaming variant; the resident ones refuse it
    s = wl.ChainSpec(inputs=[("f32", (2, 65536))])
    s.out(s.op("softmax", 0), "f32")
    assert _plan_status(s) == pf.PF_OK
    assert _plan_status(s, pf.PF_VARIANT_ROW_BLOCK) == pf.PF_ERR_UNSUPPORTED
    # an innermost-changing permutation of 16-bit data may compute on one side only
    s = wl.ChainSpec(inputs=[("f16", (8, 64, 64))])
    v = s.op("relu", 0)
    v = s.op("permute", v, i=[0, 2, 1])
    s.out(s.op("tanh", v), "f16")
    assert _plan_status(s) == pf.PF_ERR_UNSUPPORTED
    s = wl.ChainSpec(inputs=[("f16", (8, 64, 64))])
    s.out(s.op("permute", 0, i=[0, 2, 1]), "f16")
    assert _plan_status(s) == pf.PF_OK
    # ... its transposed extents need not be whole 16-byte vectors (element-granular kernels)
    s = wl.ChainSpec(inputs=[("f16", (8, 12, 64))])
    s.out(s.op("permute", 0, i=[0, 2, 1]), "f16")
    assert _plan_status(s) == pf.PF_OK
    # ... but an innermost extent of 1 is refused
    s = wl.ChainSpec(inputs=[("f16", (8, 12, 1))])
    s.out(s.op("permute", 0, i=[1, 0, 2]), "f16")
    assert _plan_status(s) == pf.PF_ERR_UNSUPPORTED
    # a value computed before the core is used after it
    s = wl.ChainSpec(inputs=[("f32", (4, 64))])
    a = s.op("relu", 0)
    b = s.op("softmax", a)
    s.out(s.op("add", b, a), "f32")
    assert _plan_status(s) == pf.PF_ERR_UNSUPPORTED
    # forcing a variant the shape does not allow
    s = wl.ChainSpec(inputs=[("f32", (4, 8192))])
    s.out(s.op("softmax", 0), "f32")
    assert _plan_status(s, variant=pf.PF_VARIANT_ROW_WAVE) == pf.PF_ERR_UNSUPPORTED
    assert _plan_status(s) == pf.PF_OK
    # the last operator's result has to be an output
    s = wl.ChainSpec(inputs=[("f32", (4, 64))])
    a = s.op("relu", 0)
    s.op("neg", a)
    s.out(a, "f32")
    assert _plan_status(s) == pf.PF_ERR_UNSUPPORTED


def test_null_arguments_are_errors_not_crashes():
    lib = ctypes.CDLL(pf.LIB_PATH)
    lib.pf_chain_validate.argtypes = [ctypes.c_void_p]
    assert lib.pf_chain_validate(None) == pf.PF_ERR_INVALID_ARG
    lib.pf_chain_plan_get_info.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    assert lib.pf_chain_plan_get_info(None, None) == pf.PF_ERR_INVALID_ARG
    lib.pf_chain_run.argtypes = [ctypes.c_void_p] * 4
    assert lib.pf_chain_run(None, None, None, None) == pf.PF_ERR_INVALID_ARG
    lib.pf_chain_plan_destroy.argtypes = [ctypes.c_void_p]
    lib.pf_chain_plan_destroy(None)


def test_shapes_of_the_contraction_layout_and_convolution_operators():
    def shape_of(s, value):
        d = pf.make_desc(s)
        st, t = pf.pf_chain_infer_shape(d, value)
        assert st == pf.PF_OK, pf.pf_last_error()
        return tuple(t.shape[:t.rank])

    s = wl.ChainSpec(inputs=[("f16", (2, 3, 5, 8)), ("f16", (2, 3, 8)), ("f16", (2, 3, 6))])
    kc = s.op("concat_rows", 0, 1)
    mv = s.op("matvec", kc, 1)
    vm = s.op("vecmat", 2, kc)
    s.out(vm, "f16")
    assert shape_of(s, kc) == (2, 3, 6, 8) and shape_of(s, mv) == (2, 3, 6) and shape_of(s, vm) == (2, 3, 8)

    s = wl.ChainSpec(inputs=[("f32", (4, 6, 10)), ("f32", (4, 2, 10))])
    c = s.op("concat", 0, 1, i=[1])
    sl = s.op("slice", c, i=[2, 3, 4])
    s.out(sl, "f32")
    assert shape_of(s, c) == (4, 8, 10) and shape_of(s, sl) == (4, 8, 4)

    s = wl.ChainSpec(inputs=[("bf16", (1, 9, 7, 16)), ("bf16", (3, 3, 16))])
    y = s.op("dwconv2d", 0, 1)
    s.out(y, "bf16")
    assert shape_of(s, y) == (1, 9, 7, 16)

    bad = [
        (lambda s: s.op("matvec", 0, 1), [("f16", (2, 5, 8)), ("f16", (2, 7))]),
        (lambda s: s.op("vecmat", 1, 0), [("f16", (2, 5, 8)), ("f16", (2, 4))]),
        (lambda s: s.op("concat_rows", 0, 1), [("f16", (2, 5, 8)), ("f16", (3, 8))]),
        (lambda s: s.op("concat", 0, 1, i=[0]), [("f16", (2, 5)), ("f16", (2, 6))]),
        (lambda s: s.op("slice", 0, i=[1, 3, 4]), [("f16", (2, 5))]),
        (lambda s: s.op("dwconv2d", 0, 1), [("f16", (1, 4, 4, 8)), ("f16", (2, 3, 8))]),
    ]
    for make, inputs in bad:
        s = wl.ChainSpec(inputs=inputs)
        s.out(make(s), "f16")
        assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_ERR_SHAPE
    s = wl.ChainSpec(inputs=[("f16", (2, 5)), ("f16", (2, 6))])
    s.out(s.op("concat", 0, 1, i=[2]), "f16")
    assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_ERR_INVALID_ARG


def test_row_values_broadcast_over_their_rows():
    # a keep-dim reduction result may meet the full value it came from; anything else must still match exactly
    s = wl.ChainSpec(inputs=[("f32", (3, 4, 20))])
    m = s.op("reduce_max", 0)
    s.out(s.op("sub", 0, m), "f32")
    assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_OK
    s = wl.ChainSpec(inputs=[("f32", (3, 4, 20)), ("f32", (3, 5, 1))])
    s.out(s.op("sub", 0, 1), "f32")
    assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_ERR_SHAPE


def test_patterns_refused_before_any_device_work():
    # an element-wise step inside the attention pattern; arithmetic next to a concatenation
    s = wl.ChainSpec(inputs=[("f16", (1, 2, 64)), ("f16", (1, 2, 16, 64)), ("f16", (1, 2, 16, 64))])
    p = s.op("relu", s.op("softmax", s.op("matvec", 1, 0)))
    s.out(s.op("vecmat", p, 2), "f16")
    assert _plan_status(s) == pf.PF_ERR_UNSUPPORTED
    s = wl.ChainSpec(inputs=[("f16", (4, 8)), ("f16", (4, 8))])
    s.out(s.op("relu", s.op("concat", 0, 1, i=[1])), "f16")
    assert _plan_status(s) == pf.PF_ERR_UNSUPPORTED
    # a 7 x 7 depthwise kernel
    s = wl.ChainSpec(inputs=[("f16", (1, 8, 8, 16)), ("f16", (7, 7, 16))])
    s.out(s.op("dwconv2d", 0, 1), "f16")
    assert _plan_status(s) == pf.PF_ERR_UNSUPPORTED
    # a chain with in-line reductions whose rows do not fit a workgroup
    s = wl.ChainSpec(inputs=[("f32", (2, 70000))])
    m = s.op("reduce_max", 0)
    s.out(s.op("sub", 0, m), "f32")
    assert _plan_status(s) == pf.PF_ERR_UNSUPPORTED


def test_empty_and_oversized_tensors_are_refused_cleanly():
    # an extent of zero is a shape error, not an empty launch
    s = wl.ChainSpec(inputs=[("f16", (4, 0, 16))])
    s.out(s.op("relu", 0), "f16")
    assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_ERR_SHAPE
    # more rows than the row kernels index (32-bit row numbers)
    s = wl.ChainSpec(inputs=[("f16", (1 << 33, 8))])
    s.out(s.op("softmax", 0), "f16")
    assert _plan_status(s) == pf.PF_ERR_UNSUPPORTED
    assert "too large" in pf.pf_last_error()
    # more 16-byte vectors than the element-wise kernels index
    s = wl.ChainSpec(inputs=[("f32", (1 << 20, 1 << 15))])
    s.out(s.op("relu", 0), "f32")
    assert _plan_status(s) == pf.PF_ERR_UNSUPPORTED
    # a permutation of more than 2^32 elements
    s = wl.ChainSpec(inputs=[("f16", (1 << 12, 1 << 12, 1 << 9))])
    s.out(s.op("permute", 0, i=[1, 0, 2]), "f16")
    assert _plan_status(s) == pf.PF_ERR_UNSUPPORTED


def test_crafted_descriptions_cannot_wrap_a_size_or_hide_a_reduction():
    # extents whose product does not fit 64 bits (2^21 * 2^21 * 2^22 = 2^64 wraps to 0): refused when the shapes are
    # checked, before any size is computed from them
    s = wl.ChainSpec(inputs=[("f16", (1 << 21, 1 << 21, 1 << 22))])
    s.out(s.op("relu", 0), "f16")
    assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_ERR_SHAPE
    assert "2^40" in pf.pf_last_error()
    s = wl.ChainSpec(inputs=[("f32", (1 << 20, 1 << 21))])  # 2^41 elements: over the limit without wrapping anything
    s.out(s.op("relu", 0), "f32")
    assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_ERR_SHAPE
    # a reshape to extents that wrap back to the right count
    s = wl.ChainSpec(inputs=[("f16", (4, 16))])
    s.out(s.op("reshape", 0, i=[1 << 33, 1 << 33, 64]), "f16")  # 2^72 = 64 mod 2^64 ... and not 64 elements
    assert pf.pf_chain_validate(pf.make_desc(s)) == pf.PF_ERR_SHAPE
    # a negative count of integer attributes is no reduction that reduces nothing
    s = wl.ChainSpec(inputs=[("f16", (4, 16))])
    s.out(s.op("reduce_sum", 0), "f16")
    d = pf.make_desc(s)
    d.ops[0].n_i = -1
    assert pf.pf_chain_validate(d) == pf.PF_ERR_INVALID_ARG
    d.ops[0].n_i = 7
    assert pf.pf_chain_validate(d) == pf.PF_ERR_INVALID_ARG


# ---- recomposition of basic operators into composite ones (host only)

def _recompose(spec):
    st, out, changed = pf.pf_chain_recompose(pf.make_desc(spec))
    assert st == pf.PF_OK
    return pf.desc_to_spec(out), changed


def _oracle_outputs(spec, inputs):
    from oracle import pf_oracle as orc
    return orc.evaluate_outputs(spec, [wl.widen(t) for t in inputs])


def _basic_softmax(shape, scale=None, causal=False, swap_tail=None):
    s = wl.ChainSpec(inputs=[("f32", shape)])
    v = 0
    if scale is not None:
        v = s.op("scale", v, f=[scale])
    if causal:
        v = s.op("causal_mask", v)
    e = s.op("exp", s.op("sub", v, s.op("reduce_max", v)))
    y = s.op("div", e, s.op("reduce_sum", e))
    if swap_tail:
        y = s.op(swap_tail, y)
    s.out(y, "f32")
    return s


def test_recompose_softmax_keeps_the_function():
    spec = _basic_softmax((2, 5, 5), scale=0.25, causal=True, swap_tail="neg")
    new, changed = _recompose(spec)
    assert changed and [o.name for o in new.ops] == ["scale", "causal_mask", "softmax", "neg"]
    assert new.outputs == [(4, "f32")]
    x = wl.random_tensor((2, 5, 5), "f32", 3001, scale=2.0)
    a, b = _oracle_outputs(spec, [x]), _oracle_outputs(new, [x])
    np.testing.assert_allclose(a[0], b[0], rtol=0, atol=1e-15)


@pytest.mark.parametrize("order", [0, 1, 2, 3])
def test_recompose_layernorm_and_rmsnorm(order):
    rows, n = 4, 24
    ins = [("f32", (rows, n)), ("f32", (rows, n)), ("f32", (n,)), ("f32", (n,))]
    s = wl.ChainSpec(inputs=list(ins))
    h = s.op("add", 0, 1)
    c = s.op("sub", h, s.op("reduce_mean", h))
    r = s.op("rsqrt", s.op("addc", s.op("reduce_mean", s.op("mul", c, c)), f=[2.0 ** -10]))     # (exact in fp32, the type the C struct carries it in)
    y = s.op("mul", c, r) if order & 1 else s.op("mul", r, c)
    y = s.op("mul", y, 2) if order & 2 else s.op("mul", 2, y)
    y = s.op("add", y, 3) if order & 1 else s.op("add", 3, y)
    s.out(s.op("gelu_erf", y), "f32")
    s.out(h, "f32")
    new, changed = _recompose(s)
    assert changed and [o.name for o in new.ops] == ["add", "layernorm", "gelu_erf"]
    assert new.ops[1].src == (4, 2, 3) and new.ops[1].f[0] == 2.0 ** -10
    assert new.outputs == [(6, "f32"), (4, "f32")]
    inputs = [wl.random_tensor(sh, dt, 3010 + k) for k, (dt, sh) in enumerate(ins)]
    for a, b in zip(_oracle_outputs(s, inputs), _oracle_outputs(new, inputs)):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)

    s = wl.ChainSpec(inputs=[("f32", (rows, n)), ("f32", (n,))])
    r = s.op("rsqrt", s.op("addc", s.op("reduce_mean", s.op("mul", 0, 0)), f=[2.0 ** -20]))
    y = s.op("mul", 0, r) if order & 1 else s.op("mul", r, 0)
    s.out(s.op("mul", y, 1) if order & 2 else s.op("mul", 1, y), "f32")
    new, changed = _recompose(s)
    assert changed and [o.name for o in new.ops] == ["rmsnorm"] and new.ops[0].src == (0, 1)
    inputs = [wl.random_tensor((rows, n), "f32", 3020), wl.random_tensor((n,), "f32", 3021)]
    np.testing.assert_allclose(_oracle_outputs(s, inputs)[0], _oracle_outputs(new, inputs)[0], rtol=0, atol=1e-13)


def test_recompose_leaves_near_misses_alone():
    # the exponentials are also an output: an interior value is used elsewhere
    s = wl.ChainSpec(inputs=[("f32", (3, 16))])
    e = s.op("exp", s.op("sub", 0, s.op("reduce_max", 0)))
    s.out(s.op("div", e, s.op("reduce_sum", e)), "f32")
    s.out(e, "f32")
    new, changed = _recompose(s)
    assert not changed and [o.name for o in new.ops] == [o.name for o in s.ops]
    # the maximum is taken of another tensor than the one it is subtracted from
    s = wl.ChainSpec(inputs=[("f32", (3, 16)), ("f32", (3, 16))])
    e = s.op("exp", s.op("sub", 0, s.op("reduce_max", 1)))
    s.out(s.op("div", e, s.op("reduce_sum", e)), "f32")
    assert not _recompose(s)[1]
    # the divisor is the mean, not the sum
    s = wl.ChainSpec(inputs=[("f32", (3, 16))])
    e = s.op("exp", s.op("sub", 0, s.op("reduce_max", 0)))
    s.out(s.op("div", e, s.op("reduce_mean", e)), "f32")
    assert not _recompose(s)[1]
    # gamma is computed inside the chain: not a parameter the composite operator can take
    s = wl.ChainSpec(inputs=[("f32", (3, 16)), ("f32", (16,))])
    r = s.op("rsqrt", s.op("addc", s.op("reduce_mean", s.op("mul", 0, 0)), f=[1e-6]))
    s.out(s.op("mul", s.op("mul", 0, r), s.op("relu", 1)), "f32")
    assert not _recompose(s)[1]
    # the square is of another tensor than the one that gets scaled
    s = wl.ChainSpec(inputs=[("f32", (3, 16)), ("f32", (16,)), ("f32", (3, 16))])
    r = s.op("rsqrt", s.op("addc", s.op("reduce_mean", s.op("mul", 2, 2)), f=[1e-6]))
    s.out(s.op("mul", s.op("mul", 0, r), 1), "f32")
    assert not _recompose(s)[1]


def test_column_family_sizes_its_slab_to_the_column():
    """Normalisation over a strided dimension: the planner takes the fewest vectors per lane that hold the column
    (32 row groups per workgroup), from the instantiated counts 1, 2, 3, 4, 6, 8, 12, 16, 24, 32.  Host logic only."""
    want = {17: 1, 32: 1, 33: 2, 64: 2, 96: 3, 128: 4, 129: 6, 192: 6, 200: 8, 256: 8, 320: 12, 384: 12, 512: 16, 513: 24,
            768: 24, 777: 32, 1024: 32}
    for c, kc in want.items():
        s = wl.ChainSpec(inputs=[("f16", (2, c, 8, 8)), ("f16", (c,)), ("f16", (c,))])
        v = s.op("permute", 0, i=[0, 2, 3, 1])
        v = s.op("layernorm", v, 1, 2, f=[1e-6])
        s.out(s.op("permute", v, i=[0, 3, 1, 2]), "f16")
        st, h = pf.pf_chain_plan(pf.make_desc(s), 0)
        assert st == pf.PF_OK and h is not None, (c, pf.pf_last_error())
        info = pf.pf_chain_plan_get_info(h)
        pf.pf_chain_plan_destroy(h)
        assert info.family == pf.PF_FAMILY_COLUMN and info.vectors_per_lane == kc, (c, info.vectors_per_lane)
    # more values per position than the registers hold: three kernels instead (a merge plan), or a refusal
    s = wl.ChainSpec(inputs=[("f16", (2, 1025, 8, 8)), ("f16", (1025,)), ("f16", (1025,))])
    v = s.op("permute", 0, i=[0, 2, 3, 1])
    v = s.op("layernorm", v, 1, 2, f=[1e-6])
    s.out(s.op("permute", v, i=[0, 3, 1, 2]), "f16")
    st, h = pf.pf_chain_plan(pf.make_desc(s), 0)
    if h is not None:
        info = pf.pf_chain_plan_get_info(h)
        pf.pf_chain_plan_destroy(h)
        assert info.family != pf.PF_FAMILY_COLUMN or info.n_kernels > 1
