"""ctypes binding of include/pf_chain.h -- argument marshalling only.

The functions below carry the names of the C ABI and pass their arguments straight through; everything a
chain computes is computed by the HIP kernels behind `pf_chain_run`.  PyTorch appears only as the owner of
device memory and streams.  If the shared library has not been built the import of this module fails
loudly: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

PF_CHAIN_VERSION = 1
PF_MAX_RANK = 6
PF_MAX_INPUTS = 8
PF_MAX_OPS = 32
PF_MAX_OUTPUTS = 3

# pf_status
PF_OK, PF_ERR_INVALID_ARG, PF_ERR_SHAPE, PF_ERR_DTYPE, PF_ERR_UNSUPPORTED, PF_ERR_ALIGNMENT, PF_ERR_ALIAS, \
    PF_ERR_NOMEM, PF_ERR_HIP = range(9)
# pf_dtype
PF_F32, PF_F16, PF_BF16 = range(3)
DTYPE_CODE = {"f32": PF_F32, "f16": PF_F16, "bf16": PF_BF16}
# pf_op
OP_CODE = {name: i for i, name in enumerate([
    "add", "sub", "mul", "div", "max", "min", "scale", "addc", "neg", "relu", "sigmoid", "silu", "gelu_erf",
    "tanh", "exp", "rsqrt", "causal_mask", "reduce_sum", "reduce_max", "reduce_mean", "softmax", "layernorm",
    "rmsnorm", "groupnorm", "permute", "reshape", "concat_rows", "matvec", "vecmat", "concat", "slice", "dwconv2d"])}
# pf_family
PF_FAMILY_ELEMENTWISE, PF_FAMILY_ROW, PF_FAMILY_GROUP, PF_FAMILY_TRANSPOSE, PF_FAMILY_ATTENTION, PF_FAMILY_GATHER, PF_FAMILY_STENCIL, PF_FAMILY_POOL, PF_FAMILY_COLUMN = range(9)
PF_VARIANT_ROW_WAVE, PF_VARIANT_ROW_BLOCK, PF_VARIANT_ROW_STREAM = 0, 1, 2
PF_SPEC_GENERIC, PF_SPEC_JIT = 0, 255
PF_VARIANT_STENCIL_DIRECT, PF_VARIANT_STENCIL_STAGED, PF_VARIANT_STENCIL_STRIDED = 0, 1, 2
PF_VARIANT_ATTN_ONE_PASS, PF_VARIANT_ATTN_STREAM = 0, 1
PF_VARIANT_GROUP_TWO_PASS, PF_VARIANT_GROUP_RESIDENT = 0, 1
PF_VARIANT_T_ROWS, PF_VARIANT_T_LDS_ROWS, PF_VARIANT_T_TILE = 0, 1, 2


class pf_tensor_desc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("rank", C.c_int32), ("shape", C.c_int64 * PF_MAX_RANK)]


class pf_op_desc(C.Structure):
    _fields_ = [("op", C.c_int32), ("n_src", C.c_int32), ("src", C.c_int32 * 3), ("f", C.c_float * 2),
                ("i", C.c_int64 * PF_MAX_RANK), ("n_i", C.c_int32)]


class pf_chain_desc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("version", C.c_uint32),
                ("n_inputs", C.c_int32), ("inputs", pf_tensor_desc * PF_MAX_INPUTS),
                ("n_ops", C.c_int32), ("ops", pf_op_desc * PF_MAX_OPS),
                ("n_outputs", C.c_int32), ("out_value", C.c_int32 * PF_MAX_OUTPUTS),
                ("out_dtype", C.c_int32 * PF_MAX_OUTPUTS)]


class pf_plan_info(C.Structure):
    _fields_ = [("family", C.c_int32), ("variant", C.c_int32), ("grid", C.c_uint32 * 3), ("block", C.c_uint32 * 3),
                ("lds_bytes", C.c_uint32), ("workspace_bytes", C.c_uint64),
                ("compulsory_read_bytes", C.c_uint64), ("compulsory_write_bytes", C.c_uint64),
                ("n_launches", C.c_int32), ("n_micro_ops", C.c_int32), ("spec_id", C.c_int32),
                ("vectors_per_lane", C.c_int32), ("n_kernels", C.c_int32), ("interpreter_fallback", C.c_int32)]


class pf_partition(C.Structure):
    _fields_ = [("n_parts", C.c_int32), ("first_op", C.c_int32 * (PF_MAX_OPS + 1)),
                ("predicted_us", C.c_double * PF_MAX_OPS), ("bytes", C.c_uint64 * PF_MAX_OPS)]


# (PF_CHAIN_LIB names another build of the same library: the one with sanitized host code, see build.py --sanitize)
LIB_PATH = os.environ.get("PF_CHAIN_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libpf_chain.so")
EXPORTS = ["pf_chain_validate", "pf_chain_infer_shape", "pf_chain_plan", "pf_chain_plan_variant",
           "pf_chain_plan_get_info", "pf_chain_run", "pf_chain_plan_poll_error", "pf_chain_plan_destroy", "pf_status_str",
           "pf_last_error", "pf_copy_probe", "pf_jit_compile_count", "pf_jit_cache_hits", "pf_chain_recompose",
           "pf_chain_partition", "pf_chain_segment_cost", "pf_chain_plan_get_partition", "pf_chain_run_static"]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
            "There is no fallback path.")
    lib = C.CDLL(LIB_PATH)
    vp = C.c_void_p
    lib.pf_chain_validate.argtypes = [C.POINTER(pf_chain_desc)]
    lib.pf_chain_infer_shape.argtypes = [C.POINTER(pf_chain_desc), C.c_int32, C.POINTER(pf_tensor_desc)]
    lib.pf_chain_plan.argtypes = [C.POINTER(pf_chain_desc), C.c_int32, C.POINTER(vp)]
    lib.pf_chain_plan_variant.argtypes = [C.POINTER(pf_chain_desc), C.c_int32, C.c_int32, C.POINTER(vp)]
    lib.pf_chain_plan_get_info.argtypes = [vp, C.POINTER(pf_plan_info)]
    lib.pf_chain_run.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp]
    lib.pf_chain_run_static.argtypes = [C.POINTER(pf_chain_desc), C.c_int32, C.POINTER(vp), C.POINTER(vp), vp]
    lib.pf_chain_plan_poll_error.argtypes = [vp, C.POINTER(C.c_int32)]
    lib.pf_chain_plan_destroy.argtypes = [vp]
    lib.pf_chain_plan_destroy.restype = None
    lib.pf_status_str.argtypes = [C.c_int]
    lib.pf_status_str.restype = C.c_char_p
    lib.pf_last_error.argtypes = []
    lib.pf_last_error.restype = C.c_char_p
    lib.pf_copy_probe.argtypes = [vp, vp, C.c_uint64, C.c_int32, vp]
    lib.pf_chain_recompose.argtypes = [C.POINTER(pf_chain_desc), C.POINTER(pf_chain_desc), C.POINTER(C.c_int32)]
    lib.pf_chain_partition.argtypes = [C.POINTER(pf_chain_desc), C.POINTER(pf_partition)]
    lib.pf_chain_plan_get_partition.argtypes = [vp, C.POINTER(pf_partition)]
    lib.pf_chain_segment_cost.argtypes = [C.POINTER(pf_chain_desc), C.c_int32, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]
    lib.pf_jit_compile_count.argtypes = []
    lib.pf_jit_compile_count.restype = C.c_uint64
    lib.pf_jit_cache_hits.argtypes = []
    lib.pf_jit_cache_hits.restype = C.c_uint64
    for name in EXPORTS:
        if name not in ("pf_chain_plan_destroy", "pf_status_str", "pf_last_error", "pf_jit_compile_count", "pf_jit_cache_hits"):
            getattr(lib, name).restype = C.c_int
    return lib


_lib = _load()


class PfError(RuntimeError):
    def __init__(self, status: int, detail: str):
        self.status = status
        self.detail = detail
        super().__init__(f"{pf_status_str(status)}: {detail}")


# ---- the C ABI, same names ---------------------------------------------------------------------

def pf_status_str(status: int) -> str:
    return _lib.pf_status_str(int(status)).decode()


def pf_last_error() -> str:
    return _lib.pf_last_error().decode()


def pf_chain_validate(desc: pf_chain_desc) -> int:
    return _lib.pf_chain_validate(C.byref(desc))


def pf_chain_infer_shape(desc: pf_chain_desc, value: int):
    """Returns (status, pf_tensor_desc or None)."""
    out = pf_tensor_desc()
    st = _lib.pf_chain_infer_shape(C.byref(desc), int(value), C.byref(out))
    return st, (out if st == PF_OK else None)


def pf_chain_plan(desc: pf_chain_desc, device: int = 0):
    """Returns (status, plan handle or None)."""
    handle = C.c_void_p()
    st = _lib.pf_chain_plan(C.byref(desc), int(device), C.byref(handle))
    return st, (handle if st == PF_OK else None)


def pf_chain_plan_variant(desc: pf_chain_desc, device: int, variant: int):
    handle = C.c_void_p()
    st = _lib.pf_chain_plan_variant(C.byref(desc), int(device), int(variant), C.byref(handle))
    return st, (handle if st == PF_OK else None)


def pf_chain_plan_get_info(plan) -> pf_plan_info:
    info = pf_plan_info()
    st = _lib.pf_chain_plan_get_info(plan, C.byref(info))
    if st != PF_OK:
        raise PfError(st, pf_last_error())
    return info


def pf_chain_run(plan, input_ptrs: Sequence[int], output_ptrs: Sequence[int], stream: int = 0) -> int:
    ins = (C.c_void_p * len(input_ptrs))(*[C.c_void_p(int(p)) for p in input_ptrs])
    outs = (C.c_void_p * len(output_ptrs))(*[C.c_void_p(int(p)) for p in output_ptrs])
    return _lib.pf_chain_run(plan, ins, outs, C.c_void_p(int(stream)))


class PointerSet:
    """The pointer arrays of one call of pf_chain_run, marshalled once: a caller that launches the same buffers again
    and again (a serving loop, a benchmark) passes this instead of two Python sequences, and the call then costs one
    foreign-function call instead of rebuilding two arrays."""

    __slots__ = ("ins", "outs")

    def __init__(self, input_ptrs: Sequence[int], output_ptrs: Sequence[int]):
        self.ins = (C.c_void_p * len(input_ptrs))(*[C.c_void_p(int(p)) for p in input_ptrs])
        self.outs = (C.c_void_p * len(output_ptrs))(*[C.c_void_p(int(p)) for p in output_ptrs])


def pf_chain_run_set(plan, ptrs: PointerSet, stream) -> int:
    """pf_chain_run on pointer arrays marshalled beforehand; `stream` is a ctypes.c_void_p (or None)."""
    return _lib.pf_chain_run(plan, ptrs.ins, ptrs.outs, stream)


PF_STATIC_SCRATCH_BYTES = 2 << 20


def pf_chain_run_static(desc: pf_chain_desc, device: int, input_ptrs: Sequence[int], output_ptrs: Sequence[int], stream: int = 0) -> int:
    ins = (C.c_void_p * len(input_ptrs))(*[C.c_void_p(int(p)) for p in input_ptrs])
    outs = (C.c_void_p * len(output_ptrs))(*[C.c_void_p(int(p)) for p in output_ptrs])
    return _lib.pf_chain_run_static(C.byref(desc), int(device), ins, outs, C.c_void_p(int(stream)))


def pf_chain_plan_poll_error(plan):
    """Returns (status, flag)."""
    flag = C.c_int32(0)
    st = _lib.pf_chain_plan_poll_error(plan, C.byref(flag))
    return st, flag.value


def pf_chain_plan_destroy(plan) -> None:
    _lib.pf_chain_plan_destroy(plan)


def pf_copy_probe(src_ptr: int, dst_ptr: int, nbytes: int, variant: int = 2, stream: int = 0) -> int:
    return _lib.pf_copy_probe(C.c_void_p(int(src_ptr)), C.c_void_p(int(dst_ptr)), C.c_uint64(int(nbytes)),
                              C.c_int32(int(variant)), C.c_void_p(int(stream)))


def pf_chain_recompose(desc: pf_chain_desc):
    """(status, rewritten desc or None, changed)."""
    out = pf_chain_desc()
    changed = C.c_int32(0)
    st = _lib.pf_chain_recompose(C.byref(desc), C.byref(out), C.byref(changed))
    return st, (out if st == PF_OK else None), bool(changed.value)


def pf_chain_partition(desc: pf_chain_desc):
    """(status, [(first_op, last_op, predicted_us, bytes), ...]) of the cheapest split into kernels."""
    out = pf_partition()
    st = _lib.pf_chain_partition(C.byref(desc), C.byref(out))
    if st != PF_OK:
        return st, None
    return st, [(out.first_op[k], out.first_op[k + 1], out.predicted_us[k], out.bytes[k]) for k in range(out.n_parts)]


def pf_chain_segment_cost(desc: pf_chain_desc, first_op: int, last_op: int):
    """(status, predicted_us, bytes) of operators first_op .. last_op - 1 run as one kernel."""
    us = C.c_double(0.0)
    nbytes = C.c_uint64(0)
    st = _lib.pf_chain_segment_cost(C.byref(desc), C.c_int32(first_op), C.c_int32(last_op), C.byref(us), C.byref(nbytes))
    return st, us.value, nbytes.value


def pf_jit_compile_count() -> int:
    return int(_lib.pf_jit_compile_count())


def pf_jit_cache_hits() -> int:
    return int(_lib.pf_jit_cache_hits())


# ---- marshalling helpers -------------------------------------------------------------------------

def make_desc(spec) -> pf_chain_desc:
    """Chain description object (inputs / ops / outputs attributes) -> C struct.  No checking here: that
    is pf_chain_validate's job."""
    d = pf_chain_desc()
    d.struct_size = C.sizeof(pf_chain_desc)
    d.version = PF_CHAIN_VERSION
    d.n_inputs = len(spec.inputs)
    for k, (dt, shape) in enumerate(spec.inputs[:PF_MAX_INPUTS]):
        d.inputs[k].dtype = DTYPE_CODE[dt]
        d.inputs[k].rank = len(shape)
        for j, e in enumerate(shape[:PF_MAX_RANK]):
            d.inputs[k].shape[j] = int(e)
    d.n_ops = len(spec.ops)
    for k, op in enumerate(spec.ops[:PF_MAX_OPS]):
        o = d.ops[k]
        o.op = OP_CODE[op.name]
        o.n_src = len(op.src)
        for j, s in enumerate(op.src[:3]):
            o.src[j] = int(s)
        for j, f in enumerate(op.f[:2]):
            o.f[j] = float(f)
        o.n_i = len(op.i)
        for j, i in enumerate(op.i[:PF_MAX_RANK]):
            o.i[j] = int(i)
    d.n_outputs = len(spec.outputs)
    for k, (v, dt) in enumerate(spec.outputs[:PF_MAX_OUTPUTS]):
        d.out_value[k] = int(v)
        d.out_dtype[k] = DTYPE_CODE[dt]
    return d


def desc_to_spec(d: pf_chain_desc):
    """C struct -> workloads.ChainSpec (the inverse of make_desc)."""
    import workloads as wl
    names = {v: k for k, v in OP_CODE.items()}
    dts = {v: k for k, v in DTYPE_CODE.items()}
    spec = wl.ChainSpec(inputs=[(dts[d.inputs[k].dtype], tuple(d.inputs[k].shape[j] for j in range(d.inputs[k].rank)))
                                for k in range(d.n_inputs)])
    for k in range(d.n_ops):
        o = d.ops[k]
        spec.ops.append(wl.OpSpec(names[o.op], tuple(o.src[j] for j in range(o.n_src)), (o.f[0], o.f[1]),
                                  tuple(o.i[j] for j in range(o.n_i))))
    for k in range(d.n_outputs):
        spec.out(d.out_value[k], dts[d.out_dtype[k]])
    return spec


class Plan:
    """Owns a plan handle; releases it on garbage collection."""

    def __init__(self, spec_or_desc, device: int = 0, variant: Optional[int] = None):
        self.desc = spec_or_desc if isinstance(spec_or_desc, pf_chain_desc) else make_desc(spec_or_desc)
        if variant is None:
            st, handle = pf_chain_plan(self.desc, device)
        else:
            st, handle = pf_chain_plan_variant(self.desc, device, variant)
        if st != PF_OK:
            raise PfError(st, pf_last_error())
        self.handle = handle
        self.device = device

    def info(self) -> pf_plan_info:
        return pf_chain_plan_get_info(self.handle)

    def partition(self):
        """[(first_op, last_op, predicted_us, bytes), ...] of the kernels this plan runs."""
        out = pf_partition()
        st = _lib.pf_chain_plan_get_partition(self.handle, C.byref(out))
        if st != PF_OK:
            raise PfError(st, pf_last_error())
        return [(out.first_op[k], out.first_op[k + 1], out.predicted_us[k], out.bytes[k]) for k in range(out.n_parts)]

    def output_shapes(self) -> List[tuple]:
        shapes = []
        for k in range(self.desc.n_outputs):
            st, t = pf_chain_infer_shape(self.desc, self.desc.out_value[k])
            if st != PF_OK:
                raise PfError(st, pf_last_error())
            shapes.append(tuple(t.shape[j] for j in range(t.rank)))
        return shapes

    def run_ptrs(self, input_ptrs: Sequence[int], output_ptrs: Sequence[int], stream: int = 0) -> None:
        st = pf_chain_run(self.handle, input_ptrs, output_ptrs, stream)
        if st != PF_OK:
            raise PfError(st, pf_last_error())

    def run_set(self, ptrs: "PointerSet", stream: "C.c_void_p") -> None:
        """run_ptrs on a PointerSet built beforehand; `stream` as ctypes.c_void_p (also built beforehand)."""
        st = _lib.pf_chain_run(self.handle, ptrs.ins, ptrs.outs, stream)
        if st != PF_OK:
            raise PfError(st, pf_last_error())

    def run(self, inputs, outputs, stream=None) -> None:
        """inputs / outputs: torch CUDA tensors (contiguous).  Launches on torch's current stream unless a
        raw stream handle is given."""
        import torch
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        for t in list(inputs) + list(outputs):
            if not t.is_cuda or not t.is_contiguous():
                raise ValueError("tensors must be contiguous device tensors")
        self.run_ptrs([t.data_ptr() for t in inputs], [t.data_ptr() for t in outputs], stream)

    def poll_error(self) -> int:
        st, flag = pf_chain_plan_poll_error(self.handle)
        if st != PF_OK:
            raise PfError(st, pf_last_error())
        return flag

    def close(self) -> None:
        if getattr(self, "handle", None) is not None:
            pf_chain_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def run_chain(spec, inputs, device: int = 0, variant: Optional[int] = None):
    """Plan, allocate outputs with torch, run once.  Returns the list of output tensors."""
    import torch
    plan = Plan(spec, device, variant)
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
    outs = [torch.empty(shape, dtype=tdt[dt], device=f"cuda:{device}")
            for shape, (_, dt) in zip(plan.output_shapes(), spec.outputs)]
    plan.run(inputs, outs)
    torch.cuda.synchronize(device)
    plan.close()
    return outs
