"""TEST INFRASTRUCTURE -- the unfused fp64 CPU evaluator of a chain of memory-intensive operators.

`evaluate(spec, inputs)` walks the chain operator by operator; every operator is one call into the plain C
routines of pf_oracle.c and materialises one complete float64 tensor (the unfused program whose
intermediates the fused kernels keep on chip: paper section 5.1, gOperator merging).  Nothing here is
shared with the HIP library, and nothing in the product may import this package: only tests, the smoke
check and the benchmark's CPU-baseline leg do.

`build()` compiles pf_oracle.c with gcc into oracle/libpf_oracle.so (plain C, -O2, OpenMP for the
row/group loops so the same code can be timed on one core and on all cores).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pf_oracle.c")
_LIB = os.path.join(_HERE, "libpf_oracle.so")
_lib = None

_BINARY = {"add": 0, "sub": 1, "mul": 2, "div": 3, "max": 4, "min": 5}
_UNARY = {"scale": 0, "addc": 1, "neg": 2, "relu": 3, "sigmoid": 4, "silu": 5, "gelu_erf": 6, "tanh": 7,
          "exp": 8, "rsqrt": 9}
_REDUCE = {"reduce_sum": 0, "reduce_max": 1, "reduce_mean": 2}


def build(force: bool = False) -> str:
    """Compile the C oracle.  Returns the path of the shared library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # (PF_ORACLE_LIB names another build of the same C file: the one instrumented by the host sanitizers)
        lib = ctypes.CDLL(os.environ["PF_ORACLE_LIB"]) if os.environ.get("PF_ORACLE_LIB") else ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        i64 = ctypes.c_int64
        lib.orc_set_threads.argtypes = [ctypes.c_int]
        lib.orc_max_threads.argtypes = []
        lib.orc_ew_binary.argtypes = [ctypes.c_int, dp, i64, dp, i64, dp]
        lib.orc_ew_unary.argtypes = [ctypes.c_int, dp, i64, ctypes.c_double, dp]
        lib.orc_causal_mask.argtypes = [dp, i64, i64, i64, dp]
        lib.orc_reduce_last.argtypes = [ctypes.c_int, dp, i64, i64, dp]
        lib.orc_row_broadcast_binary.argtypes = [ctypes.c_int, dp, i64, i64, dp, dp]
        lib.orc_softmax_last.argtypes = [dp, i64, i64, dp]
        lib.orc_concat_bytes.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(i64), ctypes.POINTER(i64),
                                         ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
        lib.orc_slice_bytes.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(i64), ctypes.c_int32, i64, i64,
                                        ctypes.c_int32, ctypes.c_void_p]
        lib.orc_dwconv2d_nhwc.argtypes = [dp, i64, i64, i64, i64, dp, i64, i64, i64, dp]
        lib.orc_concat_rows.argtypes = [dp, i64, i64, i64, dp, dp]
        lib.orc_matvec.argtypes = [dp, i64, i64, i64, dp, dp]
        lib.orc_vecmat.argtypes = [dp, i64, i64, i64, dp, dp]
        lib.orc_layernorm_last.argtypes = [dp, i64, i64, dp, dp, ctypes.c_double, dp]
        lib.orc_rmsnorm_last.argtypes = [dp, i64, i64, dp, ctypes.c_double, dp]
        lib.orc_groupnorm_nhwc.argtypes = [dp, i64, i64, i64, i64, dp, dp, ctypes.c_double, dp]
        lib.orc_permute_bytes.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(i64),
                                          ctypes.POINTER(ctypes.c_int32), ctypes.c_int32, ctypes.c_void_p]
        _lib = lib
    return _lib


def set_threads(n: int) -> int:
    return _load().orc_set_threads(int(n))


def max_threads() -> int:
    return _load().orc_max_threads()


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle: {what} failed with code {rc}")


def _is_trailing(small: Sequence[int], big: Sequence[int]) -> bool:
    small = tuple(small)
    while small and small[0] == 1:
        small = small[1:]
    return len(small) <= len(big) and tuple(big[len(big) - len(small):]) == small


# ---- one function per operator ---------------------------------------------------------------

def _is_row_value(small, big) -> bool:
    """`small` is `big` with the last extent collapsed to 1: what a keep-dim reduction over the last dim gives."""
    return len(small) == len(big) and small[-1] == 1 and big[-1] != 1 and tuple(small[:-1]) == tuple(big[:-1])


def broadcast_rows(v: np.ndarray, n: int) -> np.ndarray:
    """The broadcast basic operator (section 6) in the direction a reduction needs: a per-row value repeated
    over a last dimension of extent n.  Data movement only."""
    v = _f64(v)
    return np.ascontiguousarray(np.repeat(v, n, axis=-1))


def _broadcasts_onto(small, big) -> bool:
    """`small` broadcasts onto `big`: aligned at the last dimension, every extent equal or 1."""
    if len(small) > len(big):
        return False
    return all(s == g or s == 1 for s, g in zip(small, big[len(big) - len(small):]))


def broadcast_to(v: np.ndarray, shape) -> np.ndarray:
    """The broadcast basic operator (section 6) in full: align the shapes at the last dimension and repeat the
    operand along every dimension where its extent is 1 (or missing).  Data movement only; the copy is
    written out in full like every other intermediate here."""
    v = _f64(v)
    shape = tuple(shape)
    if not _broadcasts_onto(v.shape, shape):
        raise ValueError(f"oracle: cannot broadcast {v.shape} to {shape}")
    out = v.reshape((1,) * (len(shape) - v.ndim) + v.shape)
    for axis, extent in enumerate(shape):
        if out.shape[axis] != extent:
            out = np.repeat(out, extent, axis=axis)
    return np.ascontiguousarray(out)


def ew_binary(name: str, a: np.ndarray, b: np.ndarray) -> np.ndarray:
    a, b = _f64(a), _f64(b)
    if _is_row_value(b.shape, a.shape):
        b = broadcast_rows(b, a.shape[-1])
    elif _is_row_value(a.shape, b.shape):
        a = broadcast_rows(a, b.shape[-1])
    elif a.size >= b.size and not _is_trailing(b.shape, a.shape) and _broadcasts_onto(b.shape, a.shape):
        b = broadcast_to(b, a.shape)      # extents of 1 in the middle: an attention mask [B, 1, 1, S], a per-sample bias
    elif b.size > a.size and not _is_trailing(a.shape, b.shape) and _broadcasts_onto(a.shape, b.shape):
        a = broadcast_to(a, b.shape)
    if a.size > b.size or (a.size == b.size and a.ndim >= b.ndim):
        if not _is_trailing(b.shape, a.shape):
            raise ValueError(f"oracle: cannot broadcast {b.shape} over {a.shape}")
        shape = a.shape
    else:
        if not _is_trailing(a.shape, b.shape):
            raise ValueError(f"oracle: cannot broadcast {a.shape} over {b.shape}")
        shape = b.shape
    out = np.empty(shape, dtype=np.float64)
    _check(_load().orc_ew_binary(_BINARY[name], _p(a), a.size, _p(b), b.size, _p(out)), name)
    return out


def ew_unary(name: str, x: np.ndarray, alpha: float = 0.0) -> np.ndarray:
    x = _f64(x)
    out = np.empty_like(x)
    _check(_load().orc_ew_unary(_UNARY[name], _p(x), x.size, float(alpha), _p(out)), name)
    return out


def silu_decomposed(x: np.ndarray) -> np.ndarray:
    """SiLU as the two basic operators it is split into: a sigmoid, then a multiply (section 6)."""
    return ew_binary("mul", x, ew_unary("sigmoid", x))


def causal_mask(x: np.ndarray) -> np.ndarray:
    x = _f64(x)
    if x.ndim < 2:
        raise ValueError("oracle: causal_mask needs rank >= 2")
    si, sj = x.shape[-2], x.shape[-1]
    outer = x.size // (si * sj)
    out = np.empty_like(x)
    _check(_load().orc_causal_mask(_p(x), outer, si, sj, _p(out)), "causal_mask")
    return out


def reduce_last(name: str, x: np.ndarray) -> np.ndarray:
    x = _f64(x)
    n = x.shape[-1]
    rows = x.size // n
    out = np.empty(x.shape[:-1] + (1,), dtype=np.float64)
    _check(_load().orc_reduce_last(_REDUCE[name], _p(x), rows, n, _p(out)), name)
    return out


def reduce_axes(name: str, x: np.ndarray, axes) -> np.ndarray:
    """The reduce basic operator (section 6) over any set of dimensions, extents kept as 1: the reduced
    dimensions are moved behind the others (a transposition: data movement only), flattened, and reduced by the
    same routine as a reduction over the last dimension."""
    x = _f64(x)
    axes = sorted(int(a) for a in axes)
    if not axes or len(set(axes)) != len(axes) or axes[0] < 0 or axes[-1] >= x.ndim:
        raise ValueError(f"oracle: reduce axes {axes} for rank {x.ndim}")
    kept = [d for d in range(x.ndim) if d not in axes]
    moved = np.ascontiguousarray(np.transpose(x, kept + axes))
    n = int(np.prod([x.shape[d] for d in axes], dtype=np.int64))
    flat = moved.reshape(tuple(x.shape[d] for d in kept) + (n,))
    red = reduce_last(name, flat)                       # [kept..., 1]
    return np.ascontiguousarray(red.reshape(tuple(1 if d in axes else x.shape[d] for d in range(x.ndim))))


def dwconv2d_nhwc(x: np.ndarray, wgt: np.ndarray, stride: int = 1) -> np.ndarray:
    """Depthwise convolution (cross-correlation, zero padding of half the kernel extent on every side, the same
    stride along both axes) of channels-last x [n, h, w, c] with per-channel kernels wgt [kh, kw, c]
    (section 6, the EfficientNet fragment).  Stride 1 keeps the spatial size."""
    x, wgt = _f64(x), _f64(wgt)
    if x.ndim != 4 or wgt.ndim != 3 or wgt.shape[2] != x.shape[3] or stride < 1:
        raise ValueError(f"oracle: dwconv2d shapes {x.shape} and {wgt.shape}, stride {stride}")
    n, h, w, c = x.shape
    out = np.empty((n, (h - 1) // stride + 1, (w - 1) // stride + 1, c), dtype=np.float64)
    _check(_load().orc_dwconv2d_nhwc(_p(x), n, h, w, c, _p(wgt), wgt.shape[0], wgt.shape[1], int(stride), _p(out)), "dwconv2d")
    return out


def concat_rows(x: np.ndarray, r: np.ndarray) -> np.ndarray:
    """x [..., t, d] with one more row r [..., d] appended along the second-to-last axis (the cache
    concatenation of an attention layer that generates one token: section 8, GPT-2 case study)."""
    x, r = _f64(x), _f64(r)
    if x.ndim < 2 or tuple(r.shape) != tuple(x.shape[:-2]) + (x.shape[-1],):
        raise ValueError(f"oracle: concat_rows shapes {x.shape} and {r.shape}")
    t, d = x.shape[-2], x.shape[-1]
    outer = x.size // (t * d)
    out = np.empty(x.shape[:-2] + (t + 1, d), dtype=np.float64)
    _check(_load().orc_concat_rows(_p(x), outer, t, d, _p(r), _p(out)), "concat_rows")
    return out


def matvec(a: np.ndarray, x: np.ndarray) -> np.ndarray:
    """y[..., j] = sum_c a[..., j, c] * x[..., c]."""
    a, x = _f64(a), _f64(x)
    if a.ndim < 2 or tuple(x.shape) != tuple(a.shape[:-2]) + (a.shape[-1],):
        raise ValueError(f"oracle: matvec shapes {a.shape} and {x.shape}")
    t, d = a.shape[-2], a.shape[-1]
    out = np.empty(a.shape[:-1], dtype=np.float64)
    _check(_load().orc_matvec(_p(a), a.size // (t * d), t, d, _p(x), _p(out)), "matvec")
    return out


def vecmat(p: np.ndarray, a: np.ndarray) -> np.ndarray:
    """y[..., c] = sum_j p[..., j] * a[..., j, c]."""
    p, a = _f64(p), _f64(a)
    if a.ndim < 2 or tuple(p.shape) != tuple(a.shape[:-1]):
        raise ValueError(f"oracle: vecmat shapes {p.shape} and {a.shape}")
    t, d = a.shape[-2], a.shape[-1]
    out = np.empty(a.shape[:-2] + (d,), dtype=np.float64)
    _check(_load().orc_vecmat(_p(p), a.size // (t * d), t, d, _p(a), _p(out)), "vecmat")
    return out


def softmax(x: np.ndarray) -> np.ndarray:
    x = _f64(x)
    n = x.shape[-1]
    out = np.empty_like(x)
    _check(_load().orc_softmax_last(_p(x), x.size // n, n, _p(out)), "softmax")
    return out


def layernorm(x: np.ndarray, gamma, beta, eps: float) -> np.ndarray:
    x = _f64(x)
    n = x.shape[-1]
    g = None if gamma is None else _f64(gamma).reshape(-1)
    b = None if beta is None else _f64(beta).reshape(-1)
    for v in (g, b):
        if v is not None and v.size != n:
            raise ValueError("oracle: layernorm parameter size")
    out = np.empty_like(x)
    _check(_load().orc_layernorm_last(_p(x), x.size // n, n, None if g is None else _p(g),
                                      None if b is None else _p(b), float(eps), _p(out)), "layernorm")
    return out


def rmsnorm(x: np.ndarray, gamma, eps: float) -> np.ndarray:
    x = _f64(x)
    n = x.shape[-1]
    g = None if gamma is None else _f64(gamma).reshape(-1)
    if g is not None and g.size != n:
        raise ValueError("oracle: rmsnorm parameter size")
    out = np.empty_like(x)
    _check(_load().orc_rmsnorm_last(_p(x), x.size // n, n, None if g is None else _p(g), float(eps),
                                    _p(out)), "rmsnorm")
    return out


def groupnorm_nhwc(x: np.ndarray, gamma, beta, groups: int, eps: float) -> np.ndarray:
    """x is channels-last: [N, spatial..., C]."""
    x = _f64(x)
    if x.ndim < 2:
        raise ValueError("oracle: groupnorm needs rank >= 2")
    nb, c = x.shape[0], x.shape[-1]
    hw = x.size // (nb * c)
    g = None if gamma is None else _f64(gamma).reshape(-1)
    b = None if beta is None else _f64(beta).reshape(-1)
    for v in (g, b):
        if v is not None and v.size != c:
            raise ValueError("oracle: groupnorm parameter size")
    out = np.empty_like(x)
    _check(_load().orc_groupnorm_nhwc(_p(x), nb, hw, c, int(groups), None if g is None else _p(g),
                                      None if b is None else _p(b), float(eps), _p(out)), "groupnorm")
    return out


def permute(x: np.ndarray, perm: Sequence[int]) -> np.ndarray:
    """Works on any fixed-size dtype; the elements are moved as raw bytes."""
    x = np.ascontiguousarray(x)
    rank = x.ndim
    if len(perm) != rank:
        raise ValueError("oracle: permutation rank")
    shape = (ctypes.c_int64 * rank)(*x.shape)
    pm = (ctypes.c_int32 * rank)(*[int(p) for p in perm])
    out = np.empty(tuple(x.shape[p] for p in perm), dtype=x.dtype)
    _check(_load().orc_permute_bytes(x.ctypes.data, rank, shape, pm, x.dtype.itemsize, out.ctypes.data),
           "permute")
    return out


def concat(a: np.ndarray, b: np.ndarray, axis: int) -> np.ndarray:
    """Concatenation along `axis`; any fixed-size dtype, elements moved as raw bytes."""
    a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
    if a.ndim != b.ndim or a.dtype != b.dtype or not 0 <= axis < a.ndim:
        raise ValueError("oracle: concat operands")
    if any(a.shape[k] != b.shape[k] for k in range(a.ndim) if k != axis):
        raise ValueError(f"oracle: concat shapes {a.shape} and {b.shape}")
    sa = (ctypes.c_int64 * a.ndim)(*a.shape)
    sb = (ctypes.c_int64 * b.ndim)(*b.shape)
    shape = list(a.shape)
    shape[axis] += b.shape[axis]
    out = np.empty(tuple(shape), dtype=a.dtype)
    _check(_load().orc_concat_bytes(a.ctypes.data, b.ctypes.data, a.ndim, sa, sb, int(axis), a.dtype.itemsize,
                                    out.ctypes.data), "concat")
    return out


def slice_axis(x: np.ndarray, axis: int, start: int, length: int) -> np.ndarray:
    """x[..., start:start+length, ...] along `axis`; elements moved as raw bytes."""
    x = np.ascontiguousarray(x)
    if not 0 <= axis < x.ndim or start < 0 or length < 1 or start + length > x.shape[axis]:
        raise ValueError("oracle: slice range")
    sx = (ctypes.c_int64 * x.ndim)(*x.shape)
    shape = list(x.shape)
    shape[axis] = int(length)
    out = np.empty(tuple(shape), dtype=x.dtype)
    _check(_load().orc_slice_bytes(x.ctypes.data, x.ndim, sx, int(axis), int(start), int(length), x.dtype.itemsize,
                                   out.ctypes.data), "slice")
    return out


def reshape(x: np.ndarray, shape: Sequence[int]) -> np.ndarray:
    x = np.ascontiguousarray(x)
    if int(np.prod(shape, dtype=np.int64)) != x.size:
        raise ValueError("oracle: reshape size")
    return x.reshape(tuple(int(s) for s in shape)).copy()


# ---- the chain walker ------------------------------------------------------------------------

def _eval_op(op, vals: List[np.ndarray]) -> np.ndarray:
    name = op.name
    a = [vals[s] for s in op.src]
    if name in _BINARY:
        return ew_binary(name, a[0], a[1])
    if name in ("scale", "addc"):
        return ew_unary(name, a[0], op.f[0])
    if name in _UNARY:
        return ew_unary(name, a[0])
    if name == "causal_mask":
        return causal_mask(a[0])
    if name in _REDUCE:
        return reduce_axes(name, a[0], op.i) if len(op.i) else reduce_last(name, a[0])
    if name == "softmax":
        return softmax(a[0])
    if name == "dwconv2d":
        return dwconv2d_nhwc(a[0], a[1], stride=int(op.i[0]) if len(op.i) else 1)
    if name == "concat_rows":
        return concat_rows(a[0], a[1])
    if name == "matvec":
        return matvec(a[0], a[1])
    if name == "vecmat":
        return vecmat(a[0], a[1])
    if name == "layernorm":
        return layernorm(a[0], a[1], a[2], op.f[0])
    if name == "rmsnorm":
        return rmsnorm(a[0], a[1], op.f[0])
    if name == "groupnorm":
        return groupnorm_nhwc(a[0], a[1], a[2], op.i[0], op.f[0])
    if name == "permute":
        return permute(a[0], op.i)
    if name == "reshape":
        return reshape(a[0], op.i)
    if name == "concat":
        return concat(a[0], a[1], op.i[0])
    if name == "slice":
        return slice_axis(a[0], op.i[0], op.i[1], op.i[2])
    raise KeyError(f"oracle: unknown op {name}")


def evaluate(spec, inputs: Sequence[np.ndarray]) -> List[np.ndarray]:
    """Evaluate the chain on float64 inputs.  Returns every value (inputs first, then one per op); nothing is
    rounded anywhere."""
    if len(inputs) != len(spec.inputs):
        raise ValueError("oracle: wrong number of inputs")
    vals: List[np.ndarray] = []
    for (_, shape), t in zip(spec.inputs, inputs):
        arr = _f64(t)
        if tuple(arr.shape) != tuple(shape):
            raise ValueError(f"oracle: input shape {arr.shape} != declared {shape}")
        vals.append(arr)
    for op in spec.ops:
        vals.append(_eval_op(op, vals))
    return vals


def evaluate_outputs(spec, inputs: Sequence[np.ndarray]) -> List[np.ndarray]:
    vals = evaluate(spec, inputs)
    return [vals[v] for v, _ in spec.outputs]


def evaluate_layout_bits(spec, inputs_bits: Sequence[np.ndarray]) -> List[np.ndarray]:
    """Chains made only of permute / reshape, evaluated on raw bit patterns (unsigned integer arrays)."""
    vals = [np.ascontiguousarray(t) for t in inputs_bits]
    for op in spec.ops:
        if op.name == "permute":
            vals.append(permute(vals[op.src[0]], op.i))
        elif op.name == "reshape":
            vals.append(reshape(vals[op.src[0]], op.i))
        elif op.name == "concat":
            vals.append(concat(vals[op.src[0]], vals[op.src[1]], op.i[0]))
        elif op.name == "slice":
            vals.append(slice_axis(vals[op.src[0]], op.i[0], op.i[1], op.i[2]))
        else:
            raise ValueError("oracle: evaluate_layout_bits accepts only permute, reshape, concat and slice")
    return [vals[v] for v, _ in spec.outputs]
