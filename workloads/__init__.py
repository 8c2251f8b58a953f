"""Chain descriptions and seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds *no arithmetic of the method*: it only says which operators a chain consists of
(names, operand ids, attributes), draws the random input tensors and quantises them to their storage
dtype.  The CPU oracle and the HIP library each interpret a :class:`ChainSpec` with code of their own.

Chain vocabulary: the four basic operator kinds a memory-intensive subgraph is split into
(element-wise, broadcast, reduce, transpose; paper section 6, "GIR-Graph generation"), with the
composite operators (softmax, the normalisations, SiLU, GELU) kept as named ops as well, so a chain can
be written either way.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np
import torch

DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}

# op name -> number of operands.  Binary element-wise ops broadcast a lower-rank operand over the
# leading dimensions of the other one (its shape must equal the trailing dimensions).
OP_ARITY: Dict[str, int] = {
    "add": 2, "sub": 2, "mul": 2, "div": 2, "max": 2, "min": 2,
    "scale": 1, "addc": 1, "neg": 1, "relu": 1, "sigmoid": 1, "silu": 1, "gelu_erf": 1,
    "tanh": 1, "exp": 1, "rsqrt": 1,
    "causal_mask": 1,
    "reduce_sum": 1, "reduce_max": 1, "reduce_mean": 1,
    "softmax": 1, "layernorm": 3, "rmsnorm": 2, "groupnorm": 3,
    "permute": 1, "reshape": 1,
    # one-token attention against cached keys / values: append a row, matrix-vector, vector-matrix
    "concat_rows": 2, "matvec": 2, "vecmat": 2,
    # layout: concatenation along axis i[0]; slice [i[1], i[1] + i[2]) along axis i[0]
    "concat": 2, "slice": 1,
    # depthwise convolution of channels-last x [n, h, w, c] with kernels [kh, kw, c], stride 1, "same" zero padding
    "dwconv2d": 2,
}


@dataclass
class OpSpec:
    name: str
    src: Tuple[int, ...]               # value ids: 0..n_inputs-1 are inputs, n_inputs+k is the result of op k
    f: Tuple[float, ...] = ()          # float attributes (scale factor, constant, eps)
    i: Tuple[int, ...] = ()            # integer attributes (permutation, new shape, group count)


@dataclass
class ChainSpec:
    inputs: List[Tuple[str, Tuple[int, ...]]]          # (dtype name, shape) per input, contiguous row-major
    ops: List[OpSpec] = field(default_factory=list)
    outputs: List[Tuple[int, str]] = field(default_factory=list)   # (value id, dtype name)

    # small builder helpers (bookkeeping only)
    def op(self, name: str, *src: int, f: Sequence[float] = (), i: Sequence[int] = ()) -> int:
        if name not in OP_ARITY:
            raise KeyError(name)
        self.ops.append(OpSpec(name, tuple(int(s) for s in src), tuple(float(x) for x in f),
                               tuple(int(x) for x in i)))
        return len(self.inputs) + len(self.ops) - 1

    def out(self, value: int, dtype: str) -> None:
        self.outputs.append((int(value), dtype))


def quantise(x: np.ndarray, dtype: str) -> torch.Tensor:
    """fp32 numpy array -> contiguous CPU torch tensor in the storage dtype (round to nearest even)."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(DTYPES[dtype]).contiguous()


def widen(t: torch.Tensor) -> np.ndarray:
    """Storage-dtype tensor (CPU) -> float64 numpy array holding exactly the same values."""
    return t.detach().cpu().to(torch.float64).numpy()


def raw_bits(t: torch.Tensor) -> np.ndarray:
    """Bit pattern of a tensor as an unsigned integer array of the same shape (for layout-only checks)."""
    t = t.detach().cpu().contiguous()
    view = {2: torch.int16, 4: torch.int32}[t.element_size()]
    udt = {2: np.uint16, 4: np.uint32}[t.element_size()]
    return t.view(view).numpy().view(udt)


BASE_SEED = 20230704


def _rng(k: int, salt: int = 0) -> np.random.Generator:
    return np.random.default_rng(BASE_SEED + k + 1000 * salt)


# ---------------------------------------------------------------------------------------------
# The five benchmark chains.  Every builder takes the sizes as arguments so the parity tests can run
# the same chain at sizes the oracle finishes in seconds; the defaults are the full sizes.
# Tensors are drawn in the order they are listed, as fp32, then cast to the storage dtype.
# ---------------------------------------------------------------------------------------------

def c1_bias_res_layernorm_gelu(rows: int = 256, n: int = 768, dtype: str = "f32", eps: float = 1e-5,
                               salt: int = 0):
    """x + res + bias -> LayerNorm(gamma, beta) -> GELU(erf); x, res [rows, n]; bias, gamma, beta [n]."""
    g = _rng(1, salt)
    x = g.standard_normal((rows, n), dtype=np.float32)
    res = g.standard_normal((rows, n), dtype=np.float32)
    bias = g.standard_normal(n, dtype=np.float32)
    gamma = 1.0 + 0.1 * g.standard_normal(n, dtype=np.float32)
    beta = g.standard_normal(n, dtype=np.float32)
    c = ChainSpec(inputs=[(dtype, (rows, n)), (dtype, (rows, n)), (dtype, (n,)), (dtype, (n,)), (dtype, (n,))])
    v = c.op("add", 0, 1)
    v = c.op("add", v, 2)
    v = c.op("layernorm", v, 3, 4, f=[eps])
    v = c.op("gelu_erf", v)
    c.out(v, dtype)
    return c, [quantise(t, dtype) for t in (x, res, bias, gamma, beta)]


def c2_causal_softmax(b: int = 8, h: int = 12, s: int = 512, dtype: str = "f16", scale: float = 0.125,
                      sigma: float = 2.0, salt: int = 0, s_k: int | None = None):
    """scores * scale -> causal mask (j > i -> -inf) -> softmax over the last dim; scores [b, h, s, s_k]."""
    s_k = s if s_k is None else s_k
    g = _rng(2, salt)
    scores = sigma * g.standard_normal((b, h, s, s_k), dtype=np.float32)
    c = ChainSpec(inputs=[(dtype, (b, h, s, s_k))])
    v = c.op("scale", 0, f=[scale])
    v = c.op("causal_mask", v)
    v = c.op("softmax", v)
    c.out(v, dtype)
    return c, [quantise(scores, dtype)]


def c3_bias_res_layernorm(rows: int = 16384, n: int = 1024, dtype: str = "f16", eps: float = 1e-5,
                          salt: int = 0):
    """x + bias + res -> LayerNorm(gamma, beta); x, res [rows, n]; bias, gamma, beta [n]."""
    g = _rng(3, salt)
    x = g.standard_normal((rows, n), dtype=np.float32)
    res = g.standard_normal((rows, n), dtype=np.float32)
    bias = g.standard_normal(n, dtype=np.float32)
    gamma = 1.0 + 0.1 * g.standard_normal(n, dtype=np.float32)
    beta = g.standard_normal(n, dtype=np.float32)
    c = ChainSpec(inputs=[(dtype, (rows, n)), (dtype, (rows, n)), (dtype, (n,)), (dtype, (n,)), (dtype, (n,))])
    v = c.op("add", 0, 2)
    v = c.op("add", v, 1)
    v = c.op("layernorm", v, 3, 4, f=[eps])
    c.out(v, dtype)
    return c, [quantise(t, dtype) for t in (x, res, bias, gamma, beta)]


def c4_bias_scale_permute(b: int = 32, s: int = 512, h: int = 16, d: int = 64, dtype: str = "bf16",
                          scale: float = 0.125, salt: int = 0):
    """(Q + bias[h, d]) * scale -> permute [b, s, h, d] -> [b, h, s, d]."""
    g = _rng(4, salt)
    q = g.uniform(-1.0, 1.0, (b, s, h, d)).astype(np.float32)
    bias = g.uniform(-1.0, 1.0, (h, d)).astype(np.float32)
    c = ChainSpec(inputs=[(dtype, (b, s, h, d)), (dtype, (h, d))])
    v = c.op("add", 0, 1)
    v = c.op("scale", v, f=[scale])
    v = c.op("permute", v, i=[0, 2, 1, 3])
    c.out(v, dtype)
    return c, [quantise(q, dtype), quantise(bias, dtype)]


def c5_groupnorm_silu(n: int = 16, h: int = 64, w: int = 64, ch: int = 512, groups: int = 32,
                      dtype: str = "f16", eps: float = 1e-5, salt: int = 0):
    """GroupNorm(groups, affine) -> SiLU on NHWC x [n, h, w, ch]; gamma, beta [ch]."""
    g = _rng(5, salt)
    x = g.standard_normal((n, h, w, ch), dtype=np.float32)
    off = g.uniform(-2.0, 2.0, ch).astype(np.float32)
    x = x + off            # one offset per channel, shared over n, h, w
    gamma = 1.0 + 0.1 * g.standard_normal(ch, dtype=np.float32)
    beta = g.standard_normal(ch, dtype=np.float32)
    c = ChainSpec(inputs=[(dtype, (n, h, w, ch)), (dtype, (ch,)), (dtype, (ch,))])
    v = c.op("groupnorm", 0, 1, 2, f=[eps], i=[groups])
    v = c.op("silu", v)
    c.out(v, dtype)
    return c, [quantise(t, dtype) for t in (x, gamma, beta)]


def x1_bias_scale_transpose(b: int = 32, s: int = 512, d: int = 1024, dtype: str = "bf16", scale: float = 0.125,
                            salt: int = 0):
    """(K + bias[d]) * scale -> [b, s, d] -> [b, d, s]: a chain whose permutation changes the innermost dim."""
    g = _rng(6, salt)
    k = g.uniform(-1.0, 1.0, (b, s, d)).astype(np.float32)
    bias = g.uniform(-1.0, 1.0, d).astype(np.float32)
    c = ChainSpec(inputs=[(dtype, (b, s, d)), (dtype, (d,))])
    v = c.op("add", 0, 1)
    v = c.op("scale", v, f=[scale])
    v = c.op("permute", v, i=[0, 2, 1])
    c.out(v, dtype)
    return c, [quantise(k, dtype), quantise(bias, dtype)]


def x2_decode_attention(b: int = 8, h: int = 25, t: int = 1023, d: int = 64, dtype: str = "f16",
                        cache_outputs: bool = False, salt: int = 0):
    """Attention of one new token against t cached keys and values per head (not a BASELINE config; the
    paper's GPT-2 case study with a key-value cache): K' = concat(K, k), V' = concat(V, v),
    o = softmax(K' q / sqrt(d)) V'.  q, k, v [b, h, d]; K, V [b, h, t, d]; o [b, h, d]."""
    g = _rng(7, salt)
    q = g.standard_normal((b, h, d), dtype=np.float32)
    k = g.standard_normal((b, h, d), dtype=np.float32)
    v = g.standard_normal((b, h, d), dtype=np.float32)
    kc = g.standard_normal((b, h, t, d), dtype=np.float32)
    vc = g.standard_normal((b, h, t, d), dtype=np.float32)
    c = ChainSpec(inputs=[(dtype, (b, h, d)), (dtype, (b, h, d)), (dtype, (b, h, d)), (dtype, (b, h, t, d)), (dtype, (b, h, t, d))])
    k_all = c.op("concat_rows", 3, 1)
    s = c.op("matvec", k_all, 0)
    s = c.op("scale", s, f=[1.0 / float(np.sqrt(d))])
    p = c.op("softmax", s)
    v_all = c.op("concat_rows", 4, 2)
    o = c.op("vecmat", p, v_all)
    c.out(o, dtype)
    if cache_outputs:
        c.out(k_all, dtype)
        c.out(v_all, dtype)
    return c, [quantise(x, dtype) for x in (q, k, v, kc, vc)]


def x4_relu_dwconv(n: int = 32, h: int = 56, w: int = 56, c: int = 240, k: int = 3, dtype: str = "f16", salt: int = 0,
                   stride: int = 1):
    """RELU -> depthwise k x k convolution (stride 1 or more) -> + bias on channels-last x [n, h, w, c] (not a
    BASELINE config; the EfficientNet fragment of the paper's section 6).  Weights [k, k, c] ~ N(0, 1/k),
    bias [c] ~ N(0, 1)."""
    g = _rng(9, salt)
    x = g.standard_normal((n, h, w, c), dtype=np.float32)
    wgt = (g.standard_normal((k, k, c), dtype=np.float32) / np.float32(k))
    bias = g.standard_normal(c, dtype=np.float32)
    s = ChainSpec(inputs=[(dtype, (n, h, w, c)), (dtype, (k, k, c)), (dtype, (c,))])
    v = s.op("relu", 0)
    v = s.op("dwconv2d", v, 1, i=[stride] if stride != 1 else [])
    v = s.op("add", v, 2)
    s.out(v, dtype)
    return s, [quantise(x, dtype), quantise(wgt, dtype), quantise(bias, dtype)]


def x3_channel_shuffle(n: int = 128, c: int = 232, h: int = 28, w: int = 28, groups: int = 2, dtype: str = "f16",
                       salt: int = 0):
    """concat -> channel shuffle -> split on NCHW tensors (not a BASELINE config; the ShuffleNet fragment of
    the paper's section 2): a, b [n, c/2, h, w]; y = shuffle_groups(concat(a, b)); outputs y[:, :c/2], y[:, c/2:]."""
    g = _rng(8, salt)
    a = g.standard_normal((n, c // 2, h, w), dtype=np.float32)
    b = g.standard_normal((n, c // 2, h, w), dtype=np.float32)
    s = ChainSpec(inputs=[(dtype, (n, c // 2, h, w)), (dtype, (n, c // 2, h, w))])
    y = s.op("concat", 0, 1, i=[1])
    y = s.op("reshape", y, i=[n, groups, c // groups, h, w])
    y = s.op("permute", y, i=[0, 2, 1, 3, 4])
    y = s.op("reshape", y, i=[n, c, h, w])
    s.out(s.op("slice", y, i=[1, 0, c // 2]), dtype)
    s.out(s.op("slice", y, i=[1, c // 2, c // 2]), dtype)
    return s, [quantise(a, dtype), quantise(b, dtype)]


def x5_groupnorm_silu_wide_groups(n: int = 16, h: int = 64, w: int = 64, ch: int = 320, groups: int = 32, dtype: str = "f16"):
    """GroupNorm + SiLU with 10 channels per group (not a BASELINE config): a group is not a whole number of
    16-byte vectors, so the general-width kernels run."""
    return c5_groupnorm_silu(n=n, h=h, w=w, ch=ch, groups=groups, dtype=dtype, salt=3)


def x6_silu_global_mean(n: int = 32, h: int = 56, w: int = 56, c: int = 240, dtype: str = "f16"):
    """SiLU -> mean over H and W of channels-last x [n, h, w, c] (not a BASELINE config; the squeeze step of a
    squeeze-and-excite block with the activation in front of it)."""
    g = _rng(11, 0)
    x = g.standard_normal((n, h, w, c), dtype=np.float32)
    s = ChainSpec(inputs=[(dtype, (n, h, w, c))])
    s.out(s.op("reduce_mean", s.op("silu", 0), i=[1, 2]), dtype)
    return s, [quantise(x, dtype)]


def x7_channels_first_layernorm(n: int = 64, c: int = 96, h: int = 56, w: int = 56, dtype: str = "f16"):
    """LayerNorm over the channels of a channels-first x [n, c, h, w], written as move the channels to the end ->
    LayerNorm -> move them back (not a BASELINE config; the normalisation of a convolutional network's
    down-sampling layers)."""
    g = _rng(12, 0)
    x = g.standard_normal((n, c, h, w), dtype=np.float32)
    gamma = g.uniform(0.5, 1.5, c).astype(np.float32)
    beta = g.uniform(-0.5, 0.5, c).astype(np.float32)
    s = ChainSpec(inputs=[(dtype, (n, c, h, w)), (dtype, (c,)), (dtype, (c,))])
    v = s.op("permute", 0, i=[0, 2, 3, 1])
    v = s.op("layernorm", v, 1, 2, f=[1e-6])
    s.out(s.op("permute", v, i=[0, 3, 1, 2]), dtype)
    return s, [quantise(x, dtype), quantise(gamma, dtype), quantise(beta, dtype)]


CONFIGS = {
    "C1": c1_bias_res_layernorm_gelu,
    "C2": c2_causal_softmax,
    "C3": c3_bias_res_layernorm,
    "C4": c4_bias_scale_permute,
    "C5": c5_groupnorm_silu,
    "X1": x1_bias_scale_transpose,      # not a BASELINE config: the innermost-changing transpose, for context
    "X4": x4_relu_dwconv,               # not a BASELINE config: activation + depthwise convolution
    "X3": x3_channel_shuffle,           # not a BASELINE config: concat -> channel shuffle -> split
    "X2": x2_decode_attention,          # not a BASELINE config: one-token attention against a key-value cache
    "X5": x5_groupnorm_silu_wide_groups,  # not a BASELINE config: GroupNorm with groups of 10 channels
    "X6": x6_silu_global_mean,          # not a BASELINE config: activation + global average pooling
    "X7": x7_channels_first_layernorm,  # not a BASELINE config: normalisation over a strided dimension
}


def compulsory_bytes(spec: ChainSpec, out_shapes: Sequence[Sequence[int]]) -> int:
    """Every input once plus every output once, in bytes."""
    size = {"f32": 4, "f16": 2, "bf16": 2}
    total = 0
    for dt, shape in spec.inputs:
        total += size[dt] * int(np.prod(shape, dtype=np.int64))
    for (_, dt), shape in zip(spec.outputs, out_shapes):
        total += size[dt] * int(np.prod(shape, dtype=np.int64))
    return total


def random_tensor(shape, dtype: str, seed: int, dist: str = "normal", scale: float = 1.0) -> torch.Tensor:
    """Generic seeded tensor for the shape-sweep tests."""
    g = np.random.default_rng(BASE_SEED * 7 + seed)
    if dist == "normal":
        x = scale * g.standard_normal(shape, dtype=np.float32)
    elif dist == "uniform":
        x = g.uniform(-scale, scale, shape).astype(np.float32)
    elif dist == "positive":
        x = g.uniform(0.25 * scale, scale, shape).astype(np.float32)
    else:
        raise ValueError(dist)
    return quantise(x, dtype)


# ---------------------------------------------------------------------------------------------
# Seeded random chains for the differential tests: structure only (which operators, which operands,
# which shapes); values stay O(1) so that the absolute fp32 bar is meaningful.
# ---------------------------------------------------------------------------------------------

def random_chain(seed: int, transform_operands: bool = False):
    """A random chain of the canonical form `element-wise* -> [core] -> element-wise*` with random shapes,
    operand kinds (full shape, trailing broadcast, broadcast with extents of 1, scalar) and dtypes.
    With transform_operands, about half of the broadcast operands go through an operator of their own (sigmoid,
    addc, scale) before they meet the running value; the chain is otherwise the same as without.
    Returns (ChainSpec, inputs, description)."""
    g = np.random.default_rng(BASE_SEED * 13 + seed)
    g2 = np.random.default_rng(BASE_SEED * 43 + seed)  # decisions of transform_operands only: the other draws stay as they are
    dtype = str(g.choice(["f16", "bf16", "f32"]))
    inner = int(g.choice([8, 24, 64, 96, 197, 200, 512, 1000, 2048]))
    rank = int(g.integers(2, 5))
    lead = [int(g.integers(1, 6)) for _ in range(rank - 1)]
    shape = tuple(lead + [inner])
    core = str(g.choice(["none", "softmax", "layernorm", "rmsnorm", "reduce_sum", "reduce_max", "reduce_mean", "permute",
                         "row_program"]))
    if core == "permute" and (rank < 3 or (inner * (4 if dtype == "f32" else 2)) % 16 != 0):
        core = "none"
    inputs, tensors = [(dtype, shape)], [random_tensor(shape, dtype, 100 * seed, scale=0.7)]

    def new_input(shp, dist="normal", scale=0.7):
        inputs.append((dtype, tuple(shp)))
        tensors.append(random_tensor(tuple(shp), dtype, 100 * seed + len(inputs), dist=dist, scale=scale))
        return len(inputs) - 1

    ops = []          # (name, src placeholders, f, i); value ids are fixed up once the input count is known
    def emit(name, *src, f=(), i=()):
        ops.append((name, src, tuple(f), tuple(i)))
        return ("op", len(ops) - 1)

    def operand_for(cur_shape, kinds=("full", "trailing", "ones", "scalar", "row")):
        kind = str(g.choice(list(kinds)))
        if kind == "full":
            return ("in", new_input(cur_shape))
        if kind == "trailing":
            k = int(g.integers(1, len(cur_shape)))
            return ("in", new_input(cur_shape[-k:]))
        if kind == "ones":
            shp = [e if g.random() < 0.5 else 1 for e in cur_shape]
            if all(e == 1 for e in shp) or shp == list(cur_shape):
                shp = [1] * (len(cur_shape) - 1) + [cur_shape[-1]]
            return ("in", new_input(shp))
        if kind == "row":
            return ("in", new_input(list(cur_shape[:-1]) + [1]))
        return ("in", new_input((1,)))

    def elementwise_steps(v, cur_shape, n):
        for _ in range(n):
            name = str(g.choice(["add", "sub", "mul", "max", "min", "scale", "addc", "neg", "relu", "sigmoid", "silu",
                                 "gelu_erf", "tanh"]))
            if name in ("add", "sub", "mul", "max", "min"):
                # (a clamp against one value per row or per tensor can make whole rows constant, where a
                # normalisation amplifies fp32 rounding of the mean by 1 / sqrt(eps): not what is tested here)
                n_before = len(inputs)
                o = operand_for(cur_shape) if name not in ("max", "min") else operand_for(cur_shape, ("full", "trailing", "ones"))
                if transform_operands and len(inputs) > n_before and inputs[-1][1] != tuple(cur_shape) and g2.random() < 0.5:
                    how = str(g2.choice(["sigmoid", "addc", "scale"]))
                    o = emit(how, o, f=[0.5] if how != "sigmoid" else ())
                v = emit(name, v, o) if g.random() < 0.7 else emit(name, o, v)
                if name == "mul":
                    v = emit("tanh", v)          # keeps magnitudes bounded
            elif name == "scale":
                v = emit("scale", v, f=[float(g.choice([0.5, -0.75, 1.25]))])
            elif name == "addc":
                v = emit("addc", v, f=[float(g.choice([0.25, -0.5, 1.0]))])
            else:
                v = emit(name, v)
        return v

    v = elementwise_steps(("in", 0), shape, int(g.integers(0, 4)))
    out_shape = shape
    second = None     # a second output: the value that enters the core (the residual stream of a normalisation)
    if core in ("softmax", "layernorm", "rmsnorm") and v != ("in", 0) and g.random() < 0.3:
        second = v
    if core == "softmax":
        if g.random() < 0.4:
            v = emit("causal_mask", v)
        v = emit("softmax", v)
    elif core == "layernorm":
        v = emit("layernorm", v, ("in", new_input((inner,), "positive")), ("in", new_input((inner,))), f=[1e-5])
    elif core == "rmsnorm":
        v = emit("rmsnorm", v, ("in", new_input((inner,), "positive")), f=[1e-6])
    elif core.startswith("reduce_"):
        if core == "reduce_sum":
            v = emit("scale", v, f=[2.0 / inner])     # keeps the sum O(1)
        elif v == ("in", 0):
            v = emit("scale", v, f=[1.0])
        v = emit(core, v)
        out_shape = tuple(list(shape[:-1]) + [1])
    elif core == "permute":
        perm = list(range(rank - 1))
        g.shuffle(perm)
        perm = [int(p) for p in perm] + [rank - 1]
        v = emit("permute", v, i=perm)
        out_shape = tuple(shape[p] for p in perm)
    elif core == "row_program":
        # (x - mean x) / (max x - mean x + 1): two reductions, row values combined with each other
        if v == ("in", 0):
            v = emit("tanh", v)
        mean = emit("reduce_mean", v)
        top = emit("reduce_max", v)
        span = emit("addc", emit("sub", top, mean), f=[1.0])
        v = emit("div", emit("sub", v, mean), span)
    if not core.startswith("reduce_"):
        v = elementwise_steps(v, out_shape, int(g.integers(0, 3)))
    if v == ("in", 0):
        v = emit("relu", v)

    spec = ChainSpec(inputs=inputs)
    n_in = len(inputs)
    def vid(ref):
        return ref[1] if ref[0] == "in" else n_in + ref[1]
    for name, src, f, i in ops:
        spec.ops.append(OpSpec(name, tuple(vid(r) for r in src), f, i))
    spec.out(vid(v), dtype)
    if second is not None:
        spec.out(vid(second), dtype)
    return spec, tensors, f"seed {seed}: {dtype} {shape} core={core} ops={[o[0] for o in ops]} outputs={len(spec.outputs)}"


def random_groupnorm_chain(seed: int):
    """A random channels-last GroupNorm chain: random sample count, spatial extents, channel and group counts
    (groups of any width), optional element-wise steps before and after.  Returns (ChainSpec, inputs, description)."""
    g = np.random.default_rng(BASE_SEED * 17 + seed)
    dtype = str(g.choice(["f16", "bf16", "f32"]))
    vec = 4 if dtype == "f32" else 8
    c = vec * int(g.integers(1, 41))
    divisors = [d for d in range(1, c + 1) if c % d == 0 and d <= 512]
    groups = int(g.choice(divisors))
    n = int(g.integers(1, 5))
    spatial = [int(g.integers(1, 30)) for _ in range(int(g.integers(1, 3)))]
    shape = tuple([n] + spatial + [c])
    x = random_tensor(shape, dtype, 300 * seed, scale=0.8)
    pre = str(g.choice(["none", "relu", "bias", "sample_bias"]))
    # per-channel offsets; smaller in front of a RELU, where a channel pushed far below zero would be almost
    # constant and its few positive values normalise to magnitudes whose 16-bit rounding alone exceeds the bar
    off = random_tensor((c,), "f32", 300 * seed + 1, dist="uniform", scale=0.5 if pre == "relu" else 2.0)
    x = quantise(widen(x).astype(np.float32) + widen(off).astype(np.float32), dtype)
    gamma = random_tensor((c,), dtype, 300 * seed + 2, dist="positive")
    beta = random_tensor((c,), dtype, 300 * seed + 3, scale=0.5)
    ins, tensors = [(dtype, shape), (dtype, (c,)), (dtype, (c,))], [x, gamma, beta]
    s = ChainSpec(inputs=ins)
    v = 0
    if pre == "relu":
        v = s.op("relu", v)
    elif pre in ("bias", "sample_bias"):
        shp = (c,) if pre == "bias" else tuple([n] + [1] * len(spatial) + [c])
        s.inputs.append((dtype, shp))
        tensors.append(random_tensor(shp, dtype, 300 * seed + 4, scale=0.5))
        v = s.op("add", v, len(s.inputs) - 1)
    # operator ids depend on the final input count: rebuild with it known
    n_in = len(s.inputs)
    s.ops = []
    v = 0
    if pre == "relu":
        v = s.op("relu", v)
    elif pre in ("bias", "sample_bias"):
        v = s.op("add", v, n_in - 1)
    v = s.op("groupnorm", v, 1, 2, f=[1e-5], i=[groups])
    post = str(g.choice(["none", "silu", "relu"]))
    if post != "none":
        v = s.op(post, v)
    s.out(v, dtype)
    return s, tensors, f"seed {seed}: {dtype} {shape} groups={groups} pre={pre} post={post}"


def random_stencil_chain(seed: int):
    """A random depthwise-convolution chain: random image and channel extents, 3 x 3 or 5 x 5 kernels, stride
    1 to 3, a random element-wise step in front (it decides whether the staged tile is packed) and behind."""
    g = np.random.default_rng(BASE_SEED * 19 + seed)
    dtype = str(g.choice(["f16", "bf16", "f32"]))
    vec = 4 if dtype == "f32" else 8
    c = vec * int(g.integers(1, 25))
    n, h, w = int(g.integers(1, 4)), int(g.integers(1, 24)), int(g.integers(1, 24))
    k = int(g.choice([3, 5]))
    stride = int(g.choice([1, 1, 2, 3]))
    oh, ow = (h - 1) // stride + 1, (w - 1) // stride + 1
    pre = str(g.choice(["none", "relu", "sigmoid", "bias", "neg"]))
    post = str(g.choice(["none", "bias", "silu", "residual"]))
    ins = [(dtype, (n, h, w, c)), (dtype, (k, k, c))]
    tensors = [random_tensor((n, h, w, c), dtype, 500 * seed, scale=0.8), random_tensor((k, k, c), dtype, 500 * seed + 1, scale=1.0 / k)]
    extra = []
    if pre == "bias":
        extra.append(("pre", (c,)))
    if post == "bias":
        extra.append(("post", (c,)))
    if post == "residual":
        extra.append(("post", (n, oh, ow, c)))
    for j, (_, shp) in enumerate(extra):
        ins.append((dtype, shp))
        tensors.append(random_tensor(shp, dtype, 500 * seed + 2 + j, scale=0.5))
    s = ChainSpec(inputs=ins)
    v, nxt = 0, 2
    if pre == "bias":
        v = s.op("add", v, nxt)
        nxt += 1
    elif pre != "none":
        v = s.op(pre, v)
    v = s.op("dwconv2d", v, 1, i=[stride] if stride != 1 else [])
    if post in ("bias", "residual"):
        v = s.op("add", v, nxt)
    elif post == "silu":
        v = s.op("silu", v)
    s.out(v, dtype)
    return s, tensors, f"seed {seed}: {dtype} [{n},{h},{w},{c}] {k}x{k}/{stride} pre={pre} post={post}"


def random_attention_chain(seed: int):
    """One-token attention with random batch, head count, cache length, head dimension and storage type."""
    g = np.random.default_rng(BASE_SEED * 23 + seed)
    dtype = str(g.choice(["f16", "bf16", "f32"]))
    d = int(g.choice([32, 64, 128, 256] if dtype != "f32" else [16, 32, 64, 128]))
    b, h = int(g.integers(1, 4)), int(g.integers(1, 7))
    t = int(g.choice([1, 2, 31, 64, 100, 255, 256, 257, 700, 1500, 3000]))
    spec, ins = x2_decode_attention(b=b, h=h, t=t, d=d, dtype=dtype, cache_outputs=bool(g.random() < 0.3), salt=seed)
    return spec, ins, f"seed {seed}: {dtype} b={b} h={h} t={t} d={d} outputs={len(spec.outputs)}"


def random_permute_chain(seed: int):
    """(x [+ bias] [* scale]) -> random permutation of 2 to 5 dimensions; the innermost extents of both layouts are
    whole 16-byte vectors in half of the chains and arbitrary in the other half."""
    g = np.random.default_rng(BASE_SEED * 29 + seed)
    dtype = str(g.choice(["f16", "bf16", "f32"]))
    vec = 4 if dtype == "f32" else 8
    rank = int(g.integers(2, 6))
    perm = [int(p) for p in g.permutation(rank)]
    shape = [int(g.integers(1, 9)) for _ in range(rank)]
    ragged = bool(g.random() < 0.5)                          # extents that are not whole 16-byte vectors
    shape[rank - 1] = int(g.integers(2, 98)) if ragged else vec * int(g.integers(1, 13))           # innermost of the input
    shape[perm[rank - 1]] = int(g.integers(2, 98)) if ragged else vec * int(g.integers(1, 13))     # innermost of the output
    shape = tuple(shape)
    ins, tensors = [(dtype, shape)], [random_tensor(shape, dtype, 700 * seed, dist="uniform")]
    s = ChainSpec(inputs=ins)
    v = 0
    step = str(g.choice(["none", "bias", "scale", "bias_scale"]))
    if step in ("bias", "bias_scale"):
        s.inputs.append((dtype, (shape[-1],)))
        tensors.append(random_tensor((shape[-1],), dtype, 700 * seed + 1, dist="uniform"))
        v = s.op("add", v, 1)
    if step in ("scale", "bias_scale"):
        v = s.op("scale", v, f=[0.125])
    v = s.op("permute", v, i=perm)
    s.out(v, dtype)
    return s, tensors, f"seed {seed}: {dtype} {shape} perm={perm} step={step}"


def random_layout_chain(seed: int):
    """A random layout-only chain: 1 to 3 inputs joined, sliced, permuted and reshaped at random, 1 or 2 outputs.
    Returns (ChainSpec, description); the tests fill the inputs with arbitrary bit patterns."""
    g = np.random.default_rng(BASE_SEED * 31 + seed)
    dtype = str(g.choice(["f16", "bf16", "f32"]))
    rank = int(g.integers(2, 5))
    shape = [int(g.integers(1, 13)) for _ in range(rank)]
    n_inputs = int(g.integers(1, 4))
    s = ChainSpec(inputs=[(dtype, tuple(shape)) for _ in range(n_inputs)])
    pool = list(range(n_inputs))          # inputs not joined in yet
    v, cur = pool.pop(0), list(shape)
    steps = []
    for _ in range(int(g.integers(2, 7))):
        kind = str(g.choice(["concat", "slice", "permute", "reshape"]))
        if kind == "concat" and pool and cur == shape:
            ax = int(g.integers(0, len(cur)))
            v = s.op("concat", v, pool.pop(0), i=[ax]) if g.random() < 0.5 else s.op("concat", pool.pop(0), v, i=[ax])
            cur = list(cur)
            cur[ax] *= 2
        elif kind == "slice":
            ax = int(g.integers(0, len(cur)))
            if cur[ax] < 2:
                continue
            length = int(g.integers(1, cur[ax]))
            start = int(g.integers(0, cur[ax] - length + 1))
            v = s.op("slice", v, i=[ax, start, length])
            cur[ax] = length
        elif kind == "permute" and len(cur) > 1:
            perm = [int(p) for p in g.permutation(len(cur))]
            v = s.op("permute", v, i=perm)
            cur = [cur[p] for p in perm]
        elif kind == "reshape":
            if len(cur) > 1 and g.random() < 0.5:
                q = int(g.integers(0, len(cur) - 1))
                cur = cur[:q] + [cur[q] * cur[q + 1]] + cur[q + 2:]
            elif len(cur) < 6:
                q = int(g.integers(0, len(cur)))
                f = [d for d in (2, 3, 4, 5) if cur[q] % d == 0]
                if not f:
                    continue
                d = int(g.choice(f))
                cur = cur[:q] + [d, cur[q] // d] + cur[q + 1:]
            else:
                continue
            v = s.op("reshape", v, i=cur)
        else:
            continue
        steps.append(kind)
    if not any(k in ("concat", "slice") for k in steps):
        ax = int(np.argmax(cur))
        if cur[ax] >= 2:
            v = s.op("slice", v, i=[ax, 0, cur[ax] - 1])
            cur[ax] -= 1
            steps.append("slice")
    if v < n_inputs:                      # nothing was emitted at all
        v = s.op("permute", v, i=list(range(len(cur)))[::-1])
    ax = int(np.argmax(cur))
    if cur[ax] >= 2 and g.random() < 0.4:
        half = cur[ax] // 2
        s.out(s.op("slice", v, i=[ax, 0, half]), dtype)
        s.out(s.op("slice", v, i=[ax, half, cur[ax] - half]), dtype)
    else:
        s.out(v, dtype)
    # inputs never joined in are dropped from the description
    used = sorted({src for o in s.ops for src in o.src if src < n_inputs})
    if len(used) != n_inputs:
        remap = {old: new for new, old in enumerate(used)}
        shift = n_inputs - len(used)
        fix = lambda x: remap[x] if x < n_inputs else x - shift
        s = ChainSpec(inputs=[s.inputs[u] for u in used],
                      ops=[OpSpec(o.name, tuple(fix(x) for x in o.src), o.f, o.i) for o in s.ops],
                      outputs=[(fix(x), dt) for x, dt in s.outputs])
    return s, f"seed {seed}: {dtype} {tuple(shape)} x{len(s.inputs)} steps={steps} outputs={len(s.outputs)}"


def random_pool_chain(seed: int):
    """A random pooling chain: [element-wise] -> reduce_sum / max / mean over the positions of a channels-last tensor
    -> [element-wise]; random sample count, 1 to 3 spatial dimensions, channel count (whole 16-byte vectors in six
    chains of ten, any count in the others), storage type."""
    g = np.random.default_rng(BASE_SEED * 37 + seed)
    dtype = str(g.choice(["f16", "bf16", "f32"]))
    vec = 4 if dtype == "f32" else 8
    c = vec * int(g.integers(1, 65))
    if g.random() < 0.4:
        c = int(g.integers(1, 400))
    n = int(g.integers(1, 6))
    spatial = [int(g.integers(1, 48)) for _ in range(int(g.integers(1, 4)))]
    shape = tuple([n] + spatial + [c])
    positions = int(np.prod(spatial))
    op = str(g.choice(["reduce_sum", "reduce_max", "reduce_mean"]))
    # (sums are kept O(1): a 16-bit result of magnitude 16 is rounded by more than the absolute bar allows)
    x = random_tensor(shape, dtype, 900 * seed, scale=2.0 / positions if op == "reduce_sum" else 0.8)
    s = ChainSpec(inputs=[(dtype, shape)])
    tensors = [x]
    pre = str(g.choice(["none", "relu", "silu", "bias"]))
    post = str(g.choice(["none", "sigmoid", "bias", "sample_bias"]))
    if pre == "bias":
        s.inputs.append((dtype, (c,)))
        tensors.append(random_tensor((c,), dtype, 900 * seed + 1, scale=0.3 / (positions if op == "reduce_sum" else 1.0)))
    if post in ("bias", "sample_bias"):
        shp = (c,) if post == "bias" else tuple([n] + [1] * len(spatial) + [c])
        s.inputs.append((dtype, shp))
        tensors.append(random_tensor(shp, dtype, 900 * seed + 2, scale=0.3))
    v = 0
    if pre == "bias":
        v = s.op("add", v, 1)
    elif pre != "none":
        v = s.op(pre, v)
    v = s.op(op, v, i=list(range(1, len(shape) - 1)))
    if post in ("bias", "sample_bias"):
        v = s.op("add", v, len(s.inputs) - 1)
    elif post == "sigmoid":
        v = s.op("sigmoid", v)
    s.out(v, dtype)
    return s, tensors, f"seed {seed}: {dtype} {shape} {op} pre={pre} post={post}"


def random_multi_kernel_chain(seed: int):
    """A random chain with two to four exchanges wider than a lane (softmax, layer / RMS normalisation, a reduction
    over the last dimension used as a row statistic, a permutation of the leading dimensions, a transposition of the
    last two) and random element-wise steps between them: more than one kernel in nearly every case."""
    g = np.random.default_rng(BASE_SEED * 41 + seed)
    dtype = str(g.choice(["f16", "bf16", "f32"]))
    shape = [int(g.integers(2, 6)), int(g.choice([3, 8, 17, 32])), int(g.choice([16, 24, 40, 64, 128, 200, 256]))]  # (no extents of 1: a permutation that makes one innermost is refused)
    s = ChainSpec(inputs=[(dtype, tuple(shape))])
    tensors = [random_tensor(tuple(shape), dtype, 1100 * seed)]
    names = []

    def operand(shp, scale, dist="normal"):
        s.inputs.append((dtype, tuple(shp)))
        tensors.append(random_tensor(tuple(shp), dtype, 1100 * seed + len(tensors), dist=dist, scale=scale))
        return len(s.inputs) - 1

    # inputs must be declared before operators use value ids: collect the stages first, then number the values
    stages = []
    for _ in range(int(g.integers(2, 5))):
        st = str(g.choice(["softmax", "layernorm", "rmsnorm", "swap_leading", "transpose_inner", "centre"]))
        stages.append(st)
        for _ in range(int(g.integers(0, 3))):
            stages.append(str(g.choice(["ew_silu", "ew_bias", "ew_full", "ew_scale", "ew_tanh"])))
    plan = []
    cur = list(shape)
    for st in stages:
        if len(s.inputs) + 2 > 8:  # the description holds eight inputs
            st = {"layernorm": "softmax", "rmsnorm": "softmax", "ew_bias": "ew_silu", "ew_full": "ew_tanh"}.get(st, st)
        if st in ("layernorm", "rmsnorm"):
            gam = operand((cur[-1],), 1.0, "positive")
            bet = operand((cur[-1],), 0.3) if st == "layernorm" else None
            plan.append((st, gam, bet))
        elif st == "swap_leading":
            plan.append((st,))
            cur = [cur[1], cur[0], cur[2]]
        elif st == "transpose_inner":
            plan.append((st,))
            cur = [cur[0], cur[2], cur[1]]
        elif st == "ew_bias":
            plan.append((st, operand((cur[-1],), 0.3)))
        elif st == "ew_full":
            plan.append((st, operand(tuple(cur), 0.5)))
        else:
            plan.append((st,))
    n_in = len(s.inputs)
    # ChainSpec numbers operator results after the inputs that exist when op() is called, so all inputs are in place now
    v = 0
    for item in plan:
        st = item[0]
        names.append(st)
        if st == "softmax":
            v = s.op("softmax", v)
        elif st == "layernorm":
            v = s.op("layernorm", v, item[1], item[2], f=[1e-5])
        elif st == "rmsnorm":
            v = s.op("rmsnorm", v, item[1], f=[1e-5])
        elif st == "swap_leading":
            v = s.op("permute", v, i=[1, 0, 2])
        elif st == "transpose_inner":
            v = s.op("permute", v, i=[0, 2, 1])
        elif st == "centre":
            v = s.op("sub", v, s.op("reduce_mean", v))
        elif st == "ew_silu":
            v = s.op("silu", v)
        elif st == "ew_tanh":
            v = s.op("tanh", v)
        elif st == "ew_scale":
            v = s.op("scale", v, f=[0.5])
        else:
            v = s.op("add", v, item[1])
    assert len(s.inputs) == n_in
    s.out(v, dtype)
    return s, tensors, f"seed {seed}: {dtype} {tuple(shape)} " + " > ".join(names)
