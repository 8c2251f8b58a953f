"""Pins for the CPU oracle: closed forms, invariants, brute-force tiny cases, hand-expanded fixtures and
library routines.  None of the expected values comes from the oracle itself or from the HIP path.

What the method computes is the unfused operator-by-operator result (paper section 5.1: merging removes
data movement only; section 5.2: rewriting never changes the program's meaning); the paper gives no
operator formulas or worked examples, so the pins are the operators' textbook definitions.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import pf_oracle as orc
import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def load_fixture(name):
    out = {}
    with open(os.path.join(GOLD, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, rest = line.partition(":")
            out[key.strip()] = np.array([float(v) for v in rest.split()], dtype=np.float64)
    return out


# ---------------- hand-expanded fixtures ----------------

def test_fixture_layernorm_2x4():
    fx = load_fixture("layernorm_2x4.txt")
    x = fx["x"].reshape(2, 4)
    plain = orc.layernorm(x, None, None, fx["eps"][0])
    np.testing.assert_allclose(plain.ravel(), fx["normalised"], rtol=0, atol=1e-15)
    y = orc.layernorm(x, fx["gamma"], fx["beta"], fx["eps"][0])
    np.testing.assert_allclose(y.ravel(), fx["y"], rtol=0, atol=2e-15)


def test_fixture_causal_softmax_3x3():
    fx = load_fixture("causal_softmax_3x3.txt")
    spec = wl.ChainSpec(inputs=[("f32", (1, 3, 3))])
    v = spec.op("scale", 0, f=[fx["scale"][0]])
    v = spec.op("causal_mask", v)
    v = spec.op("softmax", v)
    spec.out(v, "f32")
    (y,) = orc.evaluate_outputs(spec, [fx["x"].reshape(1, 3, 3)])
    np.testing.assert_allclose(y.ravel(), fx["y"], rtol=0, atol=1e-15)
    # masked entries are exactly zero, not merely small
    assert y[0, 0, 1] == 0.0 and y[0, 0, 2] == 0.0 and y[0, 1, 2] == 0.0


def test_fixture_groupnorm_tiny():
    fx = load_fixture("groupnorm_1x2x2x4_g2.txt")
    x = fx["x"].reshape(1, 2, 2, 4)
    plain = orc.groupnorm_nhwc(x, None, None, int(fx["groups"][0]), fx["eps"][0])
    np.testing.assert_allclose(plain.ravel(), fx["normalised"], rtol=0, atol=2e-15)
    y = orc.groupnorm_nhwc(x, fx["gamma"], fx["beta"], int(fx["groups"][0]), fx["eps"][0])
    np.testing.assert_allclose(y.ravel(), fx["y"], rtol=0, atol=4e-15)


def test_fixture_permute_iota():
    fx = load_fixture("permute_2x3x2x2.txt")
    shape = tuple(int(v) for v in fx["shape"])
    perm = [int(v) for v in fx["perm"]]
    x = np.arange(int(np.prod(shape)), dtype=np.float64).reshape(shape)
    out = orc.permute(x, perm)
    assert out.shape == (2, 2, 3, 2)
    np.testing.assert_array_equal(out.ravel(), fx["out"])


def test_fixture_activation_points():
    fx = load_fixture("gelu_silu_points.txt")
    for name in ("sigmoid", "silu", "gelu_erf", "tanh"):
        got = orc.ew_unary(name, fx["x"])
        np.testing.assert_allclose(got, fx[name], rtol=4e-16, atol=1e-16, err_msg=name)


# ---------------- element-wise and broadcast ----------------

def test_binary_operand_order_and_broadcast_direction():
    a = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]])
    v = np.array([10.0, 20.0, 40.0])
    np.testing.assert_array_equal(orc.ew_binary("sub", a, v), [[-9, -18, -37], [-6, -15, -34]])
    np.testing.assert_array_equal(orc.ew_binary("sub", v, a), [[9, 18, 37], [6, 15, 34]])
    np.testing.assert_array_equal(orc.ew_binary("div", v, a), [[10, 10, 40 / 3], [2.5, 4, 40 / 6]])
    np.testing.assert_array_equal(orc.ew_binary("div", a, v), [[0.1, 0.1, 3 / 40], [0.4, 0.25, 6 / 40]])
    np.testing.assert_array_equal(orc.ew_binary("max", a, v * 0 + 3.5), [[3.5, 3.5, 3.5], [4, 5, 6]])
    np.testing.assert_array_equal(orc.ew_binary("min", a, v * 0 + 3.5), [[1, 2, 3], [3.5, 3.5, 3.5]])
    np.testing.assert_array_equal(orc.ew_binary("mul", a, v), [[10, 40, 120], [40, 100, 240]])
    np.testing.assert_array_equal(orc.ew_binary("add", a, v), [[11, 22, 43], [14, 25, 46]])


def test_broadcast_is_over_leading_dims_only():
    a = np.zeros((2, 3, 4))
    tail = np.arange(12.0).reshape(3, 4)
    out = orc.ew_binary("add", a, tail)
    for b in range(2):
        np.testing.assert_array_equal(out[b], tail)
    with pytest.raises(ValueError):
        orc.ew_binary("add", a, np.zeros((2, 3)))      # [2,3] is not a trailing shape of [2,3,4]
    with pytest.raises(ValueError):
        orc.ew_binary("add", a, np.zeros((3,)))


def test_binary_matches_numpy_on_random():
    g = np.random.default_rng(7)
    a = g.standard_normal((5, 6, 7))
    b = g.standard_normal((6, 7)) + 3.0
    for name, fn in (("add", np.add), ("sub", np.subtract), ("mul", np.multiply), ("div", np.divide),
                     ("max", np.maximum), ("min", np.minimum)):
        np.testing.assert_array_equal(orc.ew_binary(name, a, b), fn(a, b), err_msg=name)
        np.testing.assert_array_equal(orc.ew_binary(name, b, a), fn(b, a), err_msg=name + " swapped")


def test_unary_simple_ops():
    x = np.array([-2.0, -0.0, 0.5, 4.0])
    np.testing.assert_array_equal(orc.ew_unary("scale", x, -3.0), [6.0, 0.0, -1.5, -12.0])
    np.testing.assert_array_equal(orc.ew_unary("addc", x, 1.25), [-0.75, 1.25, 1.75, 5.25])
    np.testing.assert_array_equal(orc.ew_unary("neg", x), [2.0, 0.0, -0.5, -4.0])
    np.testing.assert_array_equal(orc.ew_unary("relu", x), [0.0, 0.0, 0.5, 4.0])
    np.testing.assert_allclose(orc.ew_unary("rsqrt", np.array([4.0, 0.25, 16.0])), [0.5, 2.0, 0.25], rtol=0,
                               atol=0)
    np.testing.assert_allclose(orc.ew_unary("exp", np.array([0.0, 1.0, -1.0])), [1.0, math.e, 1 / math.e],
                               rtol=1e-16)


def test_activation_identities():
    x = np.linspace(-6, 6, 97)
    gelu = orc.ew_unary("gelu_erf", x)
    silu = orc.ew_unary("silu", x)
    np.testing.assert_allclose(gelu - orc.ew_unary("gelu_erf", -x), x, atol=1e-15)     # odd part is x/2 * 2
    np.testing.assert_allclose(silu - orc.ew_unary("silu", -x), x, atol=1e-15)
    assert orc.ew_unary("gelu_erf", np.zeros(1))[0] == 0.0 and orc.ew_unary("silu", np.zeros(1))[0] == 0.0
    sig = orc.ew_unary("sigmoid", x)
    np.testing.assert_allclose(sig + orc.ew_unary("sigmoid", -x), 1.0, atol=1e-15)
    np.testing.assert_allclose(orc.ew_unary("tanh", x), 2 * orc.ew_unary("sigmoid", 2 * x) - 1, atol=1e-15)
    # composite == decomposition into sigmoid and multiply (section 6)
    np.testing.assert_allclose(orc.silu_decomposed(x), silu, rtol=0, atol=0)


def test_activations_match_torch_float64():
    g = np.random.default_rng(11)
    x = 3 * g.standard_normal(1000)
    t = torch.from_numpy(x)
    np.testing.assert_allclose(orc.ew_unary("gelu_erf", x), torch.nn.functional.gelu(t).numpy(), atol=1e-15)
    np.testing.assert_allclose(orc.ew_unary("silu", x), torch.nn.functional.silu(t).numpy(), atol=1e-15)
    np.testing.assert_allclose(orc.ew_unary("sigmoid", x), torch.sigmoid(t).numpy(), atol=1e-15)


# ---------------- causal mask ----------------

def test_causal_mask_brute_force():
    g = np.random.default_rng(3)
    x = g.standard_normal((2, 3, 4, 6))
    y = orc.causal_mask(x)
    for idx in np.ndindex(*x.shape):
        i, j = idx[-2], idx[-1]
        if j > i:
            assert y[idx] == -np.inf
        else:
            assert y[idx] == x[idx]


# ---------------- reductions ----------------

def test_reduce_last():
    x = np.array([[1.0, 5.0, -2.0, 0.0], [7.0, 7.0, 7.0, 7.0], [-1.0, -3.0, -2.0, -8.0]])
    np.testing.assert_array_equal(orc.reduce_last("reduce_sum", x), [[4.0], [28.0], [-14.0]])
    np.testing.assert_array_equal(orc.reduce_last("reduce_max", x), [[5.0], [7.0], [-1.0]])
    np.testing.assert_array_equal(orc.reduce_last("reduce_mean", x), [[1.0], [7.0], [-3.5]])
    g = np.random.default_rng(5)
    y = g.standard_normal((3, 4, 33))
    np.testing.assert_allclose(orc.reduce_last("reduce_sum", y)[..., 0], y.sum(-1), atol=1e-13)
    np.testing.assert_array_equal(orc.reduce_last("reduce_max", y)[..., 0], y.max(-1))


# ---------------- softmax ----------------

def test_softmax_closed_forms():
    n = 9
    x = np.log(np.arange(1, n + 1, dtype=np.float64))[None, :]
    np.testing.assert_allclose(orc.softmax(x)[0], np.arange(1, n + 1) / (n * (n + 1) / 2), atol=1e-15)
    # constant row under a causal mask: row i is 1/(i+1) on j <= i
    s = 7
    y = orc.softmax(orc.causal_mask(np.full((1, s, s), 3.25)))
    for i in range(s):
        np.testing.assert_allclose(y[0, i, : i + 1], 1.0 / (i + 1), atol=1e-16)
        assert np.all(y[0, i, i + 1:] == 0.0)
    assert y[0, 0, 0] == 1.0


def test_softmax_invariants():
    g = np.random.default_rng(21)
    x = 4 * g.standard_normal((6, 5, 40))
    y = orc.softmax(x)
    assert np.all(y >= 0) and np.all(y <= 1)
    np.testing.assert_allclose(y.sum(-1), 1.0, atol=1e-12)
    np.testing.assert_allclose(orc.softmax(x + 123.5), y, atol=1e-13)            # shift invariance
    np.testing.assert_allclose(y, torch.softmax(torch.from_numpy(x), -1).numpy(), atol=1e-15)
    # ratios are exp of differences
    np.testing.assert_allclose(y[..., 3] / y[..., 7], np.exp(x[..., 3] - x[..., 7]), rtol=1e-12)


def test_softmax_fully_masked_row_is_nan():
    y = orc.softmax(np.full((1, 4), -np.inf))
    assert np.all(np.isnan(y))


def test_softmax_large_values_do_not_overflow():
    y = orc.softmax(np.array([[1000.0, 1000.0, -1000.0]]))
    np.testing.assert_allclose(y[0], [0.5, 0.5, 0.0], atol=1e-300)


# ---------------- LayerNorm / RMSNorm ----------------

def test_layernorm_closed_forms():
    n = 12
    x = np.arange(n, dtype=np.float64)[None, :]
    eps = 0.5
    var = (n * n - 1) / 12.0
    want = (x[0] - (n - 1) / 2.0) / math.sqrt(var + eps)
    np.testing.assert_allclose(orc.layernorm(x, None, None, eps)[0], want, atol=1e-15)


def test_layernorm_invariants():
    g = np.random.default_rng(31)
    x = 2 * g.standard_normal((17, 96)) + 5.0
    eps = 1e-5
    y = orc.layernorm(x, None, None, eps)
    np.testing.assert_allclose(y.mean(-1), 0.0, atol=1e-12)
    var = x.var(-1)                                        # numpy: biased
    np.testing.assert_allclose(y.var(-1), var / (var + eps), rtol=1e-12)     # exactly sigma^2/(sigma^2+eps)
    np.testing.assert_allclose(orc.layernorm(x + 77.0, None, None, eps), y, atol=1e-12)
    gamma = g.standard_normal(96)
    beta = g.standard_normal(96)
    np.testing.assert_allclose(orc.layernorm(x, gamma, beta, eps), y * gamma + beta, atol=1e-14)
    t = torch.nn.functional.layer_norm(torch.from_numpy(x), (96,), torch.from_numpy(gamma),
                                       torch.from_numpy(beta), eps)
    np.testing.assert_allclose(orc.layernorm(x, gamma, beta, eps), t.numpy(), atol=1e-13)


def test_layernorm_uses_biased_variance():
    x = np.array([[0.0, 2.0]])                            # mean 1, biased var 1, unbiased var 2
    np.testing.assert_allclose(orc.layernorm(x, None, None, 0.0)[0], [-1.0, 1.0], atol=1e-16)


def test_rmsnorm():
    x = np.array([[3.0, -4.0, 0.0, 0.0]])                 # mean square 25/4
    np.testing.assert_allclose(orc.rmsnorm(x, None, 0.0)[0], [1.2, -1.6, 0.0, 0.0], atol=1e-16)
    np.testing.assert_allclose(orc.rmsnorm(x, np.array([1.0, 2.0, 3.0, 4.0]), 0.0)[0], [1.2, -3.2, 0, 0],
                               atol=1e-16)
    g = np.random.default_rng(41)
    z = g.standard_normal((9, 64))
    z -= z.mean(-1, keepdims=True)                         # zero-mean rows: RMSNorm == LayerNorm (beta = 0)
    gamma = g.standard_normal(64)
    np.testing.assert_allclose(orc.rmsnorm(z, gamma, 1e-6), orc.layernorm(z, gamma, None, 1e-6), atol=1e-13)
    eps = 0.25
    w = g.standard_normal((4, 10))
    np.testing.assert_allclose(orc.rmsnorm(w, None, eps), w / np.sqrt((w * w).mean(-1, keepdims=True) + eps),
                               atol=1e-15)


# ---------------- GroupNorm ----------------

def test_groupnorm_one_group_is_layernorm_of_flattened_sample():
    g = np.random.default_rng(51)
    x = g.standard_normal((3, 4, 5, 6)) + 2.0
    y = orc.groupnorm_nhwc(x, None, None, 1, 1e-5)
    want = orc.layernorm(x.reshape(3, -1), None, None, 1e-5).reshape(x.shape)
    np.testing.assert_allclose(y, want, atol=1e-13)


def test_groupnorm_two_independent_paths_and_torch():
    g = np.random.default_rng(52)
    n, h, w, c, groups = 2, 3, 5, 12, 3
    x = g.standard_normal((n, h, w, c)) + g.uniform(-2, 2, c)
    gamma, beta = g.standard_normal(c), g.standard_normal(c)
    eps = 1e-5
    y = orc.groupnorm_nhwc(x, gamma, beta, groups, eps)
    # path 2: to channels-first, contiguous groups normalised as rows, back to channels-last
    xc = orc.permute(x, [0, 3, 1, 2])                                      # [n, c, h, w]
    rows = xc.reshape(n * groups, (c // groups) * h * w)
    norm = orc.layernorm(rows, None, None, eps).reshape(n, c, h, w)
    norm = norm * gamma[None, :, None, None] + beta[None, :, None, None]
    want = orc.permute(norm, [0, 2, 3, 1])
    np.testing.assert_allclose(y, want, atol=1e-13)
    t = torch.nn.functional.group_norm(torch.from_numpy(x).permute(0, 3, 1, 2), groups,
                                       torch.from_numpy(gamma), torch.from_numpy(beta), eps)
    np.testing.assert_allclose(y, t.permute(0, 2, 3, 1).numpy(), atol=1e-13)


def test_groupnorm_invariants():
    g = np.random.default_rng(53)
    n, hw, c, groups = 2, 7, 8, 4
    x = g.standard_normal((n, hw, c)) * 3 + 1
    eps = 1e-3
    y = orc.groupnorm_nhwc(x, None, None, groups, eps)
    yy = y.reshape(n, hw, groups, c // groups)
    xx = x.reshape(n, hw, groups, c // groups)
    np.testing.assert_allclose(yy.mean(axis=(1, 3)), 0.0, atol=1e-13)
    var = xx.var(axis=(1, 3))
    np.testing.assert_allclose(yy.var(axis=(1, 3)), var / (var + eps), rtol=1e-12)


# ---------------- permute / reshape ----------------

def test_permute_matches_numpy_and_inverse_is_identity():
    g = np.random.default_rng(61)
    x = g.standard_normal((2, 3, 4, 5, 6))
    for perm in ([0, 1, 2, 3, 4], [4, 3, 2, 1, 0], [0, 2, 1, 4, 3], [3, 0, 4, 1, 2]):
        y = orc.permute(x, perm)
        np.testing.assert_array_equal(y, np.transpose(x, perm))
        inv = np.argsort(perm)
        np.testing.assert_array_equal(orc.permute(y, inv), x)


def test_permute_raw_bits_exact():
    g = np.random.default_rng(62)
    bits = g.integers(0, 1 << 16, size=(3, 4, 5, 2), dtype=np.uint16)       # includes NaN / inf patterns
    out = orc.permute(bits, [0, 2, 1, 3])
    assert out.dtype == np.uint16
    np.testing.assert_array_equal(out, np.transpose(bits, [0, 2, 1, 3]))
    bits32 = g.integers(0, 1 << 32, size=(4, 6), dtype=np.uint32)
    np.testing.assert_array_equal(orc.permute(bits32, [1, 0]), bits32.T)


def test_elementwise_commutes_with_permute():
    # moving element-wise work across a layout change must not change a single bit (section 5.1, swapping)
    g = np.random.default_rng(63)
    x = g.standard_normal((3, 4, 5))
    a = orc.ew_unary("gelu_erf", orc.permute(x, [2, 0, 1]))
    b = orc.permute(orc.ew_unary("gelu_erf", x), [2, 0, 1])
    np.testing.assert_array_equal(a, b)


# ---------------- chain walker ----------------

def test_chain_walker_composite_equals_primitives():
    # softmax written with the composite op and with reduce / broadcast primitives evaluated by hand
    g = np.random.default_rng(71)
    x = g.standard_normal((4, 10))
    m = orc.reduce_last("reduce_max", x)
    e = orc.ew_unary("exp", x - m)
    want = e / orc.reduce_last("reduce_sum", e)
    np.testing.assert_allclose(orc.softmax(x), want, rtol=0, atol=0)


def test_chain_walker_c1_against_numpy_formula():
    spec, ins = wl.c1_bias_res_layernorm_gelu(rows=5, n=24)
    x, res, bias, gamma, beta = [wl.widen(t) for t in ins]
    (y,) = orc.evaluate_outputs(spec, [x, res, bias, gamma, beta])
    z = (x + res) + bias
    mu = z.mean(-1, keepdims=True)
    var = ((z - mu) ** 2).mean(-1, keepdims=True)
    ln = (z - mu) / np.sqrt(var + 1e-5) * gamma + beta
    want = np.array([[0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in row] for row in ln])
    np.testing.assert_allclose(y, want, atol=1e-14)


def test_chain_walker_c4_and_c5_shapes():
    spec, ins = wl.c4_bias_scale_permute(b=2, s=3, h=2, d=8)
    (y,) = orc.evaluate_outputs(spec, [wl.widen(t) for t in ins])
    q, bias = [wl.widen(t) for t in ins]
    assert y.shape == (2, 2, 3, 8)
    np.testing.assert_array_equal(y, np.transpose((q + bias) * 0.125, (0, 2, 1, 3)))
    spec, ins = wl.c5_groupnorm_silu(n=1, h=2, w=2, ch=8, groups=2)
    (y,) = orc.evaluate_outputs(spec, [wl.widen(t) for t in ins])
    assert y.shape == (1, 2, 2, 8)


def test_thread_count_does_not_change_results():
    spec, ins = wl.c3_bias_res_layernorm(rows=64, n=128)
    wide = [wl.widen(t) for t in ins]
    orc.set_threads(1)
    (a,) = orc.evaluate_outputs(spec, wide)
    orc.set_threads(4)
    (b,) = orc.evaluate_outputs(spec, wide)
    orc.set_threads(orc.max_threads())
    np.testing.assert_array_equal(a, b)


# ---- broadcast of a reduced value back over its row (chains written in basic operators, section 6) ----

def test_row_broadcast_direction_and_values():
    x = np.array([[1.0, 2.0, 4.0], [8.0, 16.0, 32.0]])
    v = np.array([[2.0], [4.0]])
    # worked by hand: the row value meets every element of its own row, operand order kept
    np.testing.assert_array_equal(orc.ew_binary("sub", x, v), [[-1.0, 0.0, 2.0], [4.0, 12.0, 28.0]])
    np.testing.assert_array_equal(orc.ew_binary("sub", v, x), [[1.0, 0.0, -2.0], [-4.0, -12.0, -28.0]])
    np.testing.assert_array_equal(orc.ew_binary("div", x, v), [[0.5, 1.0, 2.0], [2.0, 4.0, 8.0]])
    np.testing.assert_array_equal(orc.ew_binary("div", v, x), [[2.0, 1.0, 0.5], [0.5, 0.25, 0.125]])
    np.testing.assert_array_equal(orc.ew_binary("max", x, v), [[2.0, 2.0, 4.0], [8.0, 16.0, 32.0]])
    # higher rank: one value per row of the last dimension
    x3 = np.arange(12, dtype=np.float64).reshape(2, 2, 3)
    v3 = np.array([[[1.0], [10.0]], [[100.0], [1000.0]]])
    want = x3 + np.array([1.0, 10.0, 100.0, 1000.0]).reshape(2, 2, 1)
    np.testing.assert_array_equal(orc.ew_binary("add", x3, v3), want)
    # not a row value: different leading extents
    with pytest.raises(ValueError):
        orc.ew_binary("add", x, np.ones((3, 1)))


def _softmax_in_basic_operators(shape):
    s = wl.ChainSpec(inputs=[("f32", shape)])
    m = s.op("reduce_max", 0)
    d = s.op("sub", 0, m)
    e = s.op("exp", d)
    t = s.op("reduce_sum", e)
    s.out(s.op("div", e, t), "f32")
    return s


def test_softmax_written_in_basic_operators():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((7, 33)) * 3.0
    y = orc.evaluate_outputs(_softmax_in_basic_operators((7, 33)), [x])[0]
    # the composite is defined as exactly these steps
    np.testing.assert_array_equal(y, orc.softmax(x))
    # closed form: softmax of logarithms of positive weights is the weights normalised
    w = rng.uniform(0.5, 2.0, (4, 9))
    y = orc.evaluate_outputs(_softmax_in_basic_operators((4, 9)), [np.log(w)])[0]
    np.testing.assert_allclose(y, w / w.sum(-1, keepdims=True), rtol=1e-14)


def test_layernorm_written_in_basic_operators():
    rng = np.random.default_rng(6)
    rows, n, eps = 5, 40, 1e-5
    x = rng.standard_normal((rows, n)) * 2.0 + 1.5
    g = rng.standard_normal(n)
    b = rng.standard_normal(n)
    s = wl.ChainSpec(inputs=[("f32", (rows, n)), ("f32", (n,)), ("f32", (n,))])
    mu = s.op("reduce_mean", 0)
    c = s.op("sub", 0, mu)
    var = s.op("reduce_mean", s.op("mul", c, c))
    r = s.op("rsqrt", s.op("addc", var, f=[eps]))
    y = s.op("mul", c, r)
    y = s.op("add", s.op("mul", y, 1), 2)
    s.out(y, "f32")
    got = orc.evaluate_outputs(s, [x, g, b])[0]
    np.testing.assert_allclose(got, orc.layernorm(x, g, b, eps), rtol=1e-13, atol=1e-14)
    # textbook definition, written independently
    mean = x.mean(-1, keepdims=True)
    want = (x - mean) / np.sqrt(((x - mean) ** 2).mean(-1, keepdims=True) + eps) * g + b
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-14)


# ---- one-token attention against cached keys and values (section 8, GPT-2 case study) ----

def test_concat_matvec_vecmat_worked_by_hand():
    # t = 2 cached rows, d = 3: rows and columns deliberately of different extent so that a transposed operand
    # or a contraction over the wrong axis cannot give the same numbers
    K = np.array([[[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]]])          # [1, 2, 3]
    k = np.array([[7.0, 8.0, 9.0]])                               # [1, 3]
    Kc = orc.concat_rows(K, k)
    np.testing.assert_array_equal(Kc, [[[1.0, 2.0, 3.0], [4.0, 5.0, 6.0], [7.0, 8.0, 9.0]]])
    q = np.array([[1.0, 0.0, -1.0]])
    np.testing.assert_array_equal(orc.matvec(Kc, q), [[-2.0, -2.0, -2.0]])          # row . q
    q = np.array([[1.0, 10.0, 100.0]])
    np.testing.assert_array_equal(orc.matvec(Kc, q), [[321.0, 654.0, 987.0]])
    p = np.array([[1.0, 10.0, 100.0]])
    np.testing.assert_array_equal(orc.vecmat(p, Kc), [[741.0, 852.0, 963.0]])       # sum_j p_j row_j
    # several heads stay apart
    A = np.stack([np.eye(3), 2.0 * np.eye(3)])[None]               # [1, 2, 3, 3]
    x = np.array([[[1.0, 2.0, 3.0], [1.0, 2.0, 3.0]]])
    np.testing.assert_array_equal(orc.matvec(A, x), [[[1.0, 2.0, 3.0], [2.0, 4.0, 6.0]]])
    np.testing.assert_array_equal(orc.vecmat(x, A), [[[1.0, 2.0, 3.0], [2.0, 4.0, 6.0]]])
    with pytest.raises(ValueError):
        orc.matvec(Kc, np.ones((1, 2)))
    with pytest.raises(ValueError):
        orc.vecmat(np.ones((1, 2)), Kc)


def test_matvec_vecmat_against_library_contractions_and_linearity():
    rng = np.random.default_rng(11)
    A = rng.standard_normal((2, 3, 17, 5))
    x = rng.standard_normal((2, 3, 5))
    p = rng.standard_normal((2, 3, 17))
    np.testing.assert_allclose(orc.matvec(A, x), np.einsum("bhtd,bhd->bht", A, x), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(orc.vecmat(p, A), np.einsum("bht,bhtd->bhd", p, A), rtol=1e-13, atol=1e-13)
    # adjointness: <A x, p> = <x, p A>
    lhs = (orc.matvec(A, x) * p).sum()
    rhs = (x * orc.vecmat(p, A)).sum()
    assert abs(lhs - rhs) < 1e-11


def test_one_token_attention_chain_equals_its_definition():
    spec, ins = wl.x2_decode_attention(b=2, h=3, t=13, d=8, dtype="f32", cache_outputs=True)
    q, k, v, K, V = [wl.widen(t) for t in ins]
    o, Kc, Vc = orc.evaluate_outputs(spec, [q, k, v, K, V])
    Kd = np.concatenate([K, k[:, :, None, :]], axis=2)
    Vd = np.concatenate([V, v[:, :, None, :]], axis=2)
    np.testing.assert_array_equal(Kc, Kd)
    np.testing.assert_array_equal(Vc, Vd)
    s = np.einsum("bhtd,bhd->bht", Kd, q) / np.sqrt(8.0)
    w = np.exp(s - s.max(-1, keepdims=True))
    w /= w.sum(-1, keepdims=True)
    np.testing.assert_allclose(o, np.einsum("bht,bhtd->bhd", w, Vd), rtol=1e-12, atol=1e-13)
    # a constant value cache returns that constant whatever the keys are (weights sum to one)
    Vconst = np.full_like(V, 0.75)
    o2 = orc.evaluate_outputs(spec, [q, k, np.full_like(v, 0.75), K, Vconst])[0]
    np.testing.assert_allclose(o2, 0.75, rtol=1e-14)


# ---- concatenation / slicing / channel shuffle (the ShuffleNet fragment of section 2) ----

def test_concat_and_slice_worked_by_hand():
    a = np.array([[[1, 2], [3, 4]], [[5, 6], [7, 8]]], dtype=np.uint16)            # [2, 2, 2]
    b = np.array([[[11, 12]], [[13, 14]]], dtype=np.uint16)                         # [2, 1, 2]
    y = orc.concat(a, b, 1)
    np.testing.assert_array_equal(y, [[[1, 2], [3, 4], [11, 12]], [[5, 6], [7, 8], [13, 14]]])
    np.testing.assert_array_equal(orc.slice_axis(y, 1, 2, 1), b)
    np.testing.assert_array_equal(orc.slice_axis(y, 1, 0, 2), a)
    np.testing.assert_array_equal(orc.slice_axis(y, 2, 1, 1), [[[2], [4], [12]], [[6], [8], [14]]])
    np.testing.assert_array_equal(orc.concat(a, a, 2)[0], [[1, 2, 1, 2], [3, 4, 3, 4]])
    np.testing.assert_array_equal(orc.concat(a, a, 0).shape, (4, 2, 2))
    with pytest.raises(ValueError):
        orc.concat(a, b, 2)
    with pytest.raises(ValueError):
        orc.slice_axis(a, 1, 1, 2)


def test_concat_slice_against_library_and_inverse():
    rng = np.random.default_rng(21)
    for dt in (np.uint16, np.uint32, np.float64):
        a = rng.integers(0, 60000, (3, 4, 5, 2)).astype(dt)
        b = rng.integers(0, 60000, (3, 7, 5, 2)).astype(dt)
        y = orc.concat(a, b, 1)
        np.testing.assert_array_equal(y, np.concatenate([a, b], axis=1))
        np.testing.assert_array_equal(orc.slice_axis(y, 1, 0, 4), a)
        np.testing.assert_array_equal(orc.slice_axis(y, 1, 4, 7), b)
        np.testing.assert_array_equal(orc.slice_axis(y, 2, 1, 3), y[:, :, 1:4])


def test_channel_shuffle_chain_has_its_closed_form():
    # shuffled[n, j * g + i] = concat[n, i * (c / g) + j]: with g = 2 the halves of a and b interleave
    for groups, c in ((2, 12), (4, 16)):
        spec, ins = wl.x3_channel_shuffle(n=2, c=c, h=3, w=5, groups=groups, dtype="f16")
        bits = [wl.raw_bits(t) for t in ins]
        o0, o1 = orc.evaluate_layout_bits(spec, bits)
        cat = np.concatenate(bits, axis=1)
        want = np.empty_like(cat)
        per = c // groups
        for i in range(groups):
            for j in range(per):
                want[:, j * groups + i] = cat[:, i * per + j]
        np.testing.assert_array_equal(o0, want[:, :c // 2])
        np.testing.assert_array_equal(o1, want[:, c // 2:])
    # g = 2: output 0 interleaves the first halves of a and b channel by channel
    spec, ins = wl.x3_channel_shuffle(n=1, c=8, h=1, w=2, groups=2, dtype="f32")
    a, b = [wl.raw_bits(t) for t in ins]
    o0, o1 = orc.evaluate_layout_bits(spec, [a, b])
    np.testing.assert_array_equal(o0[0], [a[0, 0], b[0, 0], a[0, 1], b[0, 1]])
    np.testing.assert_array_equal(o1[0], [a[0, 2], b[0, 2], a[0, 3], b[0, 3]])


# ---- depthwise convolution (section 6, the EfficientNet fragment) ----

def test_depthwise_convolution_worked_by_hand():
    # one channel, 3 x 3 image 1..9, kernel with nine different weights: correlation (not flipped), zero padding
    x = np.arange(1.0, 10.0).reshape(1, 3, 3, 1)
    k = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0], [7.0, 8.0, 9.0]]).reshape(3, 3, 1)
    y = orc.dwconv2d_nhwc(x, k)[0, :, :, 0]
    # centre: sum_{a,b} k[a,b] x[a,b] = 1*1 + 2*2 + ... + 9*9 = 285
    assert y[1, 1] == 285.0
    # top-left output sees x[0:2, 0:2] under k[1:3, 1:3]: 5*1 + 6*2 + 8*4 + 9*5 = 94
    assert y[0, 0] == 94.0
    # bottom-right output sees x[1:3, 1:3] under k[0:2, 0:2]: 1*5 + 2*6 + 4*8 + 5*9 = 94
    assert y[2, 2] == 94.0
    # top-right: x[0:2, 1:3] under k[1:3, 0:2]: 4*2 + 5*3 + 7*5 + 8*6 = 106 ; bottom-left: x[1:3,0:2] under k[0:2,1:3]
    assert y[0, 2] == 106.0 and y[2, 0] == 2 * 4 + 3 * 5 + 5 * 7 + 6 * 8
    # a kernel that is 1 at (row 0, col 1) reads the pixel above: y[i, j] = x[i - 1, j], zero in the first row
    k = np.zeros((3, 3, 1))
    k[0, 1, 0] = 1.0
    y = orc.dwconv2d_nhwc(x, k)[0, :, :, 0]
    np.testing.assert_array_equal(y, [[0, 0, 0], [1, 2, 3], [4, 5, 6]])
    # ... and at (row 1, col 2) the pixel to the right
    k = np.zeros((3, 3, 1))
    k[1, 2, 0] = 1.0
    np.testing.assert_array_equal(orc.dwconv2d_nhwc(x, k)[0, :, :, 0], [[2, 3, 0], [5, 6, 0], [8, 9, 0]])


def test_depthwise_convolution_against_library_and_invariants():
    rng = np.random.default_rng(31)
    for kh, kw in ((3, 3), (5, 5), (1, 3)):
        x = rng.standard_normal((2, 7, 6, 5))
        k = rng.standard_normal((kh, kw, 5))
        y = orc.dwconv2d_nhwc(x, k)
        ref = torch.nn.functional.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2), torch.from_numpy(k).permute(2, 0, 1)[:, None],
                                         padding=(kh // 2, kw // 2), groups=5).permute(0, 2, 3, 1).numpy()
        np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)
        # channels do not mix: changing one channel of x changes only that channel of y
        x2 = x.copy()
        x2[..., 3] += 1.0
        d = orc.dwconv2d_nhwc(x2, k) - y
        assert np.abs(d[..., [0, 1, 2, 4]]).max() == 0.0 and np.abs(d[..., 3]).max() > 0.0
    # the centre-one kernel is the identity
    k = np.zeros((3, 3, 5))
    k[1, 1] = 1.0
    np.testing.assert_array_equal(orc.dwconv2d_nhwc(x, k), x)
    # the chain RELU -> dwconv -> + bias pads with zeros AFTER the activation
    spec, ins = wl.x4_relu_dwconv(n=1, h=4, w=5, c=8, dtype="f32")
    xs, ws, bs = [wl.widen(t) for t in ins]
    got = orc.evaluate_outputs(spec, [xs, ws, bs])[0]
    np.testing.assert_allclose(got, orc.dwconv2d_nhwc(np.maximum(xs, 0.0), ws) + bs, rtol=1e-14)


def test_strided_depthwise_convolution():
    # worked by hand: 4 x 5 image 1..20, one channel, stride 2, the kernel that reads the pixel to the left
    x = np.arange(1.0, 21.0).reshape(1, 4, 5, 1)
    k = np.zeros((3, 3, 1))
    k[1, 0, 0] = 1.0
    y = orc.dwconv2d_nhwc(x, k, stride=2)
    assert y.shape == (1, 2, 3, 1)                       # (4 - 1) // 2 + 1, (5 - 1) // 2 + 1
    # outputs sit at input positions (0, 0), (0, 2), (0, 4), (2, 0), (2, 2), (2, 4); each reads column j - 1
    np.testing.assert_array_equal(y[0, :, :, 0], [[0, 2, 4], [0, 12, 14]])
    # all-ones 3 x 3 kernel: sums of the 3 x 3 neighbourhoods of those positions (zero outside the image)
    y = orc.dwconv2d_nhwc(x, np.ones((3, 3, 1)), stride=2)[0, :, :, 0]
    assert y[0, 0] == 1 + 2 + 6 + 7 and y[1, 1] == 7 + 8 + 9 + 12 + 13 + 14 + 17 + 18 + 19 and y[1, 2] == 9 + 10 + 14 + 15 + 19 + 20
    rng = np.random.default_rng(33)
    for (kh, kw), stride, (h, w) in (((3, 3), 2, (7, 6)), ((5, 5), 2, (8, 9)), ((3, 3), 3, (7, 7)), ((5, 5), 1, (6, 5))):
        x = rng.standard_normal((2, h, w, 4))
        k = rng.standard_normal((kh, kw, 4))
        y = orc.dwconv2d_nhwc(x, k, stride=stride)
        # a strided result is the dense one sampled at every stride-th position (same padding, same taps)
        np.testing.assert_array_equal(y, orc.dwconv2d_nhwc(x, k)[:, ::stride, ::stride, :])
        # and the library's grouped convolution agrees
        ref = torch.nn.functional.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2), torch.from_numpy(k).permute(2, 0, 1)[:, None],
                                         stride=stride, padding=(kh // 2, kw // 2), groups=4).permute(0, 2, 3, 1).numpy()
        np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)
    # through the chain walker: the attribute i[0] is the stride
    x = rng.standard_normal((2, 8, 9, 4))
    k = rng.standard_normal((5, 5, 4))
    spec = wl.ChainSpec(inputs=[("f32", (2, 8, 9, 4)), ("f32", (5, 5, 4))])
    spec.out(spec.op("dwconv2d", spec.op("relu", 0), 1, i=[2]), "f32")
    (got,) = orc.evaluate_outputs(spec, [x, k])
    np.testing.assert_array_equal(got, orc.dwconv2d_nhwc(np.maximum(x, 0.0), k, stride=2))


def test_reduction_over_other_dimensions():
    # spatial pooling of a channels-last tensor: reduce over H and W, keep N and C
    rng = np.random.default_rng(41)
    x = rng.standard_normal((2, 3, 4, 5))
    s = orc.reduce_axes("reduce_sum", x, [1, 2])
    assert s.shape == (2, 1, 1, 5)
    for n in range(2):
        for c in range(5):
            acc = 0.0
            for h in range(3):
                for w in range(4):
                    acc += x[n, h, w, c]
            assert abs(s[n, 0, 0, c] - acc) < 1e-13
    np.testing.assert_allclose(orc.reduce_axes("reduce_mean", x, [1, 2]), x.mean(axis=(1, 2), keepdims=True), rtol=0, atol=1e-14)
    np.testing.assert_array_equal(orc.reduce_axes("reduce_max", x, [2, 1]), x.max(axis=(1, 2), keepdims=True))
    # a single middle dimension, and the last dimension named explicitly (equals the default)
    np.testing.assert_allclose(orc.reduce_axes("reduce_sum", x, [2]), x.sum(axis=2, keepdims=True), rtol=0, atol=1e-14)
    np.testing.assert_array_equal(orc.reduce_axes("reduce_mean", x, [3]), orc.reduce_last("reduce_mean", x))
    # the mean of a tensor that is constant along the pooled dimensions is that constant, for every channel
    y = np.broadcast_to(np.arange(5.0), (2, 3, 4, 5))
    np.testing.assert_array_equal(orc.reduce_axes("reduce_mean", y, [1, 2])[1, 0, 0], np.arange(5.0))
    with pytest.raises(ValueError):
        orc.reduce_axes("reduce_sum", x, [1, 1])
    with pytest.raises(ValueError):
        orc.reduce_axes("reduce_sum", x, [4])
    # through the chain walker: i = the dimensions to reduce
    spec = wl.ChainSpec(inputs=[("f32", (2, 3, 4, 5))])
    spec.out(spec.op("reduce_mean", spec.op("relu", 0), i=[1, 2]), "f32")
    (got,) = orc.evaluate_outputs(spec, [x])
    np.testing.assert_allclose(got, np.maximum(x, 0).mean(axis=(1, 2), keepdims=True), rtol=0, atol=1e-14)


# ---- the broadcast basic operator with extents of 1 anywhere (paper section 6)

def test_broadcast_to_against_explicit_loops():
    rng = np.random.default_rng(77)
    v = rng.standard_normal((2, 1, 3, 1))
    out = orc.broadcast_to(v, (2, 4, 3, 5))
    assert out.shape == (2, 4, 3, 5) and out.flags["C_CONTIGUOUS"]
    for b in range(2):
        for h in range(4):
            for i in range(3):
                for j in range(5):
                    assert out[b, h, i, j] == v[b, 0, i, 0]
    # a lower-rank operand is aligned at the last dimension
    w = rng.standard_normal((3, 1))
    out = orc.broadcast_to(w, (2, 4, 3, 5))
    for b in range(2):
        for h in range(4):
            for i in range(3):
                for j in range(5):
                    assert out[b, h, i, j] == w[i, 0]
    with pytest.raises(ValueError):
        orc.broadcast_to(rng.standard_normal((2, 3)), (2, 4, 3, 5))      # 2 is neither 3 nor 1
    with pytest.raises(ValueError):
        orc.broadcast_to(rng.standard_normal((1, 2, 4, 3, 5)), (2, 4, 3, 5))   # more dimensions than the target
    out = orc.broadcast_to(rng.standard_normal((4, 1, 1)), (2, 4, 3, 5))       # aligned at the right: 4 meets 4
    assert out.shape == (2, 4, 3, 5) and np.all(out[0] == out[1]) and np.all(out[:, :, :1, :1] == out)


def test_binary_operator_with_a_mask_broadcast_over_heads_and_rows():
    # scores [B, H, S, S] + mask [B, 1, 1, S]: the padding mask of an encoder, added before the softmax
    rng = np.random.default_rng(78)
    B, H, S = 2, 3, 4
    a = rng.standard_normal((B, H, S, S))
    m = rng.standard_normal((B, 1, 1, S))
    out = orc.ew_binary("add", a, m)
    rev = orc.ew_binary("sub", m, a)                 # operand order is kept when the first operand is the small one
    for b in range(B):
        for h in range(H):
            for i in range(S):
                for j in range(S):
                    assert out[b, h, i, j] == a[b, h, i, j] + m[b, 0, 0, j]
                    assert rev[b, h, i, j] == m[b, 0, 0, j] - a[b, h, i, j]
    # [B, 1, S, 1]: one value per (batch, row), shared by heads and columns
    r = rng.standard_normal((B, 1, S, 1))
    out = orc.ew_binary("mul", a, r)
    for b in range(B):
        for h in range(H):
            for i in range(S):
                for j in range(S):
                    assert out[b, h, i, j] == a[b, h, i, j] * r[b, 0, i, 0]
    # the chain walker takes the same path
    spec = wl.ChainSpec(inputs=[("f32", (B, H, S, S)), ("f32", (B, 1, 1, S))])
    spec.out(spec.op("softmax", spec.op("add", 0, 1)), "f32")
    (y,) = orc.evaluate_outputs(spec, [a, m])
    e = np.exp((a + m) - (a + m).max(-1, keepdims=True))
    np.testing.assert_allclose(y, e / e.sum(-1, keepdims=True), rtol=0, atol=1e-15)
