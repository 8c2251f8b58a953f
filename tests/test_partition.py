"""Host-side pins of the merge-plan search for chains that need several kernels (section 6, graph merging with a
performance model): the split returned is the cheapest of all splits under the exported cost function (brute
force over every set of cut points), a segment's bytes are what its tensors add up to, and chains of one kernel
stay whole."""
import itertools

import pytest

import workloads as wl
from paper_2307_04995_amd import binding as pf


def _convnext_norm(n, c, h, w, dtype, activation=True):
    s = wl.ChainSpec(inputs=[(dtype, (n, c, h, w)), (dtype, (c,)), (dtype, (c,))])
    v = s.op("permute", 0, i=[0, 2, 3, 1])
    v = s.op("layernorm", s.op("silu", v) if activation else v, 1, 2, f=[2.0 ** -20])
    v = s.op("permute", v, i=[0, 3, 1, 2])
    s.out(v, dtype)
    return s


def _brute_force(desc, n_ops):
    best = None
    for r in range(n_ops):
        for cuts in itertools.combinations(range(1, n_ops), r):
            edges = [0] + list(cuts) + [n_ops]
            total, ok = 0.0, True
            for a, b in zip(edges[:-1], edges[1:]):
                st, us, _ = pf.pf_chain_segment_cost(desc, a, b)
                if st != pf.PF_OK:
                    ok = False
                    break
                total += us
            if ok and (best is None or total < best - 1e-12):
                best = total
    return best


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_layout_norm_layout_is_three_kernels_with_the_bytes_of_its_tensors(dtype):
    n, c, h, w = 8, 96, 56, 56
    d = pf.make_desc(_convnext_norm(n, c, h, w, dtype))
    st, parts = pf.pf_chain_partition(d)
    assert st == pf.PF_OK
    assert [(a, b) for a, b, _, _ in parts] in ([(0, 2), (2, 3), (3, 4)], [(0, 1), (1, 3), (3, 4)])  # the activation goes with either neighbour
    # every kernel moves fp32 tensors, whatever the storage type: a split chain rounds once, at its end
    t = n * c * h * w * 4
    want = [2 * t, 2 * t + 2 * c * 4, 2 * t]
    if dtype == "f16":
        # ... and the copies that widen the inputs (2 bytes read, 4 written per element) and round the output are
        # priced with the first and the last kernel
        want[0] += (n * c * h * w + 2 * c) * 6
        want[2] += n * c * h * w * 6
    assert [nb for _, _, _, nb in parts] == want
    for a, b, us, nb in parts:
        st, us2, nb2 = pf.pf_chain_segment_cost(d, a, b)
        assert st == pf.PF_OK and us2 == us and nb2 == nb
        assert us > nb / 8.0e6  # never below the time the bytes take at the memory's peak rate


def test_layout_changes_that_cancel_around_a_normalisation_are_one_kernel():
    # exactly: move the channels to the end, normalise, move them back -- a normalisation over a strided dimension
    n, c, h, w = 8, 96, 56, 56
    d = pf.make_desc(_convnext_norm(n, c, h, w, "f16", activation=False))
    st, parts = pf.pf_chain_partition(d)
    assert st == pf.PF_OK and [(a, b) for a, b, _, _ in parts] == [(0, 3)]
    assert parts[0][3] == 2 * n * c * h * w * 2 + 2 * c * 2


def test_a_chain_of_one_kernel_stays_whole():
    s = wl.ChainSpec(inputs=[("f16", (4, 64, 256)), ("f16", (256,))])
    s.out(s.op("silu", s.op("softmax", s.op("add", 0, 1))), "f16")
    st, parts = pf.pf_chain_partition(pf.make_desc(s))
    assert st == pf.PF_OK and [(a, b) for a, b, _, _ in parts] == [(0, 3)]


def test_a_row_statistic_crosses_the_cut_instead_of_the_tensor():
    # x -> softmax -> (row maximum -> sigmoid) -> y * that -> RMS normalisation: cutting after the statistic moves
    # one value per row, cutting before it moves the whole tensor once more
    r, c = 4096, 512
    s = wl.ChainSpec(inputs=[("f32", (r, c)), ("f32", (r, c)), ("f32", (c,))])
    p = s.op("softmax", 0)
    m = s.op("sigmoid", s.op("reduce_max", p))
    v = s.op("rmsnorm", s.op("mul", 1, m), 2, f=[2.0 ** -20])
    s.out(v, "f32")
    d = pf.make_desc(s)
    st, parts = pf.pf_chain_partition(d)
    assert st == pf.PF_OK, pf._lib.pf_last_error()
    total = sum(us for _, _, us, _ in parts)
    assert abs(total - _brute_force(d, len(s.ops))) < 1e-9
    # the tensor of probabilities is written once and read once; no kernel reads it a second time
    assert sum(nb for _, _, _, nb in parts) <= (2 + 2 + 1) * r * c * 4 + 4 * r * 4 + 2 * c * 4


@pytest.mark.parametrize("seed", range(40))
def test_the_split_is_the_cheapest_of_all_splits(seed):
    s, _, what = wl.random_multi_kernel_chain(seed)
    if len(s.ops) > 11:
        pytest.skip("brute force over more than 2^10 splits")
    d = pf.make_desc(s)
    st, parts = pf.pf_chain_partition(d)
    best = _brute_force(d, len(s.ops))
    if best is None:
        assert st != pf.PF_OK, what
        return
    assert st == pf.PF_OK, what
    assert len(parts) >= 1, what
    assert parts[0][0] == 0 and parts[-1][1] == len(s.ops) and all(a[1] == b[0] for a, b in zip(parts[:-1], parts[1:])), what
    assert abs(sum(us for _, _, us, _ in parts) - best) < 1e-9, what


def test_bad_ranges_are_refused():
    d = pf.make_desc(_convnext_norm(1, 8, 4, 4, "f32"))
    assert pf.pf_chain_segment_cost(d, 2, 2)[0] == pf.PF_ERR_INVALID_ARG
    assert pf.pf_chain_segment_cost(d, 0, 5)[0] == pf.PF_ERR_INVALID_ARG
    assert pf.pf_chain_segment_cost(d, 0, 3)[0] == pf.PF_ERR_UNSUPPORTED  # two exchanges: not one kernel
