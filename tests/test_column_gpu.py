"""GPU parity for the column family: layer / RMS normalisation over a dimension that is not the innermost, written
as `move it to the end -> normalise -> move it back` and run as one kernel without any layout change; element by
element against the fp64 oracle (which evaluates the three operators as written) through the C ABI."""
import numpy as np
import pytest
import torch

import workloads as wl
from pf_testlib import check_chain, env

pytestmark = pytest.mark.gpu


def _pf():
    from paper_2307_04995_amd import binding as pf
    return pf


def _chain(dtype, shape, axis, kind, eps=2.0 ** -16):
    rank = len(shape)
    c = shape[axis]
    to_end = [q for q in range(rank) if q != axis] + [axis]
    back = [to_end.index(q) for q in range(rank)]
    s = wl.ChainSpec(inputs=[(dtype, tuple(shape)), (dtype, (c,))] + ([(dtype, (c,))] if kind == "layernorm" else []))
    v = s.op("permute", 0, i=to_end)
    v = s.op("layernorm", v, 1, 2, f=[eps]) if kind == "layernorm" else s.op("rmsnorm", v, 1, f=[eps])
    s.out(s.op("permute", v, i=back), dtype)
    return s


def _inputs(dtype, shape, axis, kind, seed):
    c = shape[axis]
    t = [wl.random_tensor(tuple(shape), dtype, seed), wl.random_tensor((c,), dtype, seed + 1, dist="positive")]
    if kind == "layernorm":
        t.append(wl.random_tensor((c,), dtype, seed + 2, scale=0.3))
    return t


# channel counts on both sides of every registers-per-lane step (32, 64, 128, 512, 1024), positions with a partial
# last tile (the slab is 64 positions of 16-bit data, 32 of fp32), several outer indices, rank 3 to 5
SHAPES = [((2, 96, 7, 7), 1), ((1, 40, 14, 14), 1), ((3, 17, 5, 3), 1), ((2, 200, 6, 9), 1), ((2, 5, 3, 1), 1),  # positions that are not whole vectors
          ((2, 96, 56, 56), 1), ((3, 32, 8, 8), 1), ((1, 33, 72), 1), ((2, 64, 136), 1), ((2, 65, 40), 1), ((1, 128, 200), 1),
          ((1, 129, 64), 1), ((2, 320, 24), 1), ((1, 512, 16), 1), ((1, 513, 8), 1), ((1, 1024, 8), 1), ((2, 2, 64), 1),
          ((2, 3, 5, 7, 16), 2), ((4, 5, 6, 8), 0), ((2, 2, 24, 4, 4), 2)]


@pytest.mark.parametrize("kind", ["layernorm", "rmsnorm"])
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("shape,axis", SHAPES)
def test_normalisation_over_a_strided_dimension(shape, axis, dtype, kind):
    pf = _pf()
    s = _chain(dtype, shape, axis, kind)
    outs, info, _ = check_chain(s, _inputs(dtype, shape, axis, kind, 7100), what=f"{kind} over axis {axis} of {shape} {dtype}")
    assert info.family == pf.PF_FAMILY_COLUMN and info.n_kernels == 1 and info.n_launches == 1
    assert tuple(outs[0].shape) == tuple(shape)
    n = int(np.prod(shape)) * (4 if dtype == "f32" else 2)
    assert info.compulsory_read_bytes >= n and info.compulsory_write_bytes == n


def test_what_the_one_kernel_form_does_not_take_runs_as_three_kernels():
    pf = _pf()
    shape = (1, 1100, 16)  # more than 1024 values per position
    s = _chain("f16", shape, 1, "layernorm")
    _, info, _ = check_chain(s, _inputs("f16", shape, 1, "layernorm", 7200), what=f"{shape}")
    assert info.n_kernels == 3
    with env(PF_PARTITION="0"):  # with the split switched off the refusal names the reason
        with pytest.raises(pf.PfError) as e:
            pf.Plan(s, 0)
        assert e.value.status == pf.PF_ERR_UNSUPPORTED and "1024" in str(e.value)


def test_constant_positions_and_large_offsets():
    # a position whose values are all equal normalises to beta exactly; a large common offset does not cancel
    shape = (2, 48, 64)
    x = torch.full(shape, 3.0, dtype=torch.float32)
    x[1] = wl.random_tensor((48, 64), "f32", 7301) * 0.01 + 100.0
    gam = wl.random_tensor((48,), "f32", 7302, dist="positive")
    bet = wl.random_tensor((48,), "f32", 7303, scale=0.3)
    s = _chain("f32", shape, 1, "layernorm", eps=2.0 ** -10)
    outs, _, _ = check_chain(s, [x, gam, bet], what="constant positions, offset 100")
    assert torch.equal(outs[0][0], bet.reshape(48, 1).expand(48, 64))


def test_repeated_runs_and_in_place():
    pf = _pf()
    shape = (2, 40, 4, 16)
    s = _chain("f16", shape, 1, "rmsnorm")
    plan = pf.Plan(s, 0)
    gam = wl.random_tensor((40,), "f16", 7402, dist="positive").cuda()
    out = torch.empty(shape, dtype=torch.float16, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    from pf_testlib import compare, oracle_run
    for rep in range(3):
        x = wl.random_tensor(shape, "f16", 7410 + rep)
        xd = x.cuda()
        plan.run_ptrs([xd.data_ptr(), gam.data_ptr()], [out.data_ptr()], stream)
        torch.cuda.synchronize()
        compare(out.cpu(), oracle_run(s, [x, gam.cpu()])[0], "f16", f"run {rep}")
    # in place: a workgroup holds its whole slab before it stores any of it
    x = wl.random_tensor(shape, "f16", 7420)
    buf = x.cuda()
    plan.run_ptrs([buf.data_ptr(), gam.data_ptr()], [buf.data_ptr()], stream)
    torch.cuda.synchronize()
    compare(buf.cpu(), oracle_run(s, [x, gam.cpu()])[0], "f16", "in place")
    # a partial overlap is refused
    big = torch.empty(int(np.prod(shape)) + 64, dtype=torch.float16, device="cuda")
    with pytest.raises(pf.PfError) as e:
        plan.run_ptrs([big.data_ptr(), gam.data_ptr()], [big.data_ptr() + 64], stream)
    assert e.value.status == pf.PF_ERR_ALIAS
    plan.close()
