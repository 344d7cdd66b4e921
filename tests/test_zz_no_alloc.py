"""GPU: the delta entry point that allocates nothing (inshr_delta_static) against inshr_delta, bit
for bit, on two calls in a row, the second on a smaller input (the static scratch keeps the first
call's contents); its limits are reported as errors.  Collected last on purpose."""
import numpy as np
import pytest
import torch

from paper_2306_11800_amd import synth

pytestmark = pytest.mark.gpu


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


def same(a, b):
    assert a.delta_bits == b.delta_bits
    assert torch.equal(a.packed, b.packed)
    assert torch.equal(a.group_off, b.group_off)
    if a.perm is not None:
        assert torch.equal(a.perm, b.perm)


def test_no_alloc_delta_equals_delta_twice_in_a_row():
    from paper_2306_11800_amd import api
    ctx = api.Context(torch.device("cuda:0"))
    rng = np.random.default_rng(41)
    # first call: three tensors, several chunks and a ragged tail, unequal bits, one with a permutation
    sizes1 = [2_000_003, 786_432, 70_001]
    cfgp = [(8, 200000, 1000), (3, 0, 0), (5, 100000, 100)]
    cfgc = [(8, 200000, 1000), (6, 0, 1000), (5, 100000, 100)]
    prevs = [(0.015 * rng.standard_t(3, n)).astype(np.float32) for n in sizes1]
    curs = [(p + rng.normal(0, 1e-4, p.size)).astype(np.float32) for p in prevs]
    qp = ctx.quantize([dev(x) for x in prevs], cfgp)
    qc = ctx.quantize([dev(x) for x in curs], cfgc)
    want = ctx.delta(qp, qc)
    ctx.sync()
    got = ctx.delta(qp, qc)          # buffers of the same shapes, then overwritten
    ctx.sync()
    for g in got:
        g.packed.fill_(-1)
        g.goff_buf.fill_(-1)
    free0 = torch.cuda.mem_get_info()[0]
    ctx.delta_static(qp, qc, got)
    ctx.sync()
    assert torch.cuda.mem_get_info()[0] == free0  # nothing was allocated on the device
    for a, b in zip(got, want):
        same(a, b)
    # second call, smaller: one tensor of the first call's smallest shape, with its permutation
    qp2, qc2 = [qp[2]], [qc[2]]
    want2 = ctx.delta(qp2, qc2, want_perm=True)
    ctx.sync()
    got2 = ctx.delta(qp2, qc2, want_perm=True)
    ctx.sync()
    got2[0].packed.fill_(-1)
    got2[0].perm.fill_(-1)
    ctx.delta_static(qp2, qc2, got2)
    ctx.sync()
    same(got2[0], want2[0])
    # and the first again: the scratch carries nothing over
    for g in got:
        g.packed.fill_(-1)
    ctx.delta_static(qp, qc, got)
    ctx.sync()
    for a, b in zip(got, want):
        same(a, b)
    ctx.close()


def test_no_alloc_delta_limits():
    import ctypes as C
    from paper_2306_11800_amd import api
    ctx = api.Context(torch.device("cuda:0"))
    x = dev((0.02 * np.random.default_rng(42).standard_normal(5000)).astype(np.float32))
    q = ctx.quantize([x], [(4, 0, 0)])
    d = ctx.delta(q, q)
    ctx.sync()
    with pytest.raises(api.InshrError) as e:      # too many tensors
        ctx.delta_static(list(q) * 17, list(q) * 17, list(d) * 17)
    assert e.value.code == -4
    # too many elements: descriptors only, nothing is launched or dereferenced
    n_big = (1 << 32) - 1
    pa = (api.CCodes * 1)(api.CCodes(q[0]._ptrs[0], 5, 4, 0, n_big))
    oa = (api.CDeltaOut * 1)()
    oa[0].packed, oa[0].packed_words = d[0].packed.data_ptr(), (n_big * 5 + 63) // 64
    oa[0].group_off, oa[0].group_off_entries = d[0].goff_buf.data_ptr(), 259
    assert ctx.lib.inshr_delta_static(ctx.h, pa, pa, oa, 1) == -4
    assert b"chunks" in ctx.lib.inshr_last_device_error(ctx.h)
    ctx.close()
