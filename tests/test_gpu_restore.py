"""GPU parity of the restore side: inshr_dequantize and inshr_reconstruct (through the C ABI)
against the CPU oracle, bit for bit, and the round trips the two sides must close:
reconstruct(prev, delta(prev, cur)) gives the bytes of cur's codes, and the squared error of the
dequantized tensor is the one the search reported for the configuration."""
import os

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2306_11800_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2306_11800_amd import api
    c = api.Context(torch.device("cuda:0"))
    yield c
    c.close()


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


def u64(t):
    return t.cpu().numpy().view(np.uint64)


def ragged_batch(seed):
    rng = np.random.default_rng(seed)
    sizes = [1, 2, 63, 64, 65, 257, 4096, 12287, 12288, 12289, 16383, 16384, 16385, 50_000,
             786_432, 786_433, 1_000_003]
    prevs = [(0.02 * rng.standard_t(4, n)).astype(np.float32) for n in sizes]
    curs = [(p + rng.normal(0, 2e-4, p.size)).astype(np.float32) for p in prevs]
    return prevs, curs


CFGS = [(4, 100000, 1000), (8, 0, 0), (1, 0, 0), (2, 300000, 5000), (6, 0, 1000), (3, 500000, 0)]


def test_dequantize_matches_the_oracle(ctx):
    prevs, _ = ragged_batch(31)
    ts = [dev(x) for x in prevs]
    for cfg in CFGS:
        qs = ctx.quantize(ts, [cfg] * len(ts))
        outs = ctx.dequantize(qs)
        for q, x, got in zip(qs, prevs, outs):
            r = ref.quantize(x, cfg)
            # the oracle decodes its own symbols with the centres the HIP path stored, so that the
            # comparison is bit for bit (the centres themselves are compared elsewhere, to 1e-6)
            want = ref.dequantize(r["sym"], cfg[0], q.codebook.cpu().numpy(), r["outlier_idx"],
                                  r["outlier_val"])
            assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32)), (cfg, x.size)


def test_dequantized_error_is_the_searched_score(ctx):
    prev, _ = synth.config0(seed=33, n=1_500_001)
    grid = synth.grid_small()
    t = [dev(prev)]
    best, feas, scores = ctx.search(t, grid, synth.EPS_DEFAULT)
    for g, cfg in enumerate(grid):
        q = ctx.quantize(t, [cfg], reuse_search=True)
        xh = ctx.dequantize(q)[0].cpu().numpy().astype(np.float64)
        sse = float(((prev.astype(np.float64) - xh) ** 2).sum())
        s = scores[g]
        # the centres are rounded to fp32 before decoding; the score uses them unrounded
        assert abs(sse - s.sse) <= 1e-5 * s.sse + 1e-12 * s.sumsq, (cfg, sse, s.sse)


def test_reconstruct_matches_the_oracle_and_closes_the_round_trip(ctx):
    prevs, curs = ragged_batch(32)
    tp, tc = [dev(x) for x in prevs], [dev(x) for x in curs]
    for cp, cc in [((4, 100000, 1000), (4, 100000, 1000)), ((2, 100000, 1000), (8, 0, 0)),
                   ((8, 300000, 1000), (3, 0, 0)), ((1, 0, 0), (1, 0, 0)), ((8, 0, 0), (8, 0, 1000))]:
        qp = ctx.quantize(tp, [cp] * len(tp))
        qc = ctx.quantize(tc, [cc] * len(tc))
        ds = ctx.delta(qp, qc)
        ctx.sync()
        rec = ctx.reconstruct(qp, ds, [cc[0]] * len(tp))
        for i, (xp, xc) in enumerate(zip(prevs, curs)):
            assert torch.equal(rec[i], qc[i].packed), (cp, cc, xp.size)
            if xp.size <= 50_000:  # the oracle's own reconstruction from the oracle's own stream
                rp, rc = ref.quantize(xp, cp), ref.quantize(xc, cc)
                rd = ref.delta(rp["sym"], cp[0], rc["sym"], cc[0])
                want = ref.reconstruct(rp["sym"], cp[0], cc[0], rd["group_off"], rd["stream"])
                assert np.array_equal(u64(rec[i]), ref.pack(want, cc[0] + 1)), (cp, cc, xp.size)


def test_reconstruct_without_lane_ordered_lds_atomics(monkeypatch):
    from paper_2306_11800_amd import api
    with monkeypatch.context() as m:
        m.setenv("INSHR_NO_LDS_ORDER", "1")
        c = api.Context(torch.device("cuda:0"))
    prev, cur = synth.config0(seed=34, n=900_001)
    qp = c.quantize([dev(prev)], [(5, 100000, 1000)])
    qc = c.quantize([dev(cur)], [(4, 100000, 1000)])
    ds = c.delta(qp, qc)
    c.sync()
    rec = c.reconstruct(qp, ds, [4])
    assert torch.equal(rec[0], qc[0].packed)
    c.close()


def test_restore_errors(ctx):
    from paper_2306_11800_amd import api
    prev, cur = synth.config0(seed=35, n=100_000)
    qp = ctx.quantize([dev(prev)], [(4, 100000, 1000)])
    qc = ctx.quantize([dev(cur)], [(4, 100000, 1000)])
    ds = ctx.delta(qp, qc)
    ctx.sync()
    # group offsets that do not belong to the previous codes
    good = ds[0].group_off.clone()
    ds[0].group_off[3] += 1
    with pytest.raises(api.InshrError) as e:
        ctx.reconstruct(qp, ds, [4])
    assert e.value.code == -5
    ds[0].group_off.copy_(good)
    # a stream of all ones holds deltas >= B
    stream = ds[0].packed.clone()
    ds[0].packed.fill_(-1)
    with pytest.raises(api.InshrError) as e:
        ctx.reconstruct(qp, ds, [4])
    assert e.value.code == -1
    ds[0].packed.copy_(stream)
    assert torch.equal(ctx.reconstruct(qp, ds, [4])[0], qc[0].packed)
    # wrong width of the deltas
    ds[0].delta_bits = 6
    with pytest.raises(api.InshrError) as e:
        ctx.reconstruct(qp, ds, [4])
    assert e.value.code == -2
    # protected list that does not match the symbols
    n_out = qp[0].n_outlier
    assert n_out > 2
    qp[0].n_outlier = n_out - 1
    with pytest.raises(api.InshrError) as e:
        ctx.dequantize(qp)
    assert e.value.code == -5
    qp[0].n_outlier = n_out
    idx = qp[0].outlier_idx.clone()
    qp[0].outlier_idx[1] = qp[0].outlier_idx[0]
    with pytest.raises(api.InshrError) as e:
        ctx.dequantize(qp)
    assert e.value.code == -5
    qp[0].outlier_idx.copy_(idx)
    ctx.dequantize(qp)
