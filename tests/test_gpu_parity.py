"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on the
same seeded inputs.  Bit-exact on thresholds, boundaries, symbols, protected lists, permutations,
delta streams, counts and chosen configurations; 1e-6 relative on centres and error sums (plus an
absolute floor of 1e-12 * sumsq on error sums, the fp64 rounding of sumsq - sum_bins(...))."""
import os

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2306_11800_amd import synth

pytestmark = pytest.mark.gpu

REL = 1e-6


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


def u32(t):
    return t.cpu().numpy().view(np.uint32)


def check_scores(gscores, nC, ti, x, grid, eps, gbest, gfeas, given=None):
    # given: what ref.search returned for this tensor, when the caller computed it beforehand
    rbest, rfeas, rsc = given if given is not None else ref.search(x, grid, eps)
    border = False
    for g in range(nC):
        s, r = gscores[ti * nC + g], rsc[g]
        assert (s.n_pruned, s.n_outlier, s.n_kept, s.cost_bits) == \
            (r["n_pruned"], r["n_outlier"], r["n_kept"], r["cost_bits"]), (ti, grid[g])
        assert abs(s.sumsq - r["sumsq"]) <= REL * r["sumsq"], (ti, grid[g])
        assert abs(s.sse - r["sse"]) <= REL * r["sse"] + 1e-12 * r["sumsq"], (ti, grid[g], s.sse, r["sse"])
        if r["sumsq"] > 0 and abs(r["sse"] / r["sumsq"] - eps) <= 4 * REL * eps:
            border = True
    if not border:
        assert (gbest, gfeas) == (rbest, rfeas), (ti, gbest, rbest)
    return rbest


def check_quantized(q, x, cfg, given=None):
    r = given if given is not None else ref.quantize(x, cfg)
    assert q.sym_bits == r["sym_bits"] and q.K == r["K"]
    assert (q.n_pruned, q.n_outlier, q.n_kept) == (r["n_pruned"], r["n_outlier"], r["n_kept"])
    assert np.float32(q.tau_prune).view(np.uint32) == r["tau_prune_bits"]
    assert np.float32(q.tau_outlier).view(np.uint32) == r["tau_outlier_bits"]
    assert np.array_equal(u32(q.boundaries), r["boundaries"].view(np.uint32)), cfg
    want = ref.pack(r["sym"], r["sym_bits"])
    got = u64(q.packed)
    if not np.array_equal(got, want):
        gs = ref.unpack(got, x.size, r["sym_bits"])
        bad = np.nonzero(gs != r["sym"])[0]
        raise AssertionError(f"symbols differ at {bad[:10]} ({bad.size} of {x.size}) cfg={cfg}: "
                             f"{gs[bad[:10]]} vs {r['sym'][bad[:10]]}")
    assert np.array_equal(u32(q.outlier_idx), r["outlier_idx"])
    assert np.array_equal(u32(q.outlier_val), r["outlier_val"].view(np.uint32))
    cb = q.codebook.cpu().numpy()
    np.testing.assert_allclose(cb, r["codebook"], rtol=REL, atol=0)
    return r


def check_delta(d, rp, bp, rc, bc, want_perm, given=None):
    # (bp, bc: bits of the two sides; the numbers of bins come with the references)
    rd = given if given is not None else ref.delta(rp["sym"], bp, rc["sym"], bc, K_prev=rp["K"], K_cur=rc["K"])
    assert d.delta_bits == rd["delta_bits"]
    assert np.array_equal(u64(d.group_off), rd["group_off"])
    want = ref.pack(rd["stream"], rd["delta_bits"])
    got = u64(d.packed)
    if not np.array_equal(got, want):
        gs = ref.unpack(got, rp["sym"].size, rd["delta_bits"])
        bad = np.nonzero(gs != rd["stream"])[0]
        raise AssertionError(f"delta stream differs at {bad[:10]} ({bad.size}): {gs[bad[:10]]} vs "
                             f"{rd['stream'][bad[:10]]}")
    if want_perm:
        assert np.array_equal(u32(d.perm), rd["perm"])


def run_pipeline(ctx, prevs, curs, grid, eps, want_perm=True, check_all_cfg_quantize=False):
    """search + quantize(prev), search + quantize(cur), delta; everything checked against the oracle."""
    nC = len(grid)
    results = []
    for xs in (prevs, curs):
        ts = [dev(x) for x in xs]
        best, feas, scores = ctx.search(ts, grid, eps)
        chosen = []
        for ti, x in enumerate(xs):
            rb = check_scores(scores, nC, ti, x, grid, eps, best[ti], feas[ti])
            chosen.append(grid[rb])
        qs = ctx.quantize(ts, chosen, reuse_search=True)
        refs = [check_quantized(q, x, c) for q, x, c in zip(qs, xs, chosen)]
        if check_all_cfg_quantize:
            for g in grid:
                qg = ctx.quantize(ts, [g] * len(ts), reuse_search=True)
                for q, x in zip(qg, xs):
                    check_quantized(q, x, g)
        results.append((qs, refs, chosen))
    (qp, rp, cp), (qc, rc, cc) = results
    ds = ctx.delta(qp, qc, want_perm=want_perm)
    ctx.sync()
    for i, d in enumerate(ds):
        check_delta(d, rp[i], cp[i][0], rc[i], cc[i][0], want_perm)
    return results, ds


def test_config0_small_grid(ctx):
    prev, cur = synth.config0(seed=0, n=1 << 20)
    run_pipeline(ctx, [prev], [cur], synth.grid_small(), synth.EPS_DEFAULT)


def test_every_config_quantizes_identically(ctx):
    prev, cur = synth.config0(seed=1, n=200_003)
    run_pipeline(ctx, [prev], [cur], synth.grid_small(), synth.EPS_DEFAULT, check_all_cfg_quantize=True)


def test_full_grid_ragged_batch(ctx):
    rng = np.random.default_rng(5)
    sizes = [1, 2, 63, 64, 65, 255, 256, 257, 1000, 4096, 16383, 16384, 16385, 50_000, 300_001]
    prevs = [(0.02 * rng.standard_t(4, n)).astype(np.float32) for n in sizes]
    curs = [(p + rng.normal(0, 1e-4, p.size)).astype(np.float32) for p in prevs]
    run_pipeline(ctx, prevs, curs, synth.grid_full(), synth.EPS_DEFAULT)


def test_degenerate_tensors(ctx):
    rng = np.random.default_rng(6)
    n = 40_000
    zeros95 = rng.normal(0, 1e-3, n).astype(np.float32)
    zeros95[rng.random(n) < 0.95] = 0.0
    negz = zeros95.copy()
    negz[::7] = -0.0
    few = rng.choice(np.array([-0.5, 0.1, 0.1, 0.7, 0.0, 3.0], np.float32), n)
    prevs = [np.full(5000, 0.25, np.float32), np.zeros(3000, np.float32), zeros95, negz, few,
             np.arange(1, 4097, dtype=np.float32),
             np.array([1e-45, -1e-45, 3e-39, -2e-39, 1e-38, 0.0, 1.0] * 50, np.float32),
             np.abs(rng.normal(0, 1e-6, n)).astype(np.float32)]
    curs = [p.copy() for p in prevs]
    curs[2] = (zeros95 + (rng.random(n) < 0.01) * rng.normal(0, 1e-3, n)).astype(np.float32)
    curs[4] = rng.choice(np.array([-0.5, 0.1, 0.7, 0.0, 3.0], np.float32), n)
    run_pipeline(ctx, prevs, curs, synth.grid_small(), synth.EPS_DEFAULT)


def test_standalone_quantize_matches_reuse(ctx):
    prev, _ = synth.config0(seed=2, n=150_000)
    x2 = (0.02 * np.random.default_rng(3).standard_t(4, 70_001)).astype(np.float32)
    ts = [dev(prev), dev(x2)]
    cfgs = [(4, 100000, 1000), (8, 0, 0)]
    qs = ctx.quantize(ts, cfgs, reuse_search=False)
    for q, x, c in zip(qs, [prev, x2], cfgs):
        check_quantized(q, x, c)
    # the same through a search over a grid that contains both
    grid = synth.grid_small()
    ctx.search(ts, grid, synth.EPS_DEFAULT)
    qr = ctx.quantize(ts, cfgs, reuse_search=True)
    for a, b in zip(qs, qr):
        assert torch.equal(a.packed, b.packed)
        assert torch.equal(a.boundaries, b.boundaries)
        assert torch.equal(a.outlier_idx, b.outlier_idx)
        np.testing.assert_allclose(a.codebook.cpu().numpy(), b.codebook.cpu().numpy(), rtol=REL)


def test_delta_unequal_bits_and_given_permutation(ctx):
    prev, cur = synth.config0(seed=4, n=123_457)
    tp, tc = [dev(prev)], [dev(cur)]
    for cp, cc in [((2, 100000, 1000), (8, 0, 0)), ((8, 300000, 1000), (3, 0, 0)), ((1, 0, 0), (1, 0, 0))]:
        qp = ctx.quantize(tp, [cp])
        qc = ctx.quantize(tc, [cc])
        rp, rc = ref.quantize(prev, cp), ref.quantize(cur, cc)
        d = ctx.delta(qp, qc, want_perm=True)
        ctx.sync()
        check_delta(d[0], rp, cp[0], rc, cc[0], True)
        # previous permutation handed back: same stream
        d2 = ctx.delta(qp, qc, want_perm=False, prev_perm=[d[0].perm])
        ctx.sync()
        assert torch.equal(d2[0].packed, d[0].packed)
        assert torch.equal(d2[0].group_off, d[0].group_off)
    # delta(prev, prev) is all zero
    qp = ctx.quantize(tp, [(4, 100000, 1000)])
    d = ctx.delta(qp, qp)
    ctx.sync()
    assert not d[0].packed.any()


def test_delta_of_codes_at_8_byte_aligned_addresses(ctx):
    """The packed symbols may sit at any 8-byte aligned address (the fast copy into LDS wants 16)."""
    from paper_2306_11800_amd import api
    prev, cur = synth.config0(seed=21, n=100_003)
    cfg = (6, 100000, 1000)
    ts = [dev(prev), dev(cur)]
    q = ctx.quantize(ts, [cfg, cfg])
    shifted = []
    for x in q:
        words = x.packed.numel()
        big = torch.empty(words + 3, dtype=torch.int64, device="cuda:0")
        view = big[1:1 + words]
        assert view.data_ptr() % 16 == 8
        view.copy_(x.packed)
        y = api.Quantized(x.n, x.bits, (view,) + tuple(x._bufs[1:]))
        shifted.append(y)
    d = ctx.delta([shifted[0]], [shifted[1]], want_perm=True)
    ctx.sync()
    rp, rc = ref.quantize(prev, cfg), ref.quantize(cur, cfg)
    check_delta(d[0], rp, cfg[0], rc, cfg[0], True)
    d = ctx.delta([shifted[0]], [shifted[1]], want_perm=False)
    ctx.sync()
    check_delta(d[0], rp, cfg[0], rc, cfg[0], False)


def test_errors(ctx):
    from paper_2306_11800_amd import api
    x = np.ones(1000, np.float32)
    for bad in (np.nan, np.inf):
        y = x.copy()
        y[17] = bad
        with pytest.raises(api.InshrError) as e:
            ctx.search([dev(y)], synth.grid_small(), 0.01)
        assert e.value.code == -3
    with pytest.raises(api.InshrError) as e:
        ctx.search([dev(x)], [(9, 0, 0)], 0.01)
    assert e.value.code == -2
    with pytest.raises(api.InshrError) as e:
        ctx.search([dev(x)], [(4, 600000, 400000)], 0.01)
    assert e.value.code == -2
    with pytest.raises(api.InshrError) as e:
        ctx.quantize([dev(x)], [(4, 0, 0)], reuse_search=True)  # no matching search (last one failed)
    assert e.value.code == -5
    # still usable afterwards
    best, feas, _ = ctx.search([dev(x)], synth.grid_small(), 0.01)
    assert feas == [1]


def test_heavy_duplicates_exceed_the_lds_sort(ctx):
    """A few distinct values, each held by far more elements than one group sort takes in LDS:
    the boundaries are then selected from device memory."""
    rng = np.random.default_rng(11)
    n = 150_000
    vals = np.array([-0.5, 0.1, 0.1000001, 0.7, 0.0, 3.0], np.float32)
    prev = rng.choice(vals, n)
    cur = prev.copy()
    flip = rng.random(n) < 0.02
    cur[flip] = rng.choice(vals, int(flip.sum()))
    mixed = np.concatenate([prev[:60_000], (0.01 * rng.standard_normal(60_000)).astype(np.float32)])
    run_pipeline(ctx, [prev, mixed], [cur, mixed.copy()], synth.grid_small(), synth.EPS_DEFAULT)


def test_protected_values_in_the_last_lanes_of_a_ragged_tile(ctx):
    """The protected values sit at the very end of a tensor whose last tile misses one element, so
    that the last lane of the last wave sees fewer valid elements than its neighbours."""
    rng = np.random.default_rng(13)
    n = 2 * 16384 - 1
    prev = (0.01 * rng.standard_normal(n)).astype(np.float32)
    prev[-40:] = ((10.0 + np.arange(40)) * np.where(np.arange(40) % 3 == 0, -1.0, 1.0)).astype(np.float32)
    cur = prev.copy()
    cur[:1000] += (1e-4 * rng.standard_normal(1000)).astype(np.float32)
    run_pipeline(ctx, [prev], [cur], synth.grid_small(), synth.EPS_DEFAULT)


def test_without_lane_ordered_lds_atomics(monkeypatch):
    """The group sort and the delta scatter have a ballot-based path for devices whose LDS atomics
    do not return in lane order; INSHR_NO_LDS_ORDER=1 selects it."""
    from paper_2306_11800_amd import api
    with monkeypatch.context() as m:  # (whatever the variable was before comes back afterwards)
        m.setenv("INSHR_NO_LDS_ORDER", "1")
        c = api.Context(torch.device("cuda:0"))
    assert c.lds_ordered is False
    rng = np.random.default_rng(12)
    prev, cur = synth.config0(seed=3, n=250_007)
    few = rng.choice(np.array([-0.5, 0.1, 0.7, 0.0, 3.0], np.float32), 30_000)
    run_pipeline(c, [prev, few], [cur, few.copy()], synth.grid_small(), synth.EPS_DEFAULT)
    c.close()


def test_deterministic_bytes(ctx):
    prev, cur = synth.config0(seed=9, n=300_000)
    outs = []
    for _ in range(2):
        ts = [dev(prev)]
        ctx.search(ts, synth.grid_small(), 0.01)
        q = ctx.quantize(ts, [(4, 100000, 1000)], reuse_search=True)[0]
        outs.append((q.packed.clone(), q.boundaries.clone(), q.outlier_idx.clone()))
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)


def test_reused_batches_give_the_same_bytes(ctx):
    """Lists that carry their marshalled C arrays (Context.batch, out= of quantize and delta) against
    plain lists, over steps whose configurations differ."""
    rng = np.random.default_rng(41)
    xs = [(0.02 * rng.standard_t(4, n)).astype(np.float32) for n in (70_001, 16384, 300_000)]
    ys = [(x + rng.normal(0, 2e-4, x.size)).astype(np.float32) for x in xs]
    tp, tc = [dev(x) for x in xs], [dev(y) for y in ys]
    qp = ctx.quantize(tp, [(8, 0, 1000)] * 3)
    cb = ctx.batch(tc)
    q_re = ctx.quantize(cb, [(8, 0, 1000)] * 3)      # sizes the buffers
    d_re = ctx.delta(qp, q_re)
    ctx.sync()
    for cfgs in ([(4, 100000, 1000), (8, 0, 0), (2, 300000, 100)], [(8, 200000, 1000)] * 3,
                 [(3, 0, 0), (5, 50000, 1000), (8, 0, 1000)]):
        q_re2 = ctx.quantize(cb, cfgs, out=q_re)
        assert q_re2 is q_re
        d_re2 = ctx.delta(qp, q_re, out=d_re)
        assert d_re2 is d_re
        ctx.sync()
        q_pl = ctx.quantize(tc, cfgs)
        d_pl = ctx.delta(qp, q_pl)
        ctx.sync()
        for a, b, da, db in zip(q_re, q_pl, d_re, d_pl):
            assert (a.bits, a.sym_bits, a.n_pruned, a.n_outlier, a.n_kept) == \
                (b.bits, b.sym_bits, b.n_pruned, b.n_outlier, b.n_kept)
            assert (a.tau_prune, a.tau_outlier) == (b.tau_prune, b.tau_outlier)
            assert torch.equal(a.packed, b.packed) and torch.equal(a.codebook, b.codebook)
            assert torch.equal(a.outlier_idx, b.outlier_idx) and torch.equal(a.outlier_val, b.outlier_val)
            assert da.delta_bits == db.delta_bits
            words = (da.n * da.delta_bits + 63) // 64
            assert torch.equal(da.packed[:words], db.packed[:words])
            assert torch.equal(da.group_off, db.group_off)


def test_group_offsets_follow_a_prev_that_changes_bits(ctx):
    """delta(..., out=) after the previous codes were quantized again in place with other bits: the
    group offsets have (1 << bits) + 3 entries, and their buffer has room for any bits."""
    from paper_2306_11800_amd import api
    prev, cur = synth.config0(seed=31, n=90_001)
    tp, tc = [dev(prev)], [dev(cur)]
    qp = ctx.quantize(tp, [(8, 0, 1000)])
    qc = ctx.quantize(tc, [(3, 0, 1000)])
    r3, r8, rc = ref.quantize(prev, (3, 0, 1000)), ref.quantize(prev, (8, 0, 1000)), ref.quantize(cur, (3, 0, 1000))
    d = ctx.delta(qp, qc)                           # stream sized for 9-bit deltas
    ctx.sync()
    check_delta(d[0], r8, 8, rc, 3, False)
    for bits, r in ((3, r3), (8, r8), (3, r3)):
        qp = ctx.quantize(tp, [(bits, 0, 1000)], out=qp)  # the same list, other symbols
        d = ctx.delta(qp, qc, out=d)
        ctx.sync()
        assert d[0].group_off.numel() == (1 << bits) + 3
        words = (prev.size * d[0].delta_bits + 63) // 64  # (the stream's buffer keeps its first size)
        view = api.Delta(d[0].n, d[0].delta_bits, d[0].packed[:words], d[0].group_off, None)
        check_delta(view, r, bits, rc, 3, False)


def test_stated_group_offset_capacity_is_checked(ctx):
    import ctypes as C
    from paper_2306_11800_amd import api
    prev, cur = synth.config0(seed=32, n=10_000)
    qp = ctx.quantize([dev(prev)], [(8, 0, 0)])
    qc = ctx.quantize([dev(cur)], [(8, 0, 0)])
    pa = (api.CCodes * 1)(api.CCodes(qp[0]._ptrs[0], 9, 8, 0, 10_000))
    ca = (api.CCodes * 1)(api.CCodes(qc[0]._ptrs[0], 9, 8, 0, 10_000))
    out = torch.empty(2000, dtype=torch.int64, device="cuda:0")
    goff = torch.empty(259, dtype=torch.int64, device="cuda:0")
    oa = (api.CDeltaOut * 1)()
    oa[0].packed, oa[0].packed_words, oa[0].group_off = out.data_ptr(), out.numel(), goff.data_ptr()
    oa[0].group_off_entries = 19  # enough for 4 bits, not for 8
    assert ctx.lib.inshr_delta(ctx.h, pa, None, ca, oa, 1) == -4
    oa[0].group_off_entries = 259
    assert ctx.lib.inshr_delta(ctx.h, pa, None, ca, oa, 1) == 0
    ctx.sync()


def test_foreign_permutation_is_reported_not_followed(ctx):
    """A permutation that does not belong to the tensor (indices beyond n): the gather skips those
    elements, and the next synchronisation returns INSHR_E_ARG."""
    from paper_2306_11800_amd import api
    prev, cur = synth.config0(seed=33, n=50_000)
    qp = ctx.quantize([dev(prev)], [(4, 0, 0)])
    qc = ctx.quantize([dev(cur)], [(4, 0, 0)])
    d = ctx.delta(qp, qc, want_perm=True)
    ctx.sync()
    bad = d[0].perm.clone()
    bad[123] = 50_000       # one past the end
    bad[40_000] = -1        # 0xFFFFFFFF
    ctx.delta(qp, qc, prev_perm=[bad])
    with pytest.raises(api.InshrError) as e:
        ctx.sync()
    assert e.value.code == -1
    ctx.sync()  # reported once
    d2 = ctx.delta(qp, qc, prev_perm=[d[0].perm])  # the context works on
    ctx.sync()
    assert torch.equal(d2[0].packed, d[0].packed)


def test_ranking_path_is_reported(ctx):
    # returning LDS adds rank equal symbols on this device unless the environment forbids them
    forced_off = any(os.environ.get(k, "0") not in ("", "0") for k in ("INSHR_NO_LDS_ORDER", "INSHR_DELTA_SLOTS"))
    assert ctx.lds_ordered == (not forced_off)


def test_scratch_limit_and_growing_gather_pools(ctx, monkeypatch):
    """The gather pools hold a fraction of the elements and grow when a search finds them too small:
    a context that starts with the smallest pools (INSHR_POOL_WCAP=1) gives the same bytes as the
    default one, within a scratch limit far below 8 bytes per element; a limit below the tables is
    reported as INSHR_E_CAPACITY."""
    from paper_2306_11800_amd import api
    g = torch.Generator(device="cuda:0")
    g.manual_seed(51)
    n = 40_000_003
    x = 0.02 * torch.randn(n, device="cuda:0", generator=g)
    x[::7] = 0.25  # heavy duplicates: one bin gathers far more than an average share
    small_x = dev((0.02 * np.random.default_rng(52).standard_t(4, 700)).astype(np.float32))
    ts = [x, small_x]
    grid = synth.grid_full()
    best, feas, scores = ctx.search(ts, grid, synth.EPS_DEFAULT)
    want = ctx.quantize(ts, [grid[b] for b in best], reuse_search=True)
    with monkeypatch.context() as m:
        m.setenv("INSHR_POOL_WCAP", "1")
        small = api.Context(torch.device("cuda:0"), scratch_bytes=200 << 20)  # 8 B per element would be 320 MB
    b2, f2, s2 = small.search(ts, grid, synth.EPS_DEFAULT)
    assert (b2, f2) == (best, feas)
    for i in range(len(ts) * len(grid)):
        assert (s2[i].sse, s2[i].n_kept, s2[i].cost_bits) == (scores[i].sse, scores[i].n_kept, scores[i].cost_bits)
    got = small.quantize(ts, [grid[b] for b in best], reuse_search=True)
    for a, b in zip(got, want):
        assert torch.equal(a.packed, b.packed) and torch.equal(a.codebook, b.codebook)
        assert torch.equal(a.boundaries, b.boundaries) and torch.equal(a.outlier_idx, b.outlier_idx)
    small.close()
    tiny = api.Context(torch.device("cuda:0"), scratch_bytes=1 << 20)
    with pytest.raises(api.InshrError) as e:
        tiny.search(ts, grid, synth.EPS_DEFAULT)
    assert e.value.code == -4
    tiny.close()
