"""GPU parity of thresholds per layer type (Sec. 4.2: the same pruning fraction across all layers of
a type): groups of tensors share thresholds that are order statistics of their pooled magnitudes.
Scores, choice, symbols, protected lists, centres and delta against the CPU oracle with the same
pools."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2306_11800_amd import synth
from test_gpu_parity import check_delta, check_quantized, check_scores, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2306_11800_amd import api
    c = api.Context(torch.device("cuda:0"))
    yield c
    c.close()


def pools_of(xs, groups):
    return {g: ref.pool_of([x for x, h in zip(xs, groups) if h == g]) for g in set(groups)}


def run(ctx, xs, groups, grid, eps, quantize_all=False):
    pools = pools_of(xs, groups)
    ts = [dev(x) for x in xs]
    nC = len(grid)
    best, feas, sc = ctx.search(ts, grid, eps, groups=groups)
    rbest = []
    for i, x in enumerate(xs):
        rbest.append(check_scores(sc, nC, i, x, grid, eps, best[i], feas[i],
                                  given=ref.search(x, grid, eps, pool=pools[groups[i]])))
    picks = [best] + ([[g] * len(xs) for g in range(nC)] if quantize_all else [])
    out = None
    for pick in picks:
        cfgs = [grid[g] for g in pick]
        caps = [max(1, int(sc[i * nC + g].n_outlier)) for i, g in enumerate(pick)]
        qs = ctx.quantize(ts, cfgs, reuse_search=True, outlier_caps=caps)
        for q, x, cfg, h in zip(qs, xs, cfgs, groups):
            check_quantized(q, x, cfg, given=ref.quantize(x, cfg, pool=pools[h]))
        out = out or (qs, cfgs)
    return out


def test_groups_of_ragged_tensors_full_grid(ctx):
    rng = np.random.default_rng(81)
    sizes = [70_001, 5, 300, 4097, 400_003, 16_384, 1, 33_000]
    scale = [0.02, 0.02, 0.5, 0.001, 0.02, 0.1, 0.02, 0.003]
    xs = [(s * rng.standard_t(4, n)).astype(np.float32) for s, n in zip(scale, sizes)]
    xs[3][::3] = 0.0                                    # zeros inside a group
    xs[1][:] = [0.01, -0.03, 0.04, 0.002, -0.015]       # (tiny tensors keep something under every pair)
    xs[6][:] = [0.15]
    groups = [7, 7, 7, 2, 2, 9, 9, 4]                   # the last one stands alone
    run(ctx, xs, groups, synth.grid_full(), synth.EPS_DEFAULT)
    run(ctx, xs, groups, synth.grid_small(), synth.EPS_DEFAULT, quantize_all=True)
    # the search space of the paper (a slice that fits one call), numbers of bins 6 and 12 among them
    run(ctx, xs, groups, synth.grid_paper(prune=(0.0, 0.1, 0.3, 0.5)), 0.02)


def test_a_group_of_one_and_all_in_one(ctx):
    rng = np.random.default_rng(82)
    xs = [(0.02 * rng.standard_t(3, n)).astype(np.float32) for n in (100_003, 50_000, 70_000)]
    ts = [dev(x) for x in xs]
    grid = synth.grid_small()
    alone = ctx.search(ts, grid, 0.01)
    same = ctx.search(ts, grid, 0.01, groups=[5, 6, 7])
    assert alone[:2] == same[:2] and bytes(alone[2]) == bytes(same[2])
    run(ctx, xs, [0, 0, 0], grid, 0.01)
    # pooling is what concatenation would give: thresholds of the group = thresholds of the joined tensor
    joined = np.concatenate(xs)
    q_join = ctx.quantize([dev(joined)], [(4, 100000, 1000)])[0]
    best, feas, sc = ctx.search(ts, [(4, 100000, 1000)], 0.01, groups=[1, 1, 1])
    qs = ctx.quantize(ts, [(4, 100000, 1000)] * 3, reuse_search=True, outlier_caps=[int(sc[i].n_outlier) + 1 for i in range(3)])
    assert all(q.tau_prune == q_join.tau_prune and q.tau_outlier == q_join.tau_outlier for q in qs)
    assert sum(q.n_pruned for q in qs) == q_join.n_pruned and sum(q.n_outlier for q in qs) == q_join.n_outlier


def test_large_group_with_a_tensor_that_would_be_sampled_alone(ctx):
    """A 20 Mi-element tensor takes the sampled first sweep when it stands alone; in a group it does
    not.  Every symbol against the torch definitions with the pooled thresholds."""
    g = torch.Generator(device="cuda:0").manual_seed(83)
    a = torch.empty(20 * 1024 * 1024 + 77, device="cuda:0").normal_(0, 0.02, generator=g)
    b = torch.empty(3_000_001, device="cuda:0").normal_(0, 0.2, generator=g)
    cfg = (5, 200000, 1000)
    best, feas, sc = ctx.search([a, b], [cfg], 0.01, groups=[3, 3])
    qs = ctx.quantize([a, b], [cfg, cfg], reuse_search=True, outlier_caps=[int(sc[0].n_outlier) + 1, int(sc[1].n_outlier) + 1])
    mag = torch.cat([a.abs(), b.abs()]).sort().values
    N = mag.numel()
    tp, to = mag[N * cfg[1] // 1000000], mag[N - 1 - N * cfg[2] // 1000000]
    del mag
    for x, q in zip((a, b), qs):
        assert q.tau_prune == float(tp) and q.tau_outlier == float(to)
        pruned, prot = x.abs() < tp, x.abs() > to
        assert (q.n_pruned, q.n_outlier) == (int(pruned.sum()), int(prot.sum()))
        Y = x[~pruned & ~prot].sort().values
        M = Y.numel()
        t = Y[[j * M // 32 for j in range(1, 32)]]
        assert torch.equal(q.boundaries[:31], t)
        want = torch.bucketize(x, t, right=True) + 2
        want[pruned] = 0
        want[prot] = 1
        w = q.sym_bits
        sym = torch.from_numpy(ref.unpack(q.packed.cpu().numpy().view(np.uint64), x.numel(), w).astype(np.int64)).to(x.device)
        assert torch.equal(sym, want)
        assert torch.equal(q.outlier_idx.long(), torch.nonzero(prot).ravel())


def test_a_tensor_left_without_quantized_values_is_reported(ctx):
    from paper_2306_11800_amd import api
    rng = np.random.default_rng(84)
    big = (rng.standard_normal(50_000)).astype(np.float32)
    tiny = (1e-6 * rng.standard_normal(200)).astype(np.float32)      # all below the pooled prune threshold
    with pytest.raises(api.InshrError) as e:
        ctx.search([dev(big), dev(tiny)], [(4, 300000, 0)], 0.01, groups=[1, 1])
    assert e.value.code == -2
    with pytest.raises(ref.RefError) as r:
        ref.quantize(tiny, (4, 300000, 0), pool=ref.pool_of([big, tiny]))
    assert r.value.code == -7
    # the context still works afterwards
    best, feas, _ = ctx.search([dev(big)], [(4, 300000, 0)], 0.01)
    assert feas[0] in (0, 1)


def test_delta_after_a_pooled_search(ctx):
    rng = np.random.default_rng(85)
    prevs = [(s * rng.standard_t(4, n)).astype(np.float32) for s, n in ((0.02, 200_003), (0.05, 90_000))]
    curs = [(p + rng.normal(0, 1e-4, p.size)).astype(np.float32) for p in prevs]
    grid = synth.grid_small()
    (qp, cp) = run(ctx, prevs, [1, 1], grid, 0.01)
    (qc, cc) = run(ctx, curs, [1, 1], grid, 0.01)
    d = ctx.delta(qp, qc, want_perm=True)
    ctx.sync()
    pp, pc = pools_of(prevs, [1, 1]), pools_of(curs, [1, 1])
    for i in range(2):
        rp = ref.quantize(prevs[i], cp[i], pool=pp[1])
        rc = ref.quantize(curs[i], cc[i], pool=pc[1])
        check_delta(d[i], rp, cp[i][0], rc, cc[i][0], True)


def test_protected_share_beyond_the_fraction_needs_room(ctx):
    """With shared thresholds one tensor can hold most of the group's protected values: buffers sized
    by the fraction alone are refused (INSHR_E_CAPACITY), never overrun."""
    from paper_2306_11800_amd import api
    rng = np.random.default_rng(86)
    small = (0.02 * rng.standard_normal(200_000)).astype(np.float32)
    large = (0.5 * rng.standard_normal(3_000)).astype(np.float32)     # holds the group's largest magnitudes
    ts = [dev(small), dev(large)]
    cfg = (4, 100000, 5000)
    best, feas, sc = ctx.search(ts, [cfg], 0.01, groups=[1, 1])
    assert sc[1].n_outlier > large.size * cfg[2] // 1000000           # more than its own fraction
    with pytest.raises(api.InshrError) as e:
        ctx.quantize(ts, [cfg, cfg], reuse_search=True)               # capacity from the fraction
    assert e.value.code == -4
    best, feas, sc = ctx.search(ts, [cfg], 0.01, groups=[1, 1])
    qs = ctx.quantize(ts, [cfg, cfg], reuse_search=True, outlier_caps=[int(sc[0].n_outlier) + 1, int(sc[1].n_outlier)])
    pool = ref.pool_of([small, large])
    for q, x in zip(qs, (small, large)):
        check_quantized(q, x, cfg, given=ref.quantize(x, cfg, pool=pool))
