"""GPU, full size: the largest tensor shape of the bench (32000 x 4096 = 131 M values) in the launch
configuration the bench uses, checked on every element against definitions written with torch's
library routines on the device (sort, bucketize, stable sort, bincount) — the CPU oracle would need
minutes for this size.  Thresholds, boundaries, every symbol, the protected list, the delta stream,
the regrouping permutation, the group offsets, the reconstructed symbols and the decoded values are
compared bit for bit; centres and the error sum of the chosen configuration to 1e-6."""
import numpy as np
import pytest
import torch

from paper_2306_11800_amd import synth

pytestmark = pytest.mark.gpu

N = 32000 * 4096


@pytest.fixture(scope="module")
def ctx():
    from paper_2306_11800_amd import api
    c = api.Context(torch.device("cuda:0"))
    yield c
    c.close()


def unpack(words: torch.Tensor, n: int, w: int) -> torch.Tensor:
    """Symbol i = bits [w*i, w*i + w) of the little-endian word stream (w <= 9)."""
    b = torch.cat([words.view(torch.uint8), torch.zeros(8, dtype=torch.uint8, device=words.device)])
    out = torch.empty(n, dtype=torch.int16, device=words.device)
    step = 1 << 24
    for i0 in range(0, n, step):
        i = torch.arange(i0, min(n, i0 + step), device=words.device, dtype=torch.int64)
        bit = i * w
        byte = bit >> 3
        two = b[byte].to(torch.int32) | (b[byte + 1].to(torch.int32) << 8)
        out[i0:i0 + i.numel()] = ((two >> (bit & 7).to(torch.int32)) & ((1 << w) - 1)).to(torch.int16)
    return out


def torch_quantize(x: torch.Tensor, cfg):
    """Sec. 4 with library routines: thresholds = order statistics of |x|, boundaries = equal-frequency
    order statistics of the kept values, symbol 0 pruned / 1 protected / 2 + #{t_j <= x}."""
    bits, p_ppm, o_ppm = cfg
    n, K = x.numel(), 1 << bits
    A = torch.sort(x.abs()).values
    tau_p = A[n * p_ppm // 1_000_000]
    tau_o = A[n - 1 - n * o_ppm // 1_000_000]
    del A
    mag = x.abs()
    pruned, prot = mag < tau_p, mag > tau_o
    kept = ~(pruned | prot)
    Y = torch.sort(x[kept]).values
    M = Y.numel()
    j = torch.arange(1, K, device=x.device, dtype=torch.int64)
    t = Y[(j * M) // K]
    del Y
    sym = (2 + torch.bucketize(x, t, right=True)).to(torch.int16)
    sym[pruned] = 0
    sym[prot] = 1
    return dict(tau_p=tau_p, tau_o=tau_o, t=t, sym=sym, kept=kept, prot=prot, M=M)


def test_largest_tensor_every_element(ctx):
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(77)
    # the bench's recipe for one 2-D weight: 0.015 * Student-t(3), 0.1 % of the columns x20,
    # next step = previous + N(0, 1e-4)
    prev = torch.empty(N, dtype=torch.float32, device=dev)
    step = 1 << 26
    for s in range(0, N, step):
        e = min(N, s + step)
        z = torch.randn(4, e - s, dtype=torch.float32, device=dev, generator=g)
        prev[s:e] = 0.015 * z[0] / torch.sqrt((z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0)
        del z
    hot = torch.randperm(4096, device=dev, generator=g)[:4]
    prev.view(32000, 4096)[:, hot] *= 20.0
    cur = prev + 1e-4 * torch.randn(N, device=dev, generator=g)
    # torch orders -0.0 and +0.0 as equal while the library makes both +0.0: keep zeros out of this
    # test (tests/test_gpu_parity.py covers them against the oracle)
    prev[prev == 0] = 1e-6
    cur[cur == 0] = 1e-6
    grid = synth.grid_small()
    cfg = (8, 100000, 1000)
    refs, qs = [], []
    for x in (prev, cur):
        r = torch_quantize(x, cfg)
        best, feas, scores = ctx.search([x], grid, synth.EPS_DEFAULT)
        q = ctx.quantize([x], [cfg], reuse_search=cfg in grid)[0]
        assert q.tau_prune == float(r["tau_p"]) and q.tau_outlier == float(r["tau_o"])
        assert torch.equal(q.boundaries.view(torch.int32), r["t"].view(torch.int32))
        got = unpack(q.packed, N, 9)
        assert torch.equal(got, r["sym"]), int((got != r["sym"]).sum())
        idx = torch.nonzero(r["prot"]).flatten().to(torch.int32)
        assert torch.equal(q.outlier_idx, idx)
        assert torch.equal(q.outlier_val.view(torch.int32), x[r["prot"]].view(torch.int32))
        assert (q.n_kept, q.n_outlier) == (r["M"], idx.numel()) and q.n_pruned == N - r["M"] - idx.numel()
        # centres and error of this configuration, in fp64
        if cfg in grid:
            gi = grid.index(cfg)
            b = (r["sym"][r["kept"]] - 2).to(torch.int64)
            xv = x[r["kept"]].double()
            cnt = torch.bincount(b, minlength=256).double()
            sx = torch.zeros(256, dtype=torch.float64, device=dev).index_add_(0, b, xv)
            c = (sx / cnt.clamp(min=1)).float()
            ok = cnt > 0
            np.testing.assert_allclose(q.codebook[ok].cpu().numpy(), c[ok].cpu().numpy(), rtol=1e-6)
            sumsq = float((x.double() ** 2).sum())
            pr = r["sym"] == 0
            sse = float((x[pr].double() ** 2).sum()) + float(((xv - c.double()[b]) ** 2).sum())
            assert abs(scores[gi].sumsq - sumsq) <= 1e-9 * sumsq
            assert abs(scores[gi].sse - sse) <= 1e-6 * sse + 1e-12 * sumsq
            assert scores[gi].n_kept == r["M"]
        refs.append(r)
        qs.append(q)
        del got
    # delta: d = (s_prev - s_cur) mod (K + 2), regrouped in the stable order of s_prev
    sp, sc = refs[0]["sym"].to(torch.int32), refs[1]["sym"].to(torch.int32)
    B = (1 << cfg[0]) + 2
    d = torch.remainder(sp - sc, B).to(torch.int16)
    perm = torch.sort(refs[0]["sym"], stable=True).indices
    out = ctx.delta([qs[0]], [qs[1]], want_perm=True)[0]
    ctx.sync()
    assert out.delta_bits == 9
    assert torch.equal(out.perm.to(torch.int64) & 0xFFFFFFFF, perm)
    assert torch.equal(unpack(out.packed, N, 9), d[perm])
    goff = torch.zeros(B + 1, dtype=torch.int64, device=dev)
    goff[1:] = torch.cumsum(torch.bincount(sp, minlength=B), 0)
    assert torch.equal(out.group_off, goff)
    # the stream without the permutation is the same stream
    out2 = ctx.delta([qs[0]], [qs[1]], want_perm=False)[0]
    ctx.sync()
    assert torch.equal(out2.packed, out.packed)
    # restore side: the current symbols come back from the previous symbols and the stream, and
    # decoding them gives 0 / the protected value / the centre of the bin for every element
    rec = ctx.reconstruct([qs[0]], [out2], [cfg[0]])[0]
    assert torch.equal(rec, qs[1].packed)
    xh = ctx.dequantize([qs[1]])[0]
    sym = refs[1]["sym"].to(torch.int64)
    want = torch.where(sym >= 2, qs[1].codebook[(sym - 2).clamp(min=0)], torch.zeros((), device=dev))
    want[refs[1]["prot"]] = cur[refs[1]["prot"]]
    assert torch.equal(xh.view(torch.int32), want.view(torch.int32))


def test_largest_tensor_sketch_bins(ctx):
    """The sketch quantizer on the same shape, in the launch configuration bench.py --sketch uses
    (on top of a grid search): the bucket counts are recomputed with torch.bucketize over the exact
    bucket tops (integer arithmetic, oracle/sketch_kmeans.py), the clustering of those few hundred
    buckets is the CPU oracle's, and every symbol is compared with torch.bucketize over the
    resulting boundaries."""
    from oracle import sketch_kmeans as sk

    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(78)
    x = torch.empty(N, dtype=torch.float32, device=dev)
    step = 1 << 26
    for s in range(0, N, step):
        e = min(N, s + step)
        z = torch.randn(4, e - s, dtype=torch.float32, device=dev, generator=g)
        x[s:e] = 0.015 * z[0] / torch.sqrt((z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0)
        del z
    x[x == 0] = 1e-6
    grid = synth.grid_full()
    cfg = (8, 200000, 1000)
    alpha, sigma, max_iter = 0.01, 0.2, 100
    uni = np.random.default_rng(5).uniform(size=(1, 256))
    ctx.search([x], grid, synth.EPS_DEFAULT, want_scores=False)
    (q,), (info,) = ctx.quantize_sketch([x], [cfg], uni, alpha=alpha, sigma=sigma, max_iter=max_iter,
                                        reuse_search=True)
    # classes from order statistics of |x|
    A = torch.sort(x.abs()).values
    tau_p, tau_o = A[N * cfg[1] // 1_000_000], A[N - 1 - N * cfg[2] // 1_000_000]
    del A
    mag = x.abs()
    pruned, prot = mag < tau_p, mag > tau_o
    kept = ~(pruned | prot)
    assert q.tau_prune == float(tau_p) and q.tau_outlier == float(tau_o)
    # Algorithm 1 with library routines: bucket = first one whose top reaches |x|
    i_lo, tops = sk._bucket_tops(alpha)
    b = torch.bucketize(mag[kept], torch.from_numpy(tops).to(dev), right=False).to(torch.int64)
    neg = x[kept] < 0
    n_b = tops.size
    counts = torch.bincount(torch.where(neg, n_b - 1 - b, n_b + b), minlength=2 * n_b).cpu().numpy()
    nz = np.nonzero(counts)[0]
    sign = np.where(nz < n_b, -1, 1)
    idx = np.where(nz < n_b, n_b - 1 - nz, nz - n_b) + i_lo
    xq = sk.bucket_value(sign, idx, alpha)
    assert np.all(np.diff(xq) > 0)
    w = sk.sample_weights(xq, counts[nz], sigma)
    init = sk.weighted_kmeanspp(xq, w, 256, uni[0])
    centres, rounds = sk.weighted_lloyd(xq, w, xq[init], max_iter)
    assert info == (nz.size, rounds)
    cb = centres.astype(np.float32)
    np.testing.assert_allclose(q.codebook.cpu().numpy(), cb, rtol=1e-6, atol=0)
    bnd = np.array([sk.boundary_above(m) for m in sk.midpoints(cb.astype(np.float64))], np.float32)
    assert np.array_equal(q.boundaries.cpu().numpy().view(np.uint32), bnd.view(np.uint32))
    sym = (2 + torch.bucketize(x, torch.from_numpy(bnd).to(dev), right=True)).to(torch.int16)
    sym[pruned] = 0
    sym[prot] = 1
    got = unpack(q.packed, N, 9)
    assert torch.equal(got, sym), int((got != sym).sum())
    assert torch.equal(q.outlier_idx, torch.nonzero(prot).flatten().to(torch.int32))


def test_tile_structured_tensor_under_the_sampled_sweep(ctx):
    """24 Mi values whose scale changes from tile to tile by up to six decades: the first sweep of
    the search samples one tile in eight for a tensor of this size, its predictions of the threshold
    buckets are wrong here, and the exact sweeps are repeated for the tensor.  Thresholds,
    boundaries and every symbol are compared with the torch definitions."""
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(79)
    n = 24 << 20
    x = torch.randn(n, dtype=torch.float32, device=dev, generator=g)
    scale = torch.pow(10.0, torch.rand(n // 16384, device=dev, generator=g) * 6.0 - 3.0)
    x = (x.view(-1, 16384) * scale[:, None]).reshape(-1).contiguous()
    x[x == 0] = 1e-6
    grid = synth.grid_full()
    for cfg in ((8, 200000, 1000), (5, 0, 0)):
        r = torch_quantize(x, cfg)
        ctx.search([x], grid, synth.EPS_DEFAULT, want_scores=False)
        q = ctx.quantize([x], [cfg], reuse_search=True)[0]
        assert q.tau_prune == float(r["tau_p"]) and q.tau_outlier == float(r["tau_o"])
        K = 1 << cfg[0]
        assert torch.equal(q.boundaries[:K - 1].view(torch.int32), r["t"].view(torch.int32))
        got = unpack(q.packed, n, cfg[0] + 1)
        assert torch.equal(got, r["sym"]), int((got != r["sym"]).sum())
        assert (q.n_kept, q.n_outlier) == (r["M"], int(r["prot"].sum()))


def test_largest_tensor_search_over_bits_with_sketch_bins(ctx):
    """inshr_search_sketch on the 131 M-value shape on top of a grid search (the configuration
    bench.py --sketch times): the reported error of the chosen width equals the squared distance
    between the tensor and its decoded form computed with torch, the choice obeys the rule (fewest
    bits within the bound), and every symbol is the nearest centre of the returned codebook."""
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(80)
    x = torch.empty(N, dtype=torch.float32, device=dev)
    step = 1 << 26
    for s in range(0, N, step):
        e = min(N, s + step)
        z = torch.randn(4, e - s, dtype=torch.float32, device=dev, generator=g)
        x[s:e] = 0.015 * z[0] / torch.sqrt((z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0)
        del z
    x[x == 0] = 1e-6
    grid = synth.grid_full()
    eps = synth.EPS_DEFAULT
    uni = np.random.default_rng(6).uniform(size=(1, 256))
    ctx.search([x], grid, eps, want_scores=False)
    (q,), (ch,), _ = ctx.search_sketch([x], [(0, 200000, 1000)], uni, eps, reuse_search=True)
    bits = ch["best_bits"]
    assert q.bits == bits and 2 <= bits <= 8
    sumsq = float((x.double() ** 2).sum())
    assert abs(ch["sumsq"] - sumsq) <= 1e-9 * sumsq
    y = ctx.dequantize([q])[0]
    sse = float(((x.double() - y.double()) ** 2).sum())
    got_sse = ch["sse"][bits - 2]
    assert abs(got_sse - sse) <= 1e-6 * sse + 1e-12 * sumsq, (got_sse, sse)
    assert ch["feasible"] and got_sse <= eps * sumsq
    assert bits == 2 or ch["sse"][bits - 3] > eps * sumsq
    K = 1 << bits
    cb = q.codebook.double()
    assert bool((cb[1:] >= cb[:-1]).all())
    mids = (cb[:-1] + cb[1:]) / 2
    sym = unpack(q.packed, N, bits + 1)
    kept = sym >= 2
    want = 2 + torch.bucketize(x[kept].double(), mids, right=False)  # strictly above the midpoint -> upper centre
    assert torch.equal(sym[kept].to(torch.int64), want)
    A = torch.sort(x.abs()).values
    tau_p, tau_o = A[N * 200000 // 1_000_000], A[N - 1 - N * 1000 // 1_000_000]
    assert torch.equal(sym == 0, x.abs() < tau_p) and torch.equal(sym == 1, x.abs() > tau_o)


@pytest.mark.parametrize("n", [4096 * 4096, 11008 * 4096, 4096 * 4096 + 12345])
def test_other_bench_shapes(ctx, n):
    """The other 2-D weight shapes of the bench (and a ragged size): at 16 Mi values and more the
    first sweep of the search is sampled.  Thresholds, boundaries and every symbol against the
    torch definitions for three configurations."""
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(81)
    z = torch.randn(4, n, dtype=torch.float32, device=dev, generator=g)
    x = 0.015 * z[0] / torch.sqrt((z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0)
    del z
    x[x == 0] = 1e-6
    if n % 4096 == 0:
        hot = torch.randperm(4096, device=dev, generator=g)[:4]
        x.view(-1, 4096)[:, hot] *= 20.0
    ctx.search([x], synth.grid_full(), synth.EPS_DEFAULT, want_scores=False)
    for cfg in ((8, 200000, 1000), (7, 0, 0), (4, 400000, 100)):
        r = torch_quantize(x, cfg)
        q = ctx.quantize([x], [cfg], reuse_search=True)[0]
        K = 1 << cfg[0]
        assert q.tau_prune == float(r["tau_p"]) and q.tau_outlier == float(r["tau_o"])
        assert torch.equal(q.boundaries[:K - 1].view(torch.int32), r["t"].view(torch.int32))
        got = unpack(q.packed, n, cfg[0] + 1)
        assert torch.equal(got, r["sym"]), int((got != r["sym"]).sum())


def test_full_grid_score_table_on_a_sampled_tensor(ctx):
    """All 105 rows of the score table, and the choice, on one 4096 x 4096 tensor of the bench's
    recipe (16 Mi values: the first sweep of the search is sampled, as in the bench).  Every
    configuration is computed on its own from the definitions with torch's library routines:
    thresholds = order statistics of |x|, boundaries = order statistics of the quantized values at
    floor(j M / K), bins by bucketize, centres = fp32 of the fp64 mean, squared error in fp64."""
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(82)
    n = 4096 * 4096
    z = torch.randn(4, n, dtype=torch.float32, device=dev, generator=g)
    x = 0.015 * z[0] / torch.sqrt((z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0)
    del z
    hot = torch.randperm(4096, device=dev, generator=g)[:4]
    x.view(-1, 4096)[:, hot] *= 20.0
    x[x == 0] = 1e-6
    grid, eps = synth.grid_full(), synth.EPS_DEFAULT
    best, feas, scores = ctx.search([x], grid, eps, want_scores=True)
    A = torch.sort(x.abs()).values
    xd = x.double()
    sumsq = float((xd * xd).sum())
    mag = x.abs()
    rows, border = [], False
    kept_sorted = {}  # (prune, protect) -> its classes and sorted quantized values (data, shared by the bit widths)
    for gi, (bits, p_ppm, o_ppm) in enumerate(grid):
        K = 1 << bits
        if (p_ppm, o_ppm) not in kept_sorted:
            tau_p, tau_o = A[n * p_ppm // 1_000_000], A[n - 1 - n * o_ppm // 1_000_000]
            pruned, prot = mag < tau_p, mag > tau_o
            xk = x[~(pruned | prot)]
            kept_sorted[(p_ppm, o_ppm)] = (float((xd[pruned] ** 2).sum()), int(prot.sum()), xk, torch.sort(xk).values)
            del pruned, prot
        sq_pruned, n_prot, xk, Y = kept_sorted[(p_ppm, o_ppm)]
        M = Y.numel()
        j = torch.arange(1, K, device=dev, dtype=torch.int64)
        t = Y[(j * M) // K]
        b = torch.bucketize(xk, t, right=True)
        cnt = torch.bincount(b, minlength=K).double()
        sx = torch.bincount(b, weights=xk.double(), minlength=K)
        c = (sx / cnt.clamp(min=1)).float()
        sse = sq_pruned + float(((xk.double() - c.double()[b]) ** 2).sum())
        cost = M * bits + 32 * n_prot + 32 * K
        s = scores[gi]
        assert (s.n_pruned, s.n_outlier, s.n_kept, s.cost_bits) == (n - M - n_prot, n_prot, M, cost), grid[gi]
        assert abs(s.sumsq - sumsq) <= 1e-9 * sumsq
        assert abs(s.sse - sse) <= 1e-6 * sse + 1e-12 * sumsq, (grid[gi], s.sse, sse)
        rows.append((sse, cost))
        border = border or abs(sse / sumsq - eps) <= 4e-6 * eps
        del b
    feasible = [i for i, (sse, cost) in enumerate(rows) if sse / sumsq <= eps]
    if feasible:
        want = min(feasible, key=lambda i: (rows[i][1], i))
    else:
        want = min(range(len(rows)), key=lambda i: (rows[i][0], i))
    if not border:
        assert (best[0], feas[0]) == (want, 1 if feasible else 0)
