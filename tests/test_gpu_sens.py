"""GPU parity of the partition by magnitude and sensitivity (Sec. 4.1-4.2) against the CPU oracle:
thresholds of both metrics, classes, symbols, protected list, boundaries bit-exact; centres and
errors 1e-6."""
import numpy as np
import pytest
import torch

from oracle import ref
from test_gpu_parity import REL, dev, u32, u64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2306_11800_amd import api
    c = api.Context(torch.device("cuda:0"))
    yield c
    c.close()


def check(q, inf, x, g, cfg, by_sens):
    r = ref.quantize_sens(x, g, cfg, by_sens)
    assert q.sym_bits == r["sym_bits"] and q.K == r["K"]
    assert (q.n_pruned, q.n_outlier, q.n_kept) == (r["n_pruned"], r["n_outlier"], r["n_kept"]), (cfg, by_sens)
    assert np.float32(q.tau_prune).view(np.uint32) == r["tau_prune_bits"]
    assert np.float32(q.tau_outlier).view(np.uint32) == r["tau_outlier_bits"]
    assert np.float32(inf[0]).view(np.uint32) == r["tau_outlier_sens_bits"]
    assert np.array_equal(u32(q.boundaries)[:r["K"] - 1], r["boundaries"].view(np.uint32))
    got = u64(q.packed)
    want = ref.pack(r["sym"], r["sym_bits"])
    if not np.array_equal(got, want):
        gs = ref.unpack(got, x.size, r["sym_bits"])
        bad = np.nonzero(gs != r["sym"])[0]
        raise AssertionError(f"symbols differ at {bad[:10]} ({bad.size} of {x.size}) cfg={cfg}: {gs[bad[:10]]} vs {r['sym'][bad[:10]]}")
    assert np.array_equal(u32(q.outlier_idx), r["outlier_idx"])
    assert np.array_equal(u32(q.outlier_val), r["outlier_val"].view(np.uint32))
    np.testing.assert_allclose(q.codebook.cpu().numpy()[:r["K"]], r["codebook"], rtol=REL, atol=0)
    assert abs(inf[2] - r["sumsq"]) <= REL * r["sumsq"]
    assert abs(inf[1] - r["sse"]) <= REL * r["sse"] + 1e-12 * r["sumsq"]
    return r


def make(rng, n):
    x = (0.02 * rng.standard_t(4, n)).astype(np.float32)
    g = (1e-3 * rng.standard_normal(n) * (1 + 20 * (rng.random(n) < 0.01))).astype(np.float32)
    if n > 50:
        x[::17] = 0.0
        g[::29] = 0.0
        g[5] = -0.0
    return x, g


def test_batch_of_ragged_tensors_both_metrics(ctx):
    rng = np.random.default_rng(95)
    sizes = [1, 7, 1023, 1024, 1025, 70_001, 400_003, 33]
    cfgs = [(3, 0, 0), (2, 200000, 100000), (4, 200000, 10000), (8, 100000, 1000), (0, 400000, 1000, 12),
            (5, 300000, 500), (8, 200000, 1000), (1, 100000, 50000)]
    data = [make(rng, n) for n in sizes]
    for by in ([False] * 8, [True] * 8, [True, False] * 4):
        qs, info = ctx.quantize_sens([dev(x) for x, _ in data], [dev(g) for _, g in data], cfgs, by)
        for q, inf, (x, g), cfg, b in zip(qs, info, data, cfgs, by):
            check(q, inf, x, g, cfg, b)


def test_constant_gradient_equals_the_magnitude_quantizer(ctx):
    x = (0.02 * np.random.default_rng(96).standard_t(3, 300_007)).astype(np.float32)
    g = np.full_like(x, 2.0)
    cfg = (6, 200000, 1000)
    qs, _ = ctx.quantize_sens([dev(x)], [dev(g)], [cfg], [True])
    qm = ctx.quantize([dev(x)], [cfg])[0]
    assert torch.equal(qs[0].packed, qm.packed) and torch.equal(qs[0].outlier_idx, qm.outlier_idx)
    assert torch.equal(qs[0].boundaries[:63], qm.boundaries[:63])
    np.testing.assert_allclose(qs[0].codebook.cpu().numpy()[:64], qm.codebook.cpu().numpy()[:64], rtol=REL)


def test_decodes_and_deltas_like_any_other_codes(ctx):
    rng = np.random.default_rng(97)
    x, g = make(rng, 200_003)
    x2 = (x + rng.normal(0, 1e-4, x.size)).astype(np.float32)
    cfg = (5, 200000, 2000)
    qa, _ = ctx.quantize_sens([dev(x)], [dev(g)], [cfg], [True])
    qb, _ = ctx.quantize_sens([dev(x2)], [dev(g)], [cfg], [True])
    ra, rb = ref.quantize_sens(x, g, cfg, True), ref.quantize_sens(x2, g, cfg, True)
    xh = ctx.dequantize(qa)[0].cpu().numpy()
    want = ref.dequantize(ra["sym"], cfg[0], ra["codebook"], ra["outlier_idx"], ra["outlier_val"])
    assert np.array_equal(xh.view(np.uint32), want.view(np.uint32))
    d = ctx.delta(qa, qb)
    ctx.sync()
    rd = ref.delta(ra["sym"], cfg[0], rb["sym"], cfg[0])
    assert np.array_equal(u64(d[0].packed), ref.pack(rd["stream"], rd["delta_bits"]))


def test_errors(ctx):
    from paper_2306_11800_amd import api
    x = (0.02 * np.random.default_rng(98).standard_normal(5000)).astype(np.float32)
    g = np.ones_like(x)
    g[17] = np.inf
    with pytest.raises(api.InshrError) as e:
        ctx.quantize_sens([dev(x)], [dev(g)], [(4, 0, 0)], [False])
    assert e.value.code == -3
    g[17] = np.nan
    with pytest.raises(api.InshrError) as e:
        ctx.quantize_sens([dev(x)], [dev(g)], [(4, 100000, 1000)], [True])
    assert e.value.code == -3
    with pytest.raises(ValueError):
        ctx.quantize_sens([dev(x)], [dev(g[:10])], [(4, 0, 0)], [False])
    # the context still works
    q, _ = ctx.quantize_sens([dev(x)], [dev(np.ones_like(x))], [(4, 0, 0)], [False])
    assert q[0].n_kept == x.size


def test_large_tensor_against_torch_definitions(ctx):
    """24 Mi values (the sampled first sweep inside the threshold searches), both metrics: every
    class, symbol and protected entry against torch sort / bucketize on the device."""
    gen = torch.Generator(device="cuda:0").manual_seed(99)
    n = 24 * 1024 * 1024 + 1234
    x = torch.empty(n, device="cuda:0").normal_(0, 0.02, generator=gen)
    g = torch.empty(n, device="cuda:0").normal_(0, 1e-3, generator=gen)
    g[::1000] *= 50.0
    cfg = (5, 200000, 1000)
    n_p, n_o = n * cfg[1] // 1000000, n * cfg[2] // 1000000
    s = (g * x).abs()
    mag = x.abs()
    tau_om, tau_os = mag.sort().values[n - 1 - n_o], s.sort().values[n - 1 - n_o]
    for by_sens in (True, False):
        metric = s if by_sens else mag
        tau_p = metric.sort().values[n_p]
        prot = (mag > tau_om) | (s > tau_os)
        pruned = ~prot & (metric < tau_p)
        Y = x[~prot & ~pruned].sort().values
        M = Y.numel()
        t = Y[[j * M // 32 for j in range(1, 32)]]
        want = torch.bucketize(x, t, right=True) + 2
        want[pruned] = 0
        want[prot] = 1
        qs, info = ctx.quantize_sens([x], [g], [cfg], [by_sens])
        q = qs[0]
        assert (q.n_pruned, q.n_outlier, q.n_kept) == (int(pruned.sum()), int(prot.sum()), M)
        assert q.tau_prune == float(tau_p) and q.tau_outlier == float(tau_om) and info[0][0] == float(tau_os)
        assert torch.equal(q.boundaries[:31], t)
        sym = torch.from_numpy(ref.unpack(q.packed.cpu().numpy().view(np.uint64), n, q.sym_bits).astype(np.int64)).to(x.device)
        assert torch.equal(sym, want)
        assert torch.equal(q.outlier_idx.long(), torch.nonzero(prot).ravel())
        assert torch.equal(q.outlier_val, x[prot])
        dec = torch.zeros(n, dtype=torch.float64, device=x.device)
        kept = want >= 2
        dec[kept] = q.codebook[(want[kept] - 2)].double()
        dec[prot] = x[prot].double()
        sse = float(((x.double() - dec) ** 2).sum())
        assert abs(info[0][1] - sse) <= 1e-6 * sse
        del want, sym, dec, kept, prot, pruned, Y
