"""Pins of the sketch / weighted K-Means oracle against things other than itself: a hand example,
the sketch's relative-error guarantee and quantile bound (Sec. 4.3), library logarithms, Lloyd
rounds of scikit-learn, brute-force optimal 1-D clusterings (identical memberships for separable
clusters, appendix "Additional Details for Approximate K-Means"), the loss inequalities of
Proposition 1 and the expectation bound of Proposition 2."""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import sketch_kmeans as sk

HERE = os.path.dirname(__file__)


def test_hand_example():
    # weights: C/max = [1, .5, .25, .25], |X|/max = [.125, .25, .5, 1], sigma = .5
    #   -> W = [.5625, .375, .375, .625], total 1.9375
    # draw 1: u = .5 -> target .96875; running sums .5625, .9375, 1.3125 -> index 2 (x = 4)
    # draw 2: D = [9, 4, 0, 16], D W = [5.0625, 1.5, 0, 10], total 16.5625; u = .3 -> 4.96875 -> index 0
    # draw 3: D = [0, 1, 0, 16], D W = [0, .375, 0, 10]; u = .02 -> .2075 -> index 1
    # Lloyd from [1, 2, 4]: members {1},{2},{4,8} -> c3 = (.375*4 + .625*8)/1 = 6.5;
    #   midpoints 1.5, 4.25: {1},{2,4},{8} -> [1, 3, 8]; midpoints 2, 5.5: 2 is not above 2 ->
    #   {1,2},{4},{8} -> [(.5625 + .75)/.9375 = 1.4, 4, 8]; midpoints 2.7, 6: unchanged -> stop after 3
    g = json.load(open(os.path.join(HERE, "golden", "sketch_kmeans_hand_example.json")))
    w = sk.sample_weights(g["xq"], g["cq"], g["sigma"])
    assert np.allclose(w, g["weights"], rtol=0, atol=1e-15)
    chosen = sk.weighted_kmeanspp(g["xq"], w, g["k"], g["uniforms"])
    assert chosen == g["chosen"]
    c, rounds = sk.weighted_lloyd(g["xq"], w, np.array(g["xq"])[chosen], 100)
    assert rounds == g["rounds"]
    assert np.allclose(c, g["centres"], rtol=1e-15)


def test_bucket_index_against_library_logarithm():
    rng = np.random.default_rng(1)
    x = np.exp(rng.uniform(math.log(1e-44), math.log(3e38), 200000)).astype(np.float32)
    x = x[x > 0]
    for alpha in (0.01, 0.0055, 0.1):
        gamma = sk.gamma_of(alpha)
        i = sk.bucket_index(x, alpha)
        t = np.log(x.astype(np.float64)) / math.log(gamma)
        lib = np.ceil(t)
        near = np.abs(t - np.rint(t)) < 1e-6  # the library value is not trusted next to a bucket edge
        assert np.array_equal(i[~near], lib[~near].astype(np.int64))
        assert np.all(np.abs(i[near] - t[near]) < 1.0 + 1e-6)
        # definition: gamma^(i-1) < x <= gamma^i (fp64 powers, compared away from the edges)
        assert np.all(x[~near] <= gamma ** i[~near].astype(np.float64) * (1 + 1e-9))
        assert np.all(x[~near] > gamma ** (i[~near].astype(np.float64) - 1.0) * (1 - 1e-9))
    # exact powers of gamma rounded down / up to fp32 fall on the two sides of the edge
    gamma = sk.gamma_of(0.01)
    for e in (-3000, -17, 1, 5, 999, 4000):
        v = gamma ** e
        dn = np.float32(v) if float(np.float32(v)) <= v else np.nextafter(np.float32(v), np.float32(0))
        up = np.nextafter(dn, np.float32(np.inf))
        assert sk.bucket_index(np.array([dn]), 0.01)[0] == e
        assert sk.bucket_index(np.array([up]), 0.01)[0] == e + 1
    assert sk.bucket_index(np.array([1.0], np.float32), 0.01)[0] == 0  # gamma^0 exactly


def test_sketch_relative_error_and_counts():
    rng = np.random.default_rng(2)
    x = (rng.standard_t(3, 50000) * 0.015).astype(np.float32)
    x[::97] = 0.0
    for alpha in (0.01, 0.05):
        s, i, c = sk.sketch_histogram(x, alpha)
        v = sk.bucket_value(s, i, alpha)
        assert int(c.sum()) == x.size
        assert np.all(np.diff(v) > 0)  # sorted by value, one entry per bucket
        # every element lies within alpha (relative) of its bucket's value
        keys = np.sign(x).astype(np.int64) * ((1 << 20) + np.where(x != 0, sk.bucket_index(np.abs(x) + (x == 0), alpha), 0))
        lut = {int(ss) * ((1 << 20) + int(ii)) if ss else 0: vv for ss, ii, vv in zip(s, i, v)}
        rep = np.array([lut[int(k)] for k in keys])
        xd = x.astype(np.float64)
        assert np.all(np.abs(rep - xd) <= alpha * np.abs(xd) * (1 + 1e-12))
        assert np.count_nonzero(rep == 0.0) == np.count_nonzero(x == 0)
        # counts equal a direct count of the elements per representative
        for j in rng.integers(0, v.size, 20):
            assert c[j] == np.count_nonzero(rep == v[j])
        # no more buckets than the log range allows (Sec. 4.3: a few thousand at alpha = 1 %)
        mag = np.abs(xd[xd != 0])
        per_sign = math.ceil(math.log(mag.max() / mag.min()) / math.log(sk.gamma_of(alpha))) + 1
        assert v.size <= 2 * per_sign + 1


def test_quantile_estimates_within_alpha():
    rng = np.random.default_rng(3)
    mag = np.abs(rng.standard_t(3, 100001) * 0.015).astype(np.float32)
    srt = np.sort(mag.astype(np.float64))
    for alpha in (0.01, 0.02):
        for q in (0.0, 0.05, 0.1, 0.4, 0.5, 0.9, 0.999, 0.9999, 1.0):
            exact = srt[int(math.floor(q * (mag.size - 1)))]
            est = sk.quantile_estimate(mag, q, alpha)
            assert abs(est - exact) <= alpha * exact * (1 + 1e-12)


def test_lloyd_against_scikit_learn():
    from sklearn.cluster import KMeans

    rng = np.random.default_rng(4)
    for trial in range(6):
        m, k = int(rng.integers(30, 400)), int(rng.integers(2, 17))
        xq = np.sort(rng.standard_normal(m) * rng.uniform(0.1, 3.0))
        w = rng.uniform(0.05, 1.0, m)
        init = np.sort(rng.choice(xq, k, replace=False))
        c, rounds = sk.weighted_lloyd(xq, w, init, 300)
        km = KMeans(n_clusters=k, init=init.reshape(-1, 1), n_init=1, max_iter=300, tol=0.0,
                    algorithm="lloyd").fit(xq.reshape(-1, 1), sample_weight=w)
        assert np.allclose(np.sort(km.cluster_centers_.ravel()), c, rtol=1e-9, atol=1e-12)
        # a fixed point: every centre is the weighted mean of the points nearest to it
        a = np.argmin(np.abs(xq[:, None] - c[None, :]), axis=1)
        for j in range(k):
            if np.any(a == j):
                assert math.isclose(c[j], np.average(xq[a == j], weights=w[a == j]), rel_tol=1e-12)


def test_kmeanspp_draws():
    rng = np.random.default_rng(5)
    xq = np.sort(rng.standard_normal(12))
    w = rng.uniform(0.1, 1.0, 12)
    # as many clusters as points: every point is drawn exactly once (a drawn point has distance 0)
    for _ in range(20):
        ch = sk.weighted_kmeanspp(xq, w, 12, rng.uniform(size=12))
        assert sorted(ch) == list(range(12))
    # fewer distinct points than clusters: the last centre is repeated
    ch = sk.weighted_kmeanspp([1.0, 2.0], [1.0, 1.0], 4, [0.1, 0.9, 0.5, 0.5])
    assert ch == [0, 1, 1, 1]
    # frequencies: first draw ~ W, second draw ~ D^2 W given the first
    draws = 40000
    u = rng.uniform(size=(draws, 2))
    first = np.zeros(12)
    second = np.zeros((12, 12))
    for r in range(draws):
        a, b = sk.weighted_kmeanspp(xq, w, 2, u[r])
        first[a] += 1
        second[a, b] += 1
    assert np.all(np.abs(first / draws - w / w.sum()) < 5 * np.sqrt(w / w.sum() / draws) + 1e-3)
    a = int(np.argmax(first))
    p = (xq - xq[a]) ** 2 * w
    p /= p.sum()
    assert np.all(np.abs(second[a] / first[a] - p) < 5 * np.sqrt(p / first[a]) + 2e-3)
    assert second[a, a] == 0


def _optimal_partition(x, k, power):
    """Brute force: best split of sorted x into k contiguous clusters (means for power 2, medians
    for power 1).  Returns (loss / n, labels)."""
    x = np.sort(np.asarray(x, np.float64))
    n = x.size
    best = (math.inf, None)
    for cuts in itertools.combinations(range(1, n), k - 1):
        edges = (0,) + cuts + (n,)
        loss = 0.0
        for a, b in zip(edges[:-1], edges[1:]):
            seg = x[a:b]
            mu = seg.mean() if power == 2 else np.median(seg)
            loss += float(np.sum(np.abs(seg - mu) ** power))
        if loss < best[0]:
            best = (loss, edges)
    labels = np.zeros(n, np.int64)
    for j, (a, b) in enumerate(zip(best[1][:-1], best[1][1:])):
        labels[a:b] = j
    return best[0] / n, labels


def test_separable_clusters_keep_their_memberships():
    # split > width and alpha < (split - width) / 4: the optimal memberships over the raw values and
    # over the sketch are identical, and Lloyd from any K-Means++ start that hits every cluster
    # finds them
    rng = np.random.default_rng(6)
    centres = np.array([0.05, 0.2, 0.45, 0.9])
    x = np.concatenate([c + rng.uniform(-0.01, 0.01, 5) for c in centres]).astype(np.float32)
    x = np.sort(x)
    _, labels = _optimal_partition(x, 4, 2)
    assert np.array_equal(labels, np.repeat(np.arange(4), 5))
    hits = 0
    for seed in range(20):
        r = sk.approximate_kmeans(x, 4, 0.01, 1.0, np.random.default_rng(seed).uniform(size=4), 100)
        if len({int(np.argmin(np.abs(centres - r["xq"][j]))) for j in r["init"]}) < 4:
            continue  # the start missed a cluster: Lloyd may stay in a local optimum
        hits += 1
        assert np.array_equal(sk.assign(x, r["centres"]), labels)
        for j in range(4):  # centres within alpha (relative) of the raw means
            assert abs(r["centres"][j] - x[labels == j].astype(np.float64).mean()) <= 0.01 * r["centres"][j]
    assert hits >= 10


def test_proposition_1_losses():
    rng = np.random.default_rng(7)
    alpha = 0.05
    x = np.sort(rng.uniform(0.001, 1.0, 9)).astype(np.float32)
    s, i, c = sk.sketch_histogram(x, alpha)
    idx = sk.bucket_index(x, alpha)
    xt = 2.0 * sk.gamma_of(alpha) ** idx.astype(np.float64) / (sk.gamma_of(alpha) + 1.0)
    assert np.all(np.abs(xt - x) <= alpha * x * (1 + 1e-12))
    for k in (1, 2, 3):
        l_opt, _ = _optimal_partition(x, k, 1)
        lq_opt, _ = _optimal_partition(xt, k, 1)
        assert abs(l_opt - lq_opt) <= alpha
        # any centres: the two losses differ by at most alpha
        m = np.sort(rng.uniform(0, 1, k))
        l = np.mean(np.min(np.abs(x.astype(np.float64)[:, None] - m[None, :]), axis=1))
        lq = np.mean(np.min(np.abs(xt[:, None] - m[None, :]), axis=1))
        assert abs(l - lq) <= alpha


def test_proposition_2_expectation():
    rng = np.random.default_rng(8)
    alpha, k = 0.05, 3
    x = np.sort(rng.uniform(0.001, 1.0, 10)).astype(np.float32)
    phi_opt, _ = _optimal_partition(x, k, 2)
    idx = sk.bucket_index(x, alpha)
    xt = 2.0 * sk.gamma_of(alpha) ** idx.astype(np.float64) / (sk.gamma_of(alpha) + 1.0)
    losses = []
    for seed in range(300):  # sigma = 1: the sample weights are the bucket frequencies
        r = sk.approximate_kmeans(x, k, alpha, 1.0, np.random.default_rng(100 + seed).uniform(size=k), 100)
        losses.append(np.mean(np.min((xt[:, None] - r["centres"][None, :]) ** 2, axis=1)))
    assert np.mean(losses) <= 16 * (math.log(k) + 2) * (phi_opt + alpha ** 2)
    assert np.min(losses) >= _optimal_partition(xt, k, 2)[0] * (1 - 1e-9)


def test_quantize_values_assigns_nearest_centre():
    rng = np.random.default_rng(9)
    x = (rng.standard_t(3, 20000) * 0.015).astype(np.float32)
    mag = np.abs(x)
    lo, hi = np.quantile(mag, 0.1), np.quantile(mag, 0.999)
    cls = np.where(mag < lo, 0, np.where(mag > hi, 1, 2))
    r = sk.quantize_values(x, cls, 16, 0.01, 0.2, rng.uniform(size=16), 100)
    cb = r["codebook"].astype(np.float64)
    assert np.all(np.diff(cb) >= 0)
    q = cls == 2
    d = np.abs(x[q].astype(np.float64)[:, None] - cb[None, :])
    chosen = r["sym"][q].astype(np.int64) - 2
    assert np.all(d[np.arange(d.shape[0]), chosen] <= d.min(axis=1) * (1 + 1e-12) + 1e-300)
    assert np.array_equal(r["sym"][~q], cls[~q].astype(np.uint16))
    # the fp32 boundaries reproduce the assignment
    assert np.array_equal(chosen, np.searchsorted(r["boundaries"], x[q], side="right"))
    # more weight on magnitude (small sigma) spreads the centres further out than frequency alone
    r_freq = sk.quantize_values(x, cls, 16, 0.01, 1.0, rng.uniform(size=16), 100)
    assert r["rounds"] >= 1 and r_freq["rounds"] >= 1


def test_bound_is_tight_and_buckets_per_decade():
    # gamma = (1 + alpha) / (1 - alpha): the worst relative error of a dense sample reaches alpha
    # (a finer or coarser sketch would not), and a decade holds ln 10 / ln gamma buckets
    x = np.exp(np.linspace(math.log(1e-3), math.log(1e3), 400001)).astype(np.float32)
    for alpha in (0.01, 0.05):
        s, i, c = sk.sketch_histogram(x, alpha)
        v = sk.bucket_value(s, i, alpha)
        idx = sk.bucket_index(x, alpha)
        rep = v[np.searchsorted(i, idx)]
        rel = np.abs(rep - x.astype(np.float64)) / x.astype(np.float64)
        assert 0.99 * alpha < rel.max() <= alpha * (1 + 1e-12)
        per_decade = math.log(10.0) / math.log((1 + alpha) / (1 - alpha))
        assert abs(v.size - 6 * per_decade) <= 2


def test_conventions_at_exact_ties():
    # random_choice: u * total equal to a running sum goes to the next index (running sum must exceed it)
    assert sk.weighted_kmeanspp([1.0, 2.0, 3.0], [1.0, 1.0, 2.0], 1, [0.25]) == [1]
    assert sk.weighted_kmeanspp([1.0, 2.0, 3.0], [1.0, 1.0, 2.0], 1, [0.2499999]) == [0]
    assert sk.weighted_kmeanspp([1.0, 2.0, 3.0], [1.0, 1.0, 2.0], 1, [0.5]) == [2]
    # a point on the midpoint stays with the lower centre; the boundary is the next fp32 number
    assert list(sk.assign([2.0, np.nextafter(2.0, 3.0)], [1.0, 3.0])) == [0, 1]
    assert sk.boundary_above(2.0) == np.nextafter(np.float32(2.0), np.float32(3.0))
    assert sk.boundary_above(2.0 + 1e-12) == np.nextafter(np.float32(2.0), np.float32(3.0))
    assert sk.boundary_above(2.0 - 1e-12) == np.float32(2.0)
    assert sk.boundary_above(0.0) == np.nextafter(np.float32(0), np.float32(1))
    assert sk.boundary_above(-1e-60) == np.float32(0.0)
    # a cluster without members keeps its centre
    c, rounds = sk.weighted_lloyd([1.0, 2.0, 3.0], [1.0, 1.0, 1.0], [1.5, 2.5, 100.0], 10)
    assert list(c) == [1.5, 3.0, 100.0]  # {1, 2} (2 is on the midpoint), {3}, {}
    # ... and so does one whose members have no weight
    c, _ = sk.weighted_lloyd([0.0, 1.0, 2.0], [0.0, 1.0, 1.0], [0.25, 1.5], 10)
    assert c[0] == 0.25


def test_search_over_bits():
    rng = np.random.default_rng(10)
    x = (rng.standard_t(3, 6000) * 0.015).astype(np.float32)
    mag = np.abs(x)
    lo, hi = np.quantile(mag, 0.2), np.quantile(mag, 0.999)
    cls = np.where(mag < lo, 0, np.where(mag > hi, 1, 2))
    uni = rng.uniform(size=256)
    # the start of a narrower width is a prefix of the start of a wider one
    s, i, c = sk.sketch_histogram(x[cls == 2], 0.01)
    xq = sk.bucket_value(s, i, 0.01)
    w = sk.sample_weights(xq, c, 0.2)
    assert sk.weighted_kmeanspp(xq, w, 8, uni) == sk.weighted_kmeanspp(xq, w, 64, uni)[:8]
    r = sk.search_bits(x, cls, 0.01, 0.2, uni, 100, 0.01)
    # the error of a width is the squared distance to the decoded tensor (protected values exact)
    for b in (2, 5, 8):
        run = r["runs"][b]
        dec = np.where(cls == 0, 0.0, np.where(cls == 1, x.astype(np.float64),
                                               run["codebook"].astype(np.float64)[np.maximum(run["sym"].astype(np.int64) - 2, 0)]))
        assert math.isclose(r["sse"][b], float(np.sum((x.astype(np.float64) - dec) ** 2)), rel_tol=1e-12)
    assert math.isclose(r["sumsq"], float(np.sum(x.astype(np.float64) ** 2)), rel_tol=1e-15)
    # the choice: the fewest bits within the bound; a bound below the pruned part is never met
    ok = [b for b in range(2, 9) if r["sse"][b] <= 0.01 * r["sumsq"]]
    assert r["feasible"] == bool(ok) and r["best_bits"] == (min(ok) if ok else 8)
    tight = sk.search_bits(x, cls, 0.01, 0.2, uni, 100, 1e-9)
    assert tight["feasible"] is False and tight["best_bits"] == 8
    loose = sk.search_bits(x, cls, 0.01, 0.2, uni, 100, 0.9)
    assert loose["feasible"] is True and loose["best_bits"] == 2
    # more bins never hurt much here: 8 bits are far better than 2
    assert r["sse"][8] < 0.05 * r["sse"][2]


def test_search_over_pairs_picks_the_least_payload_within_the_bound():
    """search_grid against a direct enumeration: quantize every (pair, width), decode, measure."""
    from oracle import ref
    rng = np.random.default_rng(61)
    x = (0.02 * rng.standard_t(3, 4000)).astype(np.float32)
    uni = rng.uniform(size=256)
    pairs = [(0, 0), (200000, 0), (200000, 5000), (500000, 5000)]
    classes = [np.minimum(ref.quantize(x, (8, p, o))["sym"], 2) for p, o in pairs]
    sumsq = float(np.sum(x.astype(np.float64) ** 2))
    for eps in (5e-2, 5e-3, 1e-12):
        got = sk.search_grid(x, classes, 0.01, 0.2, uni, 100, eps)
        cand = []
        for q, c in enumerate(classes):
            for b in range(2, 9):
                r = sk.quantize_values(x, c, 1 << b, 0.01, 0.2, uni, 100)
                dec = np.zeros(x.size)
                kept = c >= 2
                dec[kept] = r["codebook"].astype(np.float64)[r["sym"][kept].astype(np.int64) - 2]
                dec[c == 1] = x[c == 1]
                err = float(np.sum((x.astype(np.float64) - dec) ** 2))
                cand.append((err, int(kept.sum()) * b + 32 * int((c == 1).sum()) + 32 * (1 << b), q, b))
        ok = [(cost, q, b) for err, cost, q, b in cand if err <= eps * sumsq]
        if ok:
            assert got["feasible"] and (got["pair"], got["bits"]) == min(ok)[1:]
        else:
            assert not got["feasible"] and got["bits"] == 8
            assert got["pair"] == min((err, q) for err, cost, q, b in cand if b == 8)[1]
