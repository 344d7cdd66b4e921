"""Oracle of the sketch-based boundary rule (TEST INFRASTRUCTURE ONLY): plain, slow numpy / Python.

Sec. 4.3 and Algorithm 1 (log-space quantile sketch without bucket merging), Sec. 4.4 and
Algorithm 2 (K-Means on the sketch's buckets with sample weights mixed from frequency and
magnitude), Algorithm 3 (weighted K-Means++ initialisation).  The values that are neither pruned
nor protected are clustered; the cluster centres become the codebook and every value takes the
nearest centre.

Readings where the paper is silent (all of them repeated in the design notes):
  * signed values: a bucket is (sign, ceil(log_gamma |x|)); exact zeros form one bucket of value 0;
  * the value of bucket i is 2 gamma^i / (gamma + 1), the point of (gamma^(i-1), gamma^i] whose
    relative distance to both ends is alpha (the estimate DDSketch returns);
  * Normalize divides by the largest absolute entry (both lists then lie in [0, 1]);
  * the distance of Algorithm 3 is the squared distance, as in K-Means++; random_choice(P) takes
    a uniform number u in [0, 1) and returns the first index whose running sum of P exceeds
    u * sum(P); the uniform numbers are inputs; when every remaining distance is zero (fewer
    distinct buckets than clusters) the last chosen centre is repeated;
  * WeightedKMeans runs Lloyd rounds from that start until the memberships repeat, at most
    max_iter rounds; a cluster without weight keeps its centre;
  * a point goes to the upper of two neighbouring centres when it lies strictly above their
    midpoint (midpoint = fl64((a + b) / 2)), otherwise to the lower one;
  * the codebook is the centres rounded to fp32; raw values are assigned with the same rule.

Only tests/ may import this module; it imports nothing from the HIP package.
"""
import functools
import math

import numpy as np


def gamma_of(alpha):
    """Algorithm 1, first step."""
    return (1.0 + alpha) / (1.0 - alpha)


@functools.lru_cache(maxsize=8)
def _bucket_tops(alpha):
    """(i_lo, tops): tops[j] = largest fp32 number <= gamma^(i_lo + j), exactly (integer
    arithmetic on gamma = p / q), for all buckets a positive fp32 number can fall into."""
    gamma = gamma_of(alpha)
    p, q = gamma.as_integer_ratio()

    def le_pow(c, pw, qw):
        """c <= pw / qw for a non-negative float c."""
        a, b = float(c).as_integer_ratio()
        return a * qw <= pw * b

    def floor32(i, pw, qw):
        c = np.float32(min(gamma ** i, fmax))
        while not le_pow(c, pw, qw):
            c = np.nextafter(c, np.float32(-np.inf), dtype=np.float32)
        while True:
            with np.errstate(over="ignore"):
                up = np.nextafter(c, np.float32(np.inf), dtype=np.float32)
            if not np.isfinite(up) or not le_pow(up, pw, qw):
                break
            c = up
        return c

    fmax = float(np.finfo(np.float32).max)
    tiny = float(np.nextafter(np.float32(0), np.float32(1)))  # smallest positive fp32
    up_list, pw, qw, i = [], 1, 1, 0
    while True:  # gamma^i for i = 0, 1, ... until it covers the largest fp32 number
        up_list.append(floor32(i, pw, qw))
        if le_pow(fmax, pw, qw):
            break
        pw, qw, i = pw * p, qw * q, i + 1
    dn_list, pw, qw, i = [], q, p, -1
    while True:  # gamma^i for i = -1, -2, ... until it drops below the smallest positive number
        c = floor32(i, pw, qw)
        dn_list.append(c)
        if not le_pow(tiny, pw, qw):
            break
        pw, qw, i = pw * q, qw * p, i - 1
    tops = np.array(dn_list[::-1] + up_list, dtype=np.float32)
    return -len(dn_list), tops


def bucket_index(absx, alpha):
    """ceil(log_gamma |x|) for positive fp32 numbers: the smallest i with |x| <= gamma^i."""
    absx = np.asarray(absx, dtype=np.float32)
    i_lo, tops = _bucket_tops(float(alpha))
    return i_lo + np.searchsorted(tops, absx, side="left").astype(np.int64)


def bucket_value(sign, index, alpha):
    gamma = gamma_of(alpha)
    return np.array([0.0 if s == 0 else s * (2.0 * gamma ** int(i) / (gamma + 1.0))
                     for s, i in zip(sign, index)], dtype=np.float64)


def sketch_histogram(x, alpha):
    """Algorithm 1 on signed values.  Returns (sign, index, count) sorted by bucket value."""
    x = np.asarray(x, dtype=np.float32).ravel()
    sign = np.sign(x).astype(np.int64)
    idx = np.zeros(x.size, np.int64)
    nz = sign != 0
    idx[nz] = bucket_index(np.abs(x[nz]), alpha)
    # one sortable key per bucket: negative values by descending index, zero, positive ascending
    order_key = sign * (idx + (1 << 20))
    keys, counts = np.unique(order_key, return_counts=True)
    s = np.sign(keys)
    i = np.abs(keys) - (1 << 20)
    i[s == 0] = 0
    return s, i, counts.astype(np.int64)


def quantile_estimate(x_abs, q, alpha):
    """Sec. 4.3: the sketch's estimate of the magnitude of rank floor(q (n - 1)) — the buckets are
    summed up until the one that holds the rank is found."""
    s, i, c = sketch_histogram(np.abs(np.asarray(x_abs, np.float32)), alpha)
    rank = int(math.floor(q * (int(c.sum()) - 1)))
    j = int(np.searchsorted(np.cumsum(c), rank, side="right"))
    return float(bucket_value(s[j:j + 1], i[j:j + 1], alpha)[0])


def sample_weights(xq, cq, sigma):
    """Algorithm 2, steps 2 and 3."""
    xq = np.asarray(xq, np.float64)
    cq = np.asarray(cq, np.float64)
    mx = np.max(np.abs(xq))
    x_hat = np.abs(xq) / mx if mx > 0.0 else np.zeros_like(xq)
    c_hat = cq / np.max(cq)
    return sigma * c_hat + (1.0 - sigma) * x_hat


def _choice(p, u):
    """First index whose running sum exceeds u * total (sums taken in index order)."""
    total = 0.0
    for v in p:
        total += float(v)
    target = u * total
    run = 0.0
    last = 0
    for j, v in enumerate(p):
        if v > 0.0:
            last = j
        run += float(v)
        if run > target:
            return j
    return last  # (rounding: u * total == total)


def weighted_kmeanspp(xq, w, k, uniforms):
    """Algorithm 3.  Returns the k chosen indices, in the order they were drawn."""
    xq = np.asarray(xq, np.float64)
    w = np.asarray(w, np.float64)
    chosen = [_choice(w, float(uniforms[0]))]
    d = (xq - xq[chosen[0]]) ** 2
    for r in range(1, k):
        p = d * w
        if not np.any(p > 0.0):
            chosen.append(chosen[-1])
            continue
        j = _choice(p, float(uniforms[r]))
        chosen.append(j)
        d = np.minimum(d, (xq - xq[j]) ** 2)
    return chosen


def midpoints(centres):
    c = np.asarray(centres, np.float64)
    return (c[:-1] + c[1:]) / 2.0


def assign(x, centres):
    """Index of the centre each x belongs to (centres ascending): the number of midpoints below x."""
    return np.searchsorted(midpoints(centres), np.asarray(x, np.float64), side="left")


def weighted_lloyd(xq, w, centres, max_iter):
    """Lloyd rounds with sample weights from sorted centres.  Returns (centres, rounds)."""
    xq = np.asarray(xq, np.float64)
    w = np.asarray(w, np.float64)
    c = np.array(sorted(float(v) for v in centres), dtype=np.float64)
    prev = None
    rounds = 0
    for _ in range(max_iter):
        a = assign(xq, c)
        if prev is not None and np.array_equal(a, prev):
            break
        new = c.copy()
        for j in range(c.size):
            sw, swx = 0.0, 0.0
            for i in np.nonzero(a == j)[0]:  # in index order
                sw += float(w[i])
                swx += float(w[i]) * float(xq[i])
            if sw > 0.0:
                new[j] = swx / sw
        c = new
        prev = a
        rounds += 1
    return c, rounds


def approximate_kmeans(x, k, alpha, sigma, uniforms, max_iter):
    """Algorithm 2.  Returns dict(centres fp64 ascending, rounds, n_buckets, xq, cq, w, init)."""
    s, i, cq = sketch_histogram(x, alpha)
    xq = bucket_value(s, i, alpha)
    w = sample_weights(xq, cq, sigma)
    init = weighted_kmeanspp(xq, w, k, uniforms)
    centres, rounds = weighted_lloyd(xq, w, xq[init], max_iter)
    return dict(centres=centres, rounds=rounds, n_buckets=int(xq.size), xq=xq, cq=cq, w=w, init=init)


def boundary_above(mid):
    """Smallest fp32 number strictly above the fp64 number mid."""
    c = np.float32(mid)
    if float(c) <= mid:
        c = np.nextafter(c, np.float32(np.inf), dtype=np.float32)
    else:
        while True:
            dn = np.nextafter(c, np.float32(-np.inf), dtype=np.float32)
            if float(dn) <= mid:
                break
            c = dn
    return c


def quantize_values(x, sym_class, k, alpha, sigma, uniforms, max_iter):
    """Symbols of a tensor whose classes are given (sym_class: 0 pruned, 1 protected, >= 2
    quantized, e.g. from the exact-threshold oracle): the quantized values are clustered and take
    2 + index of their centre.  Returns dict(sym, codebook fp32, boundaries fp32, rounds, n_buckets)."""
    x = np.asarray(x, np.float32).ravel()
    sym_class = np.asarray(sym_class)
    quantized = sym_class >= 2
    r = approximate_kmeans(x[quantized], k, alpha, sigma, uniforms, max_iter)
    codebook = r["centres"].astype(np.float32)
    sym = np.where(sym_class >= 2, 0, sym_class).astype(np.uint16)
    sym[quantized] = (2 + assign(x[quantized].astype(np.float64), codebook.astype(np.float64))).astype(np.uint16)
    bnd = np.array([boundary_above(m) for m in midpoints(codebook.astype(np.float64))], dtype=np.float32)
    return dict(sym=sym, codebook=codebook, boundaries=bnd, rounds=r["rounds"], n_buckets=r["n_buckets"],
                centres=r["centres"])


def search_bits(x, sym_class, alpha, sigma, uniforms, max_iter, eps, bits_range=(2, 3, 4, 5, 6, 7, 8)):
    """Sec. 5 restricted to the number of bins, with the bins of Algorithm 2: for every bit width b
    the quantized values are clustered into 2^b clusters (draw r of every width uses uniforms[r], so
    the start of a narrower width is a prefix of the start of a wider one), the squared error of the
    tensor is sum_pruned x^2 + sum_quantized (x - its centre)^2 (fp64, protected values are exact),
    and the fewest bits whose error is at most eps * sum x^2 are chosen; when no width qualifies, the
    widest (feasible = False).  Returns dict(best_bits, feasible, sse per width, sumsq, runs)."""
    x = np.asarray(x, np.float32).ravel()
    xd = x.astype(np.float64)
    sym_class = np.asarray(sym_class)
    sumsq = float(np.sum(xd * xd))
    pruned = float(np.sum(xd[sym_class == 0] ** 2))
    q = sym_class >= 2
    sse, runs = {}, {}
    for b in bits_range:
        r = quantize_values(x, sym_class, 1 << b, alpha, sigma, uniforms, max_iter)
        cb = r["codebook"].astype(np.float64)
        sse[b] = pruned + float(np.sum((xd[q] - cb[r["sym"][q].astype(np.int64) - 2]) ** 2))
        runs[b] = r
    best, feasible = max(bits_range), False
    for b in sorted(bits_range):
        if sse[b] <= eps * sumsq:
            best, feasible = b, True
            break
    return dict(best_bits=best, feasible=feasible, sse=sse, sumsq=sumsq, runs=runs)


def search_grid(x, classes_of_pair, alpha, sigma, uniforms, max_iter, eps):
    """Sec. 5 with the bins of Algorithm 2 over the whole space: for every (prune, protect) pair
    (classes_of_pair[q] = the symbol classes 0 / 1 / 2 of x under pair q) every bit width is scored
    as in search_bits; among all (pair, width) whose error is at most eps * sum x^2 the one with
    the least payload n_kept * bits + 32 * n_protected + 32 * 2^bits is chosen (ties: the lower pair,
    then the fewer bits); when none qualifies, the pair whose 8-bit error is least, with 8 bits and
    feasible = False.  Returns dict(pair, bits, feasible, per_pair=[search_bits results])."""
    per = [search_bits(x, c, alpha, sigma, uniforms, max_iter, eps) for c in classes_of_pair]
    best = None
    for q, (r, c) in enumerate(zip(per, classes_of_pair)):
        c = np.asarray(c)
        kept, prot = int(np.sum(c >= 2)), int(np.sum(c == 1))
        for b in sorted(r["sse"]):
            if r["sse"][b] <= eps * r["sumsq"]:
                cost = kept * b + 32 * prot + 32 * (1 << b)
                if best is None or cost < best[0]:
                    best = (cost, q, b)
    if best is not None:
        return dict(pair=best[1], bits=best[2], feasible=True, per_pair=per)
    q = min(range(len(per)), key=lambda i: (per[i]["sse"][8], i))
    return dict(pair=q, bits=8, feasible=False, per_pair=per)
