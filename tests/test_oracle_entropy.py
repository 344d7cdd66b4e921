"""Pins of the entropy-stage oracle (oracle/entropy.py) against things other than itself: the worked
example the section's rule gives by hand, textbook Huffman costs, Kraft's equality, Shannon's bounds,
round trips."""
import math
from collections import Counter

import numpy as np

from oracle import entropy as ent


def test_rle_rule_by_hand():
    # 0 0 0 5 5 1 7 7 7 7 0 : value tokens are minus the value, run lengths only when above one
    assert ent.rle_tokens([0, 0, 0, 5, 5, 1, 7, 7, 7, 7, 0]) == [0, 3, -5, 2, -1, -7, 4, 0]
    assert ent.rle_tokens([]) == []
    assert ent.rle_tokens([9]) == [-9]
    assert ent.rle_tokens([2, 2]) == [-2, 2]  # a run length 2 next to a value 2: signs tell them apart


def test_rle_round_trip_and_token_kinds():
    rng = np.random.default_rng(1)
    for p_same in (0.0, 0.5, 0.95, 0.999):
        v = [0]
        for _ in range(3000):
            v.append(v[-1] if rng.random() < p_same else int(rng.integers(0, 258)))
        t = ent.rle_tokens(v)
        assert ent.rle_decode(t) == v
        assert all(x <= 0 or x >= 2 for x in t)
        # no two adjacent value tokens are equal unless a run length stands between them
        for a, b in zip(t, t[1:]):
            assert not (a <= 0 and b <= 0 and a == b)


def test_huffman_textbook_costs():
    # the classic six-letter example: counts 45 13 12 16 9 5 cost 224 bits
    f = {"a": 45, "b": 13, "c": 12, "d": 16, "e": 9, "f": 5}
    L = ent.huffman_lengths(f)
    assert sum(f[s] * L[s] for s in f) == 224
    assert L["a"] == 1 and L["f"] == 4 and L["e"] == 4
    # equal counts over a power of two: a fixed-length code
    f = {i: 7 for i in range(16)}
    assert set(ent.huffman_lengths(f).values()) == {4}
    # Fibonacci counts give the deepest tree: lengths 1, 2, ..., n-1, n-1
    fib = [1, 1, 2, 3, 5, 8, 13, 21]
    L = ent.huffman_lengths({i: c for i, c in enumerate(fib)})
    assert sorted(L.values()) == [1, 2, 3, 4, 5, 6, 7, 7]
    assert ent.huffman_lengths({5: 100}) == {5: 0}
    assert ent.huffman_lengths({}) == {}


def test_huffman_kraft_and_shannon():
    rng = np.random.default_rng(2)
    for trial in range(20):
        k = int(rng.integers(2, 300))
        counts = rng.integers(1, 10 ** int(rng.integers(1, 6)), k)
        f = {i: int(c) for i, c in enumerate(counts)}
        L = ent.huffman_lengths(f)
        assert sum(2.0 ** -l for l in L.values()) == 1.0  # a full binary tree
        n = sum(f.values())
        H = -sum(c / n * math.log2(c / n) for c in f.values())
        cost = sum(f[s] * L[s] for s in f)
        assert H * n - 1e-6 <= cost < (H + 1) * n
        # sum of the merged weights is the cost (the textbook identity), computed another way
        w = sorted(f.values())
        tot = 0
        while len(w) > 1:
            a, b = w[0], w[1]
            w = sorted(w[2:] + [a + b])
            tot += a + b
        assert tot == cost


def test_group_costs_example():
    stream = [0, 0, 0, 0, 1, 0, 0, 3, 3, 3]
    goff = [0, 7, 7, 10]
    # group 0: tokens 0 4 -1 0 2 -> counts {0: 2, 4: 1, -1: 1, 2: 1} -> lengths 2 2 2 ... cost 12;
    # by hand: merge 1+1=2, 1+2=3, 2+3=5: cost 2+3+5 = 10
    c = ent.group_costs(stream, goff)
    assert c[0] == (5, 4, 10)
    assert c[1] == (0, 0, 0)
    assert c[2] == (2, 2, 2)
    assert Counter(ent.rle_tokens(stream[:7])) == Counter({0: 2, 4: 1, -1: 1, 2: 1})
