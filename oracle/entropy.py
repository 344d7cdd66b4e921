"""Oracle of the delta entropy stage (TEST INFRASTRUCTURE ONLY): plain, slow Python.

Sec. 6, "Encoding Delta": every group of the regrouped delta stream is run-length encoded and the
result is Huffman coded.  A run of r equal delta values v becomes the token -v, followed by the
token +r when r > 1 (values are never positive, run lengths are at least 2, so the two kinds cannot
be confused).  Readings where the section is silent: the value token comes before its run length;
runs never cross a group; every group has a Huffman code of its own over its tokens.

Only tests/ may import this module; it imports nothing from the HIP package.
"""
import heapq
from collections import Counter


def rle_tokens(values):
    """Tokens of one group, in order."""
    out = []
    i, n = 0, len(values)
    while i < n:
        v = int(values[i])
        j = i + 1
        while j < n and int(values[j]) == v:
            j += 1
        out.append(-v)
        if j - i > 1:
            out.append(j - i)
        i = j
    return out


def rle_decode(tokens):
    out = []
    for t in tokens:
        if t <= 0:
            out.append(-t)
        else:
            out.extend([out[-1]] * (t - 1))
    return out


def huffman_lengths(freq):
    """Code length of every symbol of a Huffman code for the given counts (a dict).  One symbol
    alone gets length 0: a sequence over one symbol is fixed by its length."""
    if len(freq) <= 1:
        return {s: 0 for s in freq}
    heap = [(f, i, (s,)) for i, (s, f) in enumerate(sorted(freq.items()))]
    heapq.heapify(heap)
    depth = {s: 0 for s in freq}
    tie = len(heap)
    while len(heap) > 1:
        fa, _, sa = heapq.heappop(heap)
        fb, _, sb = heapq.heappop(heap)
        for s in sa + sb:
            depth[s] += 1
        heapq.heappush(heap, (fa + fb, tie, sa + sb))
        tie += 1
    return depth


def huffman_cost_bits(tokens):
    """Payload bits of an optimal prefix code for the token sequence (the same for every Huffman
    tree, whatever its tie-breaking)."""
    freq = Counter(tokens)
    lengths = huffman_lengths(freq)
    return sum(freq[s] * lengths[s] for s in freq)


def group_costs(stream, group_off):
    """Per group: (number of tokens, number of distinct tokens, payload bits)."""
    res = []
    for g in range(len(group_off) - 1):
        toks = rle_tokens(stream[int(group_off[g]):int(group_off[g + 1])])
        res.append((len(toks), len(set(toks)), huffman_cost_bits(toks)))
    return res
