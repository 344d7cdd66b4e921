"""The library's host entropy stage (inshr_entropy_encode / _decode through the C ABI; no GPU needed)
against the oracle: run-length tokens and the payload size of every group are unique and must match
exactly (the total cost of a Huffman code does not depend on tie-breaking); the codes themselves are
checked for validity: the container decodes back to the same stream, bit for bit."""
import struct

import numpy as np
import pytest

from oracle import entropy as ent
from oracle import ref


def api():
    from paper_2306_11800_amd import api as a
    return a


def parse_groups(data):
    """Group headers of the container: (n_values, n_tokens, payload_bits, [(token, length)])."""
    b = bytes(data)
    magic, n_groups, n, w, _ = struct.unpack_from("<IIQII", b, 0)
    assert magic == 0x31454449
    pos, out = 24, []
    for _ in range(n_groups):
        n_values, n_tokens, payload_bits, n_sym, _ = struct.unpack_from("<QQQII", b, pos)
        pos += 32
        table = [struct.unpack_from("<iI", b, pos + 8 * i) for i in range(n_sym)]
        pos += 8 * n_sym + (payload_bits + 7) // 8
        out.append((n_values, n_tokens, payload_bits, table))
    assert pos == len(b)
    return n, w, out


def make_stream(rng, n, n_groups, levels, p_zero):
    """A regrouped delta stream: group sizes random, values mostly zero with runs."""
    cuts = np.sort(rng.integers(0, n + 1, n_groups - 1))
    goff = np.concatenate([[0], cuts, [n]]).astype(np.uint64)
    v = rng.integers(0, levels, n).astype(np.uint16)
    v[rng.random(n) < p_zero] = 0
    runs = rng.random(n) < 0.3
    for i in np.nonzero(runs)[0]:
        if i:
            v[i] = v[i - 1]
    return v, goff


@pytest.mark.parametrize("seed,n,n_groups,levels,w,p_zero", [
    (1, 5000, 18, 18, 5, 0.6), (2, 20000, 258, 258, 9, 0.9), (3, 300, 4, 4, 2, 0.0),
    (4, 1, 1, 3, 2, 0.0), (5, 40000, 66, 66, 7, 0.99), (6, 1000, 258, 258, 9, 0.2)])
def test_against_oracle(seed, n, n_groups, levels, w, p_zero):
    rng = np.random.default_rng(seed)
    v, goff = make_stream(rng, n, n_groups, levels, p_zero)
    packed = ref.pack(v, w)
    data, stats = api().entropy_encode(goff, w, packed=packed)
    data2, stats2 = api().entropy_encode(goff, w, values=v)
    assert np.array_equal(data, data2) and stats == stats2
    nn, ww, groups = parse_groups(data)
    assert (nn, ww, len(groups)) == (n, w, n_groups)
    want = ent.group_costs(v, goff)
    tot_tokens = 0
    for g, ((n_values, n_tokens, payload_bits, table), (wt, wd, wb)) in enumerate(zip(groups, want)):
        lo, hi = int(goff[g]), int(goff[g + 1])
        assert n_values == hi - lo
        assert (n_tokens, len(table), payload_bits) == (wt, wd, wb), g
        toks = ent.rle_tokens(v[lo:hi])
        assert sorted(t for t, _ in table) == sorted(set(toks))
        if len(table) > 1:  # a complete prefix code
            assert sum(2.0 ** -l for _, l in table) == 1.0
        tot_tokens += n_tokens
    assert stats[0] == tot_tokens
    assert stats[1] + stats[2] + 24 == data.size
    # validity of the codes: the container decodes to the same stream
    back, goff2 = api().entropy_decode(data, n, w, n_groups)
    assert np.array_equal(back, packed) and np.array_equal(goff2, goff)
    vals, _ = api().entropy_decode(data, n, w, n_groups, as_values=True)
    assert np.array_equal(vals, v)


def test_one_group_is_the_stream_without_regrouping():
    rng = np.random.default_rng(7)
    v = np.zeros(100_000, np.uint16)
    idx = rng.integers(0, v.size, 500)
    v[idx] = rng.integers(1, 258, 500)
    goff = np.array([0, v.size], np.uint64)
    data, stats = api().entropy_encode(goff, 9, values=v)
    toks = ent.rle_tokens(v)
    assert stats[0] == len(toks)
    assert stats[2] == (ent.huffman_cost_bits(toks) + 7) // 8
    vals, _ = api().entropy_decode(data, v.size, 9, 1, as_values=True)
    assert np.array_equal(vals, v)


def test_constant_and_empty_groups():
    v = np.full(70_000, 3, np.uint16)
    goff = np.array([0, 0, 70_000, 70_000], np.uint64)
    data, stats = api().entropy_encode(goff, 4, values=v)
    _, _, groups = parse_groups(data)
    assert groups[0][:3] == (0, 0, 0) and groups[2][:3] == (0, 0, 0)
    assert groups[1][:3] == (70_000, 2, 2)  # tokens -3 and 70000, one bit each
    vals, goff2 = api().entropy_decode(data, v.size, 4, 3, as_values=True)
    assert np.array_equal(vals, v) and np.array_equal(goff2, goff)


def test_malformed_input_is_refused():
    a = api()
    v = np.arange(100, dtype=np.uint16) % 5
    goff = np.array([0, 50, 100], np.uint64)
    data, _ = a.entropy_encode(goff, 3, values=v)
    with pytest.raises(a.InshrError):
        a.entropy_decode(data[:-3], 100, 3, 2)
    with pytest.raises(a.InshrError):
        a.entropy_decode(data, 101, 3, 2)
    bad = data.copy()
    bad[0] ^= 1
    with pytest.raises(a.InshrError):
        a.entropy_decode(bad, 100, 3, 2)
    with pytest.raises(a.InshrError):
        a.entropy_encode(np.array([0, 60, 50, 100], np.uint64), 3, values=v)

