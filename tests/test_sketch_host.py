"""CPU tests of the host logic of the sketch quantizer (no GPU call is made)."""
import pytest


def test_sketch_bucket_tables_of_the_library_match_the_exact_ones():
    """Host logic of the sketch quantizer (no GPU): the library's bucket tops (80-bit powers rounded
    down to fp32) equal the oracle's, which come from integer arithmetic, entry by entry, and its
    bucket values equal the oracle's to the last bit."""
    import numpy as np
    from oracle import sketch_kmeans as sk
    from paper_2306_11800_amd import api
    for alpha in (0.01, 0.013, 0.02, 0.1, 0.5):
        i_lo, tops, values = api.sketch_buckets(alpha)
        o_lo, o_tops = sk._bucket_tops(alpha)
        # the library's table starts a few (empty) buckets lower and ends a few higher
        assert i_lo <= o_lo and i_lo + tops.size >= o_lo + o_tops.size
        a = o_lo - i_lo
        assert np.array_equal(tops[a:a + o_tops.size].view(np.uint32), o_tops.view(np.uint32))
        assert np.all(tops[:a] == 0) and np.all(tops[a + o_tops.size:] == np.finfo(np.float32).max)
        idx = np.arange(i_lo, i_lo + tops.size)
        want = sk.bucket_value(np.ones(idx.size, np.int64), idx, alpha)
        assert np.array_equal(values.view(np.uint64), want.view(np.uint64))
    for bad in (0.001, 0.6):
        with pytest.raises(api.InshrError):
            api.sketch_buckets(bad)
