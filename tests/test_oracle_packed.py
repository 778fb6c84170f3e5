"""Pins of the oracle's packed-triangle functions (CPU only)."""
import os

import numpy as np

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_packed_sizes.txt")


def test_packed_sizes_stated_in_the_paper():
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        d, m = map(int, line.split())
        assert oracle.packed_size(d) == m


def test_pack_order_written_out():
    M = np.array([[1., 2., 3.], [20., 4., 5.], [30., 50., 6.]])      # lower triangle must be ignored
    assert oracle.pack_upper(M).tolist() == [1., 2., 3., 4., 5., 6.]
    U = oracle.unpack_upper(np.array([1., 2., 3., 4., 5., 6.]), 3)
    assert U.tolist() == [[1., 2., 3.], [2., 4., 5.], [3., 5., 6.]]


def test_pack_matches_library_indexing_and_round_trips():
    rng = np.random.default_rng(3)
    for d in (1, 2, 7, 33, 130):
        B = rng.standard_normal((d, d))
        S = B + B.T
        p = oracle.pack_upper(S)
        assert p.shape == (d * (d + 1) // 2,)
        assert np.array_equal(p, S[np.triu_indices(d)])              # numpy enumerates the upper triangle row by row too
        assert np.array_equal(oracle.unpack_upper(p, d), S)
        # offset of element (i, j), i <= j, in closed form
        i, j = rng.integers(0, d, 2)
        i, j = min(i, j), max(i, j)
        assert p[i * d - i * (i - 1) // 2 + (j - i)] == S[i, j]
