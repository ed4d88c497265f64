"""Host-side model of the candidate lists of the fused top-k epilogue (csrc/fs_topk_common.hpp,
top_insert / top_merge_lists): the insertion rule a lane applies to each of its keys and the merge
network that joins two sorted lists.  The model restates the selects and compare-exchanges of the
device code; the tests check that they compute what the comments claim -- the M best in descending
order, the earlier (lower-id) entry ahead among equal keys, and the M largest words of two lists --
on random and exhaustive small inputs."""
import itertools

import numpy as np
import pytest


def top_insert(ka, ke, x, e):
    """In place, as the device code: every comparison is taken against the list before the insertion."""
    M = len(ka)
    c = [x > ka[s] for s in range(M)]
    for s in range(M - 1, 0, -1):
        ka[s], ke[s] = (ka[s - 1], ke[s - 1]) if c[s - 1] else ((x, e) if c[s] else (ka[s], ke[s]))
    if c[0]:
        ka[0], ke[0] = x, e


def top_merge_lists(w, o):
    """w descending, o ascending; returns the M largest of the union, descending."""
    M = len(w)
    w = [max(a, b) for a, b in zip(w, o)]
    d = M // 2
    while d > 0:
        for s in range(M):
            if (s & d) == 0:
                hi, lo = max(w[s], w[s + d]), min(w[s], w[s + d])
                w[s], w[s + d] = hi, lo
        d >>= 1
    return w


@pytest.mark.parametrize("M", [4, 8])
def test_insertion_keeps_the_best_m_and_the_earlier_entry_among_equal_keys(M):
    rng = np.random.default_rng(10 + M)
    for trial in range(300):
        n = int(rng.integers(1, 33))
        # few distinct values: many ties; 0 = an id that does not exist and must never enter
        keys = rng.integers(0, 6, n).tolist() if trial % 2 else rng.integers(0, 2**32, n).tolist()
        ka, ke = [0] * M, [0] * M
        for e, x in enumerate(keys):
            top_insert(ka, ke, x, e)
        want = sorted(((x, e) for e, x in enumerate(keys) if x > 0), key=lambda t: (-t[0], t[1]))[:M]
        got = [(a, e) for a, e in zip(ka, ke) if a > 0]
        assert got == want, (keys, ka, ke)
        assert all(a == 0 for a in ka[len(want):])


@pytest.mark.parametrize("M", [4, 8])
def test_merge_network_returns_the_m_largest_sorted(M):
    rng = np.random.default_rng(20 + M)
    pad = 7                                     # a word that may repeat (padding); every other word is distinct
    for trial in range(500):
        na, nb = int(rng.integers(0, M + 1)), int(rng.integers(0, M + 1))
        words = (rng.choice(10_000, na + nb, replace=False) + 100).tolist()
        a = sorted(words[:na], reverse=True) + [pad] * (M - na)
        b = sorted(words[na:], reverse=True) + [pad] * (M - nb)
        got = top_merge_lists(list(a), list(reversed(b)))
        assert got == sorted(a + b, reverse=True)[:M], (a, b, got)


def test_merge_network_on_every_interleaving_of_two_lists_of_four():
    # which of the 8 ranks go to the first list: all 70 choices
    for first in itertools.combinations(range(8), 4):
        a = sorted((100 - r for r in first), reverse=True)
        b = sorted((100 - r for r in range(8) if r not in first), reverse=True)
        assert top_merge_lists(list(a), list(reversed(b))) == [100, 99, 98, 97]
