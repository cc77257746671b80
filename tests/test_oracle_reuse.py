"""Pins for the oracle's draft-reuse rule (no GPU)."""
import os

import numpy as np
from hypothesis import given, settings, strategies as st

from oracle.reuse import ReusePool, reuse_segment

HERE = os.path.dirname(os.path.abspath(__file__))


def test_reuse_segment_hand_worked_cases():
    n = 0
    for line in open(os.path.join(HERE, "golden", "reuse_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        x, y, a, want = [[int(t) for t in f.split()] for f in line.split("|")]
        assert reuse_segment(x, y, a[0]) == tuple(want), line
        n += 1
    assert n == 10


def _runs(eq):
    """(start, length) of the maximal runs of True in a 0-based boolean array (library route:
    differences of the padded array)."""
    d = np.diff(np.concatenate([[0], eq.astype(np.int8), [0]]))
    return list(zip(np.flatnonzero(d == 1), np.flatnonzero(d == -1) - np.flatnonzero(d == 1)))


@settings(max_examples=300, deadline=None)
@given(st.integers(0, 32).flatmap(lambda n: st.tuples(
    st.lists(st.integers(0, 3), min_size=n, max_size=n),
    st.lists(st.integers(0, 3), min_size=n + 1, max_size=n + 1), st.integers(0, n))))
def test_reuse_segment_is_the_first_longest_run_after_the_rejection(case):
    x, y, a = case
    start, length = reuse_segment(x, y, a)
    n = len(x)
    if a == n:
        assert (start, length) == (0, 0)
        return
    eq = np.array([x[i] == y[i] for i in range(n)], dtype=bool)
    eq[:a + 1] = False  # positions up to and including e = a + 1 (0-based index a) do not count
    runs = _runs(eq)
    if not runs:
        assert (start, length) == (0, 0)
        return
    longest = max(r[1] for r in runs)
    first = min(r[0] for r in runs if r[1] == longest)
    assert (start, length) == (first + 1, longest)
    # the segment is all-equal, lies after e, and cannot be extended on either side
    assert start > a + 1 and all(x[i - 1] == y[i - 1] for i in range(start, start + length))
    assert start - 1 <= a + 1 or x[start - 2] != y[start - 2]
    assert start + length > n or x[start + length - 1] != y[start + length - 1]


def test_pool_keeps_the_longer_segment_ages_it_and_respects_the_cap():
    pool = ReusePool(max_age=2, cap=8)
    assert pool.extend([1, 2]) == [1, 2]
    pool.update([5, 6, 7, 8, 9], 3, 2)           # holds [7, 8], age 0
    assert pool.extend([1, 2]) == [1, 2, 7, 8]
    pool.update([1, 2, 7, 8], 4, 1)              # shorter find: [7, 8] stays, age 1
    assert pool.tokens == [7, 8] and pool.age == 1
    pool.update([1, 2, 3, 4, 5], 2, 3)           # longer find replaces it, new lifetime
    assert pool.tokens == [2, 3, 4] and pool.age == 0
    pool.update([0], 0, 0)                       # age 1
    pool.update([0], 0, 0)                       # age 2: still within the limit
    assert pool.extend([9]) == [9, 2, 3, 4]
    pool.update([0], 0, 0)                       # age 3 > 2: dropped
    assert pool.tokens == [] and pool.extend([9]) == [9]
    pool.update([1, 2, 3, 4, 5, 6], 2, 4)        # holds [2, 3, 4, 5]
    assert pool.extend([1, 1, 1, 1]) == [1, 1, 1, 1, 2, 3, 4, 5]   # exactly the cap
    assert pool.extend([1, 1, 1, 1, 1]) == [1, 1, 1, 1, 1]        # would exceed it: dropped, not cut
    assert pool.tokens == []
